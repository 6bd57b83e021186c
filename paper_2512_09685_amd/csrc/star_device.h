// Device-side building blocks shared by the kernel files: row access, streaming
// stores, the wave64 sum, the workgroup-to-tile mapping and the launch geometry.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "star_kernels.h"

namespace star {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- row access
// A "row type" says how VEC consecutive gradient elements are fetched with one
// load and how element k is widened to fp32.
struct RowF32 {
    static constexpr int VEC = 4;
    typedef f32x4 vec;
    static __device__ __forceinline__ vec load(const void* row, int64_t chunk) {
        return __builtin_nontemporal_load(reinterpret_cast<const vec*>(row) + chunk);
    }
    template <int K>
    static __device__ __forceinline__ float get(const vec& x) { return x[K]; }
    static __device__ __forceinline__ float load1(const void* row, int64_t j) {
        return reinterpret_cast<const float*>(row)[j];
    }
};

// bf16 is the upper half of an fp32: widening is a shift (even element of a
// dword) or a mask (odd element); exact, infinities and NaNs carried over.
template <int K>
__device__ __forceinline__ float bf16_of(uint32_t dword) {
    return (K & 1) ? __uint_as_float(dword & 0xffff0000u) : __uint_as_float(dword << 16);
}

struct RowBf16x4 {
    static constexpr int VEC = 4;
    typedef u32x2 vec;
    static __device__ __forceinline__ vec load(const void* row, int64_t chunk) {
        return __builtin_nontemporal_load(reinterpret_cast<const vec*>(row) + chunk);
    }
    template <int K>
    static __device__ __forceinline__ float get(const vec& x) { return bf16_of<K>(x[K >> 1]); }
    static __device__ __forceinline__ float load1(const void* row, int64_t j) {
        return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(row)[j] << 16);
    }
};

// Streaming (non-temporal) 16-byte store.  The empty asm pins the value in
// vector registers at this point; without it the optimiser re-forms the store
// from the scalar results and the non-temporal hint is lost.
__device__ __forceinline__ void store_streaming(f32x4 x, f32x4* dst) {
    asm volatile("" : "+v"(x));
    __builtin_nontemporal_store(x, dst);
}

// Params / momentum access: streamed (non-temporal), worth ~6 % on the mixed read / read-modify-write
// traffic.  The hint does not keep a small shard from staying in the 256 MB Infinity Cache between
// calls: shards with params + momentum up to that size ran equally fast with and without it.
__device__ __forceinline__ f32x4 load_state(const float* base, int64_t idx4) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(base) + idx4);
}
__device__ __forceinline__ void store_state(f32x4 x, float* base, int64_t idx4) {
    store_streaming(x, reinterpret_cast<f32x4*>(base) + idx4);
}

// fp32 -> bf16, round to nearest even; NaN stays NaN (quiet bit forced).
__device__ __forceinline__ uint32_t bf16_bits_rne(float x) {
    uint32_t b = __float_as_uint(x);
    if ((b & 0x7fffffffu) > 0x7f800000u) return (b >> 16) | 0x40u;
    b += 0x7fffu + ((b >> 16) & 1u);
    return b >> 16;
}

// Streaming store of 4 consecutive values as fp32 or as bf16 (chunk index c).
__device__ __forceinline__ void publish_chunk(f32x4 x, void* dst, int as_bf16, int64_t c) {
    if (as_bf16) {
        u32x2 packed;
        packed[0] = bf16_bits_rne(x[0]) | (bf16_bits_rne(x[1]) << 16);
        packed[1] = bf16_bits_rne(x[2]) | (bf16_bits_rne(x[3]) << 16);
        asm volatile("" : "+v"(packed));
        __builtin_nontemporal_store(packed, reinterpret_cast<u32x2*>(dst) + c);
    } else {
        store_streaming(x, reinterpret_cast<f32x4*>(dst) + c);
    }
}

__device__ __forceinline__ void publish_element(float x, void* dst, int as_bf16, int64_t j) {
    if (as_bf16)
        reinterpret_cast<uint16_t*>(dst)[j] = (uint16_t)bf16_bits_rne(x);
    else
        reinterpret_cast<float*>(dst)[j] = x;
}

// ---------------------------------------------------------------- wave64 sum
// Sum over the 64 lanes with data-parallel-primitive moves; the total lands in
// lane 63.  Stages: swap within pairs, within quads, mirror within 8, mirror
// within 16 (every lane of a 16-lane row now holds the row's sum), then lane 15
// of rows 0 and 2 is added into rows 1 and 3, and lane 31 into rows 2 and 3.
// The order of additions is fixed, so the result is reproducible.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_take(float x) {
    // lanes outside ROW_MASK, or whose source lane is invalid, read 0
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false));
}

__device__ __forceinline__ float wave_sum_to_lane63(float x) {
    x += dpp_take<0xB1, 0xf>(x);   // quad_perm [1,0,3,2]
    x += dpp_take<0x4E, 0xf>(x);   // quad_perm [2,3,0,1]
    x += dpp_take<0x141, 0xf>(x);  // row_half_mirror
    x += dpp_take<0x140, 0xf>(x);  // row_mirror
    x += dpp_take<0x142, 0xa>(x);  // row_bcast:15 into rows 1, 3
    x += dpp_take<0x143, 0xc>(x);  // row_bcast:31 into rows 2, 3
    return x;
}

// The same in double (each move is done on the two halves of the value).  The norm sums take this
// one: which tiles a workgroup gets from the queue differs from run to run, and only sums that are
// carried in double from the per-tile level on come out the same in fp32 every time.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_take(double x) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, ROW_MASK, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, ROW_MASK, 0xf, false);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

__device__ __forceinline__ double wave_sum_to_lane63(double x) {
    x += dpp_take<0xB1, 0xf>(x);
    x += dpp_take<0x4E, 0xf>(x);
    x += dpp_take<0x141, 0xf>(x);
    x += dpp_take<0x140, 0xf>(x);
    x += dpp_take<0x142, 0xa>(x);
    x += dpp_take<0x143, 0xc>(x);
    return x;
}

// ---------------------------------------------------------------- compile-time loops
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// ---------------------------------------------------------------- workgroup -> tile mapping
// Workgroup b handles items first, first+step, ... (at most K of them, below n).
struct Span {
    int64_t first, step;
    int32_t K;
};
__device__ __forceinline__ Span make_span(const int span_g, const int span_k, const int threads = kBlock) {
    const int64_t G = span_g;
    Span s;
    s.first = ((int64_t)(blockIdx.x / span_g) * G * span_k + (blockIdx.x % span_g)) * threads + threadIdx.x;
    s.step = G * threads;
    s.K = span_k;
    return s;
}

// Dynamic order: the workgroups of a launch take tiles 0, 1, 2, ... from a queue, `claim` consecutive
// tiles at a time, and call body(tile) for each (the whole workgroup together; body may synchronise).
// Compared with a fixed assignment this keeps the tiles in flight a dense, slowly advancing window
// even though compute units progress at different rates, and it balances the end of the kernel.
// The next claim is requested before the current one is worked on, so the atomic's latency (several
// microseconds when 256 workgroups share one counter) is hidden.  Every workgroup leaves after its
// first claim beyond the last tile and requests nothing after that, so the loop ends for any queue
// state; the last one to leave puts the queue back to zero.
// The first claim of a workgroup is known without asking the counter: workgroup b gets 1 + b % claim
// tiles, laid out one after the other; the counter hands out the tiles after those (`base` on).  The
// unequal first claims are deliberate.  With equal ones all workgroups start, finish and re-claim at
// the same moments, every wave of the chip then walks the rows in step, and that pattern, once set,
// persists through the kernel: the 32-row bf16 aggregation ran 70 % slower that way (2.77 against
// 1.63 ms).  A spread of up to two tile times at the start is enough to keep the requests mixed.
__device__ __forceinline__ FirstClaim first_claim(const int claim, const int64_t ntile) {
    return first_claim_of((int64_t)blockIdx.x, (int64_t)gridDim.x, claim, ntile);
}

template <class Body>
__device__ __forceinline__ void for_each_claimed_tile(TileQueue* __restrict__ q, const int64_t ntile, const int claim,
                                                      Body&& body) {
    __shared__ unsigned long long s_first;
    const FirstClaim fc = first_claim(claim, ntile);
    const int step = claim < 0 ? -claim : claim;
    // When the first claims already cover the shard nobody asks the counter, and nobody has to put it
    // back: the same for every workgroup of the launch (base and ntile are).
    const bool counter = fc.base < (unsigned long long)ntile;
    unsigned long long nxt = 0;
    int64_t t0 = fc.t0;
    int n = fc.n;
    while (t0 < ntile) {
        if (counter && threadIdx.x == 0) nxt = fc.base + atomicAdd(&q->next, (unsigned long long)step);
        const int64_t t1 = t0 + n < ntile ? t0 + n : ntile;
        n = step;
        for (int64_t t = t0; t < t1; ++t) body(t);
        if (!counter) break;
        if (threadIdx.x == 0) s_first = nxt;
        __syncthreads();
        t0 = (int64_t)s_first;
        __syncthreads();   // everyone has read s_first before thread 0 writes it again
    }
    if (counter && threadIdx.x == 0) {
        // this workgroup's claims have all returned (their values were used above), so when the
        // count reaches the grid size nobody touches `next` any more
        const unsigned int left = atomicAdd(&q->done, 1u);
        if (left + 1 == gridDim.x) {
            atomicExch(&q->next, 0ull);
            atomicExch(&q->done, 0u);
        }
    }
}

// The same order with one tile of look-ahead, for kernels that issue the loads of the following tile
// before they work on the current one: body(tile, following) with following < 0 at the end.  The
// start of the next claim is made known to the whole workgroup when it begins the last tile of the
// current claim, so the look-ahead also crosses claims.
template <class Body>
__device__ __forceinline__ void for_each_claimed_tile_ahead(TileQueue* __restrict__ q, const int64_t ntile,
                                                            const int claim, Body&& body) {
    __shared__ unsigned long long s_first;
    const FirstClaim fc = first_claim(claim, ntile);
    const int step = claim < 0 ? -claim : claim;
    const unsigned long long base = fc.base;
    const bool counter = base < (unsigned long long)ntile;   // see for_each_claimed_tile
    unsigned long long nxt = 0;
    int64_t cur = fc.t0;
    if (cur < ntile && fc.n > 0) {   // (an even split of fewer tiles than workgroups leaves some without)
        if (counter && threadIdx.x == 0) nxt = base + atomicAdd(&q->next, (unsigned long long)step);
        int64_t end = cur + fc.n < ntile ? cur + fc.n : ntile;
        for (;;) {
            int64_t following = cur + 1;
            if (following >= end) {   // last tile of this claim: where does the next one start?
                if (!counter) {
                    following = -1;
                } else {
                    if (threadIdx.x == 0) s_first = nxt;
                    __syncthreads();
                    following = (int64_t)s_first;
                    __syncthreads();
                    if (following < ntile) {
                        // no claim is requested once the end is known: nothing may touch the queue
                        // after this workgroup has reported that it left
                        if (threadIdx.x == 0) nxt = base + atomicAdd(&q->next, (unsigned long long)step);
                        end = following + step < ntile ? following + step : ntile;
                    } else {
                        following = -1;
                    }
                }
            }
            body(cur, following);
            if (following < 0) break;
            cur = following;
        }
    }
    if (counter && threadIdx.x == 0) {
        const unsigned int left = atomicAdd(&q->done, 1u);
        if (left + 1 == gridDim.x) {
            atomicExch(&q->next, 0ull);
            atomicExch(&q->done, 0u);
        }
    }
}

// ---------------------------------------------------------------- the collapsed update of one element
constexpr int kGramFold = 64;  // tiles between folds of the pairwise-product accumulators (power of two)

template <int W>
__device__ __forceinline__ void aff_step(float& p, float& v, const float (&g)[W], const AffCoef& cf) {
    // increment of p first, one final add: p is perturbed by one rounding of p itself
    float inc = cf.dp * p;
    inc = __builtin_fmaf(cf.m01, v, inc);
    float nv = cf.m10 * p;
    nv = __builtin_fmaf(cf.m11, v, nv);
#pragma unroll
    for (int w = 0; w < W; ++w) {  // ascending worker id
        inc = __builtin_fmaf(cf.b0[w], g[w], inc);
        nv = __builtin_fmaf(cf.b1[w], g[w], nv);
    }
    p = p + inc;
    v = nv;
}

// ================================================================= host side of a launch
// Launch geometry: G workgroups per span, K tiles per workgroup, and the grid.
struct Geometry {
    int grid, span_g, span_k;
    int claim;   // > 0: tiles come from the queue, this many per claim; span_g / span_k then serve the ragged end only
    int threads; // workgroup size (kBlock unless a launcher says otherwise)
};

// Fixed assignment of tiles (short shards, launches without a queue).  items = chunks (or single
// elements when the buffers are not 16-byte aligned).  A kernel that ends with a per-workgroup norm
// reduction runs long-lived workgroups that sweep the shard as a single span; the others get one
// tile per workgroup, dispatched in address order.
// `thread_bytes`: bytes one thread has in flight per tile; long-lived workgroups are stacked on a compute unit
// (up to `max_per_cu`) until about 64 KB per unit are in flight, which light bf16 kernels need and heavy fp32
// ones already have with one workgroup; `min_per_cu` is for kernels that need a second workgroup per unit for
// their arithmetic rather than for their memory traffic.
inline Geometry pick_geometry(int64_t P, int vec, bool vec_ok, bool reduces, int num_cu, int grid_cap,
                              int thread_bytes = 256, int max_per_cu = 1, int min_per_cu = 1) {
    const int64_t items = vec_ok ? std::max<int64_t>(P / vec, P % vec) : P;
    const int64_t tiles = std::max<int64_t>(1, (items + kBlock - 1) / kBlock);
    Geometry g;
    g.claim = 0;
    g.threads = kBlock;
    if (reduces) {
        const int wg_bytes = std::max(1, thread_bytes) * kBlock;
        const int bpc = std::max(min_per_cu, std::min(max_per_cu, (64 * 1024 + wg_bytes - 1) / wg_bytes));
        g.span_g = (int)std::min<int64_t>(std::min(num_cu * bpc, grid_cap), tiles);
        g.span_k = 0x7fffffff;
        g.grid = g.span_g;
    } else {
        const int64_t max_grid = 0x7fffffff;
        g.span_g = 1;
        g.span_k = (int)((tiles + max_grid - 1) / max_grid);   // 1 unless the shard is absurdly long
        g.grid = (int)((tiles + g.span_k - 1) / g.span_k);
    }
    return g;
}

// Geometry of a launch that takes its tiles from a queue: `per_cu` long-lived workgroups per compute unit.
// Measured on MI355X, fewer waves in flight are faster as long as they keep enough bytes in flight: kernels
// that read-modify-write the state want one workgroup per unit from about 128 bytes per thread and tile
// (1 > 2 > 3 > 4 by 2-4 % each step), lighter ones and the read-mostly aggregation want two.
inline int queue_workgroups_per_cu(int thread_bytes, bool writes_state) {
    return writes_state && thread_bytes >= 128 ? 1 : 2;
}
// `tiles`: whole tiles of the shard if the launcher knows them (an estimate will do: the kernel splits
// its own count).  Up to short_tiles_per_workgroup() tiles per workgroup the launch takes the short-shard
// form of the first claims (first_claim_of) and no more workgroups than tiles.  Where the queue's order
// starts to pay, measured on the matrix-core kernel (the one that is in queue order at every length):
//   update with norms   8 tiles per workgroup (16 fp32 rows, 1 Mi elements: 27 against 34 us; 16 tiles: equal
//                       with one workgroup per unit, 2-7 % behind with two; 32 tiles: 10 % behind);
//                       16 tiles when a thread moves less than 160 bytes per tile (4 to 12 bf16 rows,
//                       6 and 8 Mi elements: 5-16 % ahead of 8)
//   norms / Gram alone  a pure read: 48 tiles (12 to 24 Mi elements: 2-10 % ahead of the queue, 32 Mi
//                       and more: 1-3 % behind with 16 to 32 rows); 128 tiles up to 128 bytes per thread and
//                       tile (8 bf16 rows, 16 to 64 Mi elements: 7-15 % ahead)
inline int short_tiles_per_workgroup(int thread_bytes, Traffic traffic) {
    if (traffic == Traffic::ReadOnly) return thread_bytes <= 128 ? 128 : 48;
    return thread_bytes < 160 ? 16 : 8;
}
inline Geometry queue_geometry(int num_cu, int grid_cap, int per_cu, int thread_bytes,
                               Traffic traffic = Traffic::Update, int64_t tiles = -1) {
    Geometry g;
    g.threads = kBlock;
    g.grid = g.span_g = std::max(1, std::min(num_cu * per_cu, grid_cap));
    g.span_k = 0x7fffffff;
    g.claim = queue_claim(thread_bytes, traffic);
    if (tiles >= 0 && tiles <= (int64_t)g.grid * short_tiles_per_workgroup(thread_bytes, traffic)) {
        g.claim = -1;
        g.grid = g.span_g = (int)std::max<int64_t>(1, std::min<int64_t>(g.grid, tiles));
    }
    return g;
}

#define STAR_FOR_EACH_W(X)                                                                                    \
    X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(20) X(24) X(28) \
    X(32)

}  // namespace star
