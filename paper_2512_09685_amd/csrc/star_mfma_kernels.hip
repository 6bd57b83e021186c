// gfx950 kernel: the collapsed update with the Gram matrix of the gradient rows
// formed on the matrix cores.
//
// The per-group norms of a long update stream are quadratic forms in the Gram
// matrix Gamma_ab = sum_j g_a[j] g_b[j] (gradient-norm signal, Sections 4.3.1
// and 7 of the paper).  Gamma is a genuine dense contraction -- W x P times
// P x W -- and the only one on this path; everything else stays element-wise
// vector code.  On the vector ALUs Gamma costs W(W+1)/2 accumulator registers
// per thread, which caps the route at 16 rows and leaves one wave per SIMD;
// here it costs 4 (16-row tile) or 16 (32-row tile) accumulator registers per
// lane, so up to 32 rows fit in one pass.
//
// Data flow per wave and tile: the lanes hold, as in the other kernels, 4
// consecutive elements of every row (coalesced 16/8-byte loads) and apply the
// element-wise update from registers.  For the matrix cores the same values
// are needed "the other way round" (lane = row): they are staged through a
// wave-private LDS panel  T[row][element], 8 bytes per lane and row at a
// time, and read back 16 bytes at a time as  lane (i, t) <- T[i][part t].
#include "star_device.h"

#include <type_traits>

namespace star {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Matrix tiles.  "Row" is a gradient row (a worker), "slot" a group of lanes that feeds one part of
// the reduction dimension; lane l feeds row l % N and slot l / N.
//   fp32 rows, N=16: v_mfma_f32_16x16x4_f32,   1 element per lane, 4 slots
//   fp32 rows, N=32: three 16x16 blocks by v_mfma_f32_16x16x4_f32 with A and B from the two halves of
//                    the rows (see kBlocks in the kernel); the 32x32x2 instruction is not used
//   bf16 rows, N=16: v_mfma_f32_16x16x32_bf16, 8 elements per lane, 4 slots
//   bf16 rows, N=32: v_mfma_f32_32x32x16_bf16, 8 elements per lane, 2 slots
// (products of two bf16 values are exact in fp32, so the bf16 instructions lose nothing; they
// run at 8 to 16 times the fp32 rate).  Result register r of lane l is
//   N=16: D[4*(l/16) + r][l%16],     N=32: D[(r%4) + 4*(l/32) + 8*(r/4)][l%32].
// Operands A and B of  D += A * B  are the same register: whatever order the instruction gives
// the reduction dimension inside a lane, it is the same for A and for B, so D accumulates
// sum_e g_i[e] g_j[e] = Gamma_ij.
template <bool WIDE>
struct GramTile;
template <>
struct GramTile<false> {
    static constexpr int N = 16, SLOTS = 4, REGS = 4;
    typedef f32x4 acc_t;
    static __device__ __forceinline__ acc_t mma(float x, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(x, x, c, 0, 0, 0);
    }
    static __device__ __forceinline__ acc_t mma(bf16x8 x, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, x, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int lane_of(int i, int j) { return 16 * (i / 4) + j; }
    static __device__ __forceinline__ int reg_of(int i) { return i % 4; }
};
template <>
struct GramTile<true> {
    static constexpr int N = 32, SLOTS = 2, REGS = 16;
    typedef f32x16 acc_t;
    static __device__ __forceinline__ acc_t mma(float x, acc_t c) {   // not reached: fp32 rows go by blocks
        return __builtin_amdgcn_mfma_f32_32x32x2f32(x, x, c, 0, 0, 0);
    }
    static __device__ __forceinline__ acc_t mma(bf16x8 x, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, x, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int lane_of(int i, int j) { return 32 * ((i % 8) / 4) + j; }
    static __device__ __forceinline__ int reg_of(int i) { return 4 * (i / 8) + (i % 4); }
};

// One row of the LDS panel holds 512 bytes of elements (128 fp32 or 256 bf16) and 16 bytes of
// padding: 16 lanes that read 16 bytes each from 16 consecutive rows at the same offset then
// touch every bank exactly once.
constexpr int kPanelRowBytes = 512 + 16;

template <int W, class R, bool UPDATE, bool WIDE>
__global__ __launch_bounds__(kBlock, 2) void aff_mfma_kernel(float* __restrict__ params, float* __restrict__ momentum,
                                                          const RowPtrs rows, const AffCoef cf, const int64_t P,
                                                          const int vec_ok, const int span_g, const int span_k,
                                                          void* __restrict__ publish, const int publish_bf16,
                                                          double* __restrict__ partials,
                                                          TileQueue* __restrict__ queue, const int claim) {
    typedef GramTile<WIDE> GT;
    typedef typename GT::acc_t acc_t;
    typedef typename R::vec vec_t;
    constexpr bool BF = std::is_same<R, RowBf16x4>::value;
    constexpr int N = GT::N;
    static_assert(W <= N, "more rows than the matrix tile holds");
    constexpr int NG = W * (W + 1) / 2;
    constexpr int kWaves = kBlock / 64;
    constexpr int kPanelBytes = N * kPanelRowBytes;
    static_assert(kPanelBytes >= 64 * 16 * 8, "the panel doubles as the reduction buffer");
    __shared__ __align__(16) unsigned char panel[kWaves][kPanelBytes];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char* const T = panel[wave];
    // rows W..N-1 of the panel are zero and never written again
    for (int w = W; w < N; ++w) *reinterpret_cast<u32x2*>(T + w * kPanelRowBytes + 8 * lane) = u32x2{0u, 0u};

    // two accumulator sets used alternately, so that consecutive matrix instructions do not wait for
    // each other's result; acc2 is the second-level sum, in double (see fold)
    acc_t acc, accb;
    double acc2[GT::REGS];
#pragma unroll
    for (int r = 0; r < GT::REGS; ++r) {
        acc[r] = 0.0f;
        accb[r] = 0.0f;
        acc2[r] = 0.0;
    }
    const unsigned char* const my_row = T + (lane % N) * kPanelRowBytes + 16 * (lane / N);
    // 17-32 fp32 rows: the 32x32 matrix is formed from its three distinct 16x16 blocks (rows 0-15 with
    // themselves, rows 0-15 with rows 16-31, rows 16-31 with themselves) by the 16x16x4 instruction with
    // A and B from the two halves -- three quarters of the matrix work of the 32x32x2 instruction, which
    // computes the mirrored block too and is what bounds this variant.  blk[0..2] / blkb[0..2] are the
    // alternating accumulator sets of the three blocks, blk2 their sums in double.
    constexpr bool kBlocks = WIDE && !BF;
    f32x4 blk[3], blkb[3];
    double blk2[12];
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        blk[b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        blkb[b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
#pragma unroll
    for (int r = 0; r < 12; ++r) blk2[r] = 0.0;
    const unsigned char* const my_lo = T + (lane % 16) * kPanelRowBytes + 16 * (lane / 16);
    const unsigned char* const my_hi = my_lo + 16 * kPanelRowBytes;

    // stage: 512 bytes per row (8 per lane) into the panel; consume: feed them to the matrix cores.
    auto stage = [&](const u32x2 (&x)[W]) {
#pragma unroll
        for (int w = 0; w < W; ++w) *reinterpret_cast<u32x2*>(T + w * kPanelRowBytes + 8 * lane) = x[w];
    };
    auto consume = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the panel is written before any lane reads it
        if constexpr (kBlocks) {
#pragma unroll
            for (int m = 0; m < 512 / 64; ++m) {   // 4 slots of 16 bytes per row and step
                const f32x4 lo = *reinterpret_cast<const f32x4*>(my_lo + 64 * m);
                const f32x4 hi = *reinterpret_cast<const f32x4*>(my_hi + 64 * m);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4(&dst)[3] = (j & 1) ? blkb : blk;
                    dst[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(lo[j], lo[j], dst[0], 0, 0, 0);
                    dst[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(lo[j], hi[j], dst[1], 0, 0, 0);
                    dst[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(hi[j], hi[j], dst[2], 0, 0, 0);
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            return;
        }
        constexpr int kReads = 512 / (16 * GT::SLOTS);
#pragma unroll
        for (int m = 0; m < kReads; ++m) {
            const unsigned char* src = my_row + 16 * GT::SLOTS * m;
            if constexpr (BF) {
                const bf16x8 y = *reinterpret_cast<const bf16x8*>(src);
                if (m & 1) accb = GT::mma(y, accb);
                else acc = GT::mma(y, acc);
            } else {
                const f32x4 y = *reinterpret_cast<const f32x4*>(src);
                acc = GT::mma(y[0], acc);
                accb = GT::mma(y[1], accb);
                acc = GT::mma(y[2], acc);
                accb = GT::mma(y[3], accb);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // all reads returned before the panel is overwritten
    };
    auto gram_512 = [&](const u32x2 (&x)[W]) {
        stage(x);
        consume();
    };
    // The Gram contribution of one tile: 4 elements per lane and row.
    auto gram_tile = [&](const vec_t (&g)[W]) {
        if constexpr (BF) {
            gram_512(g);
        } else {
            u32x2 h[W];
#pragma unroll
            for (int w = 0; w < W; ++w) h[w] = u32x2{__float_as_uint(g[w][0]), __float_as_uint(g[w][1])};
            gram_512(h);
#pragma unroll
            for (int w = 0; w < W; ++w) h[w] = u32x2{__float_as_uint(g[w][2]), __float_as_uint(g[w][3])};
            gram_512(h);
        }
    };
    // After every tile the matrix-core accumulators (256 products each by then) are folded into a
    // second set kept in double.  Two reasons.  Long fp32 chains of products of short-mantissa (bf16)
    // values drift low, about 1e-9 per term, and a tile is the natural place to cut them.  And which
    // tiles a workgroup gets from the queue differs from run to run: a tile's own sums are formed in
    // a fixed order, and adding those in double makes the order of the tiles matter only at 1e-16,
    // far below the fp32 the norms are returned in, so that they come out the same every run.
    // The fold is 4 or 16 additions per lane.
    auto fold = [&]() {
        if constexpr (kBlocks) {
#pragma unroll
            for (int b = 0; b < 3; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    blk2[4 * b + r] += (double)(blk[b][r] + blkb[b][r]);
                    blk[b][r] = 0.0f;
                    blkb[b][r] = 0.0f;
                }
            return;
        }
#pragma unroll
        for (int r = 0; r < GT::REGS; ++r) {
            acc2[r] += (double)(acc[r] + accb[r]);
            acc[r] = 0.0f;
            accb[r] = 0.0f;
        }
    };

    // Tiles come from the queue and are walked with wave-uniform control flow (the matrix instructions
    // need every lane); a lane beyond the end of the shard contributes zeros.
    const int64_t first_tile = (int64_t)(blockIdx.x / span_g) * span_g * (int64_t)span_k + (blockIdx.x % span_g);
    const int64_t nchunk = vec_ok ? P / 4 : 0;
    const int64_t ntile = (nchunk + kBlock - 1) / kBlock;
    // element-wise update of chunk c from values already in registers
    auto update_chunk = [&](int64_t c, const vec_t (&g)[W], f32x4 pq, f32x4 vq) {
        f32x4 po, vo;
        static_for<0, 4>([&](auto kc) {
            constexpr int K = decltype(kc)::value;
            float ge[W];
            static_for<0, W>([&](auto wc) {
                constexpr int Wi = decltype(wc)::value;
                ge[Wi] = R::template get<K>(g[Wi]);
            });
            float pe = pq[K], ve = vq[K];
            aff_step<W>(pe, ve, ge, cf);
            po[K] = pe;
            vo[K] = ve;
        });
        store_state(po, params, c);
        store_state(vo, momentum, c);
        if (publish) publish_chunk(po, publish, publish_bf16, c);
    };
    auto fetch = [&](int64_t c, vec_t (&g)[W], f32x4& pq, f32x4& vq) {
        if (c < nchunk) {
#pragma unroll
            for (int w = 0; w < W; ++w) g[w] = R::load(rows.p[w], c);
            if constexpr (UPDATE) {
                pq = load_state(params, c);
                vq = load_state(momentum, c);
            }
        } else {
#pragma unroll
            for (int w = 0; w < W; ++w) g[w] = vec_t{};
        }
    };
    // The loads of the following tile are issued before this tile's update and Gram work where the Gram
    // phase is long enough to matter (not with 16 bf16 rows: 128 cycles a tile, and looking ahead measured
    // 2 % slower there) and the rows of two tiles fit in registers (up to 256 bytes per thread and tile).
    constexpr bool kAhead = sizeof(vec_t) * W <= 256 && (!BF || WIDE);
    if constexpr (kAhead) {
        vec_t gn[W];
        f32x4 pn = {0, 0, 0, 0}, vn = {0, 0, 0, 0};
        bool primed = false;
        for_each_claimed_tile_ahead(queue, ntile, claim, [&](const int64_t t, const int64_t following) {
            const int64_t c = t * kBlock + threadIdx.x;
            if (!primed) {
                fetch(c, gn, pn, vn);
                primed = true;
            }
            vec_t g[W];
#pragma unroll
            for (int w = 0; w < W; ++w) g[w] = gn[w];
            const f32x4 pq = pn, vq = vn;
            if (following >= 0) fetch(following * kBlock + threadIdx.x, gn, pn, vn);
            if constexpr (UPDATE) {
                if (c < nchunk) update_chunk(c, g, pq, vq);
            }
            gram_tile(g);
            fold();
        });
    } else {
        for_each_claimed_tile(queue, ntile, claim, [&](const int64_t t) {
            const int64_t c = t * kBlock + threadIdx.x;
            vec_t g[W];
            f32x4 pq = {0, 0, 0, 0}, vq = {0, 0, 0, 0};
            fetch(c, g, pq, vq);
            if constexpr (UPDATE) {
                if (c < nchunk) update_chunk(c, g, pq, vq);
            }
            gram_tile(g);
            fold();
        });
    }
    // elements not covered by whole chunks (the ragged end, or everything when some buffer is not
    // 16-byte aligned): one element per lane, same arithmetic
    const int64_t nrest = P - nchunk * 4;
    const int64_t nrtile = (nrest + kBlock - 1) / kBlock;
    int64_t tile = first_tile;
    for (int k = 0; k < span_k && tile < nrtile; ++k, tile += span_g) {
        const int64_t r = tile * kBlock + threadIdx.x;
        vec_t g[W];
#pragma unroll
        for (int w = 0; w < W; ++w) g[w] = vec_t{};
        if (r < nrest) {
            const int64_t j = nchunk * 4 + r;
            float g1[W];
#pragma unroll
            for (int w = 0; w < W; ++w) {
                g1[w] = R::load1(rows.p[w], j);
                if constexpr (BF) g[w][0] = __float_as_uint(g1[w]) >> 16;   // exact: the value came from a bf16
                else g[w][0] = g1[w];
            }
            if constexpr (UPDATE) {
                float pj = params[j], vj = momentum[j];
                aff_step<W>(pj, vj, g1, cf);
                params[j] = pj;
                momentum[j] = vj;
                if (publish) publish_element(pj, publish, publish_bf16, j);
            }
        }
        gram_tile(g);
        fold();
    }

    // workgroup total of every Gamma entry, in double, one partial per workgroup; each wave's
    // accumulators go through its own (now idle) panel
    double* const red = reinterpret_cast<double*>(T);
    if constexpr (kBlocks) {
#pragma unroll
        for (int b = 0; b < 3; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[lane * 12 + 4 * b + r] = (double)(blk[b][r] + blkb[b][r]) + blk2[4 * b + r];
    } else {
#pragma unroll
        for (int r = 0; r < GT::REGS; ++r) red[lane * GT::REGS + r] = (double)(acc[r] + accb[r]) + acc2[r];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < NG; e += kBlock) {
        int i = 0, rem = e;
        while (rem >= W - i) {
            rem -= W - i;
            ++i;
        }
        const int j = i + rem;
        int src;
        if constexpr (kBlocks) {
            // entry (i, j), i <= j, lies in block 0 (both below 16), 1 (i below, j from 16 on) or 2; inside a
            // block, D[a][b] is register a % 4 of lane 16 * (a / 4) + b
            const int b = (i >= 16) ? 2 : (j >= 16 ? 1 : 0);
            const int a = i & 15, c = j & 15;
            src = (16 * (a / 4) + c) * 12 + 4 * b + (a % 4);
        } else {
            src = GT::lane_of(i, j) * GT::REGS + GT::reg_of(i);
        }
        double s = 0.0;
#pragma unroll
        for (int q = 0; q < kWaves; ++q) s += reinterpret_cast<const double*>(panel[q])[src];
        partials[(int64_t)e * gridDim.x + blockIdx.x] = s;
    }
}

namespace {

template <int W, class R, bool UPDATE, bool WIDE>
hipError_t launch_mfma_t(const AffArgs& a, int num_cu, int grid_cap, int* grid_out, hipStream_t s) {
    auto kern = aff_mfma_kernel<W, R, UPDATE, WIDE>;
    // Long-lived workgroups, tiles from the queue.  Two per compute unit, so that one wave's Gram phase overlaps
    // another's loads; one where a single workgroup already keeps about 48 KB and more in flight, looks a
    // tile ahead and writes the state (10 to 16 fp32 rows: 2-5 % faster with one, e.g. 16 rows 1.51 against
    // 1.56 ms on the 110 M shard; 8 rows no difference; the norms alone, a pure read, run 1.13 against
    // 1.24 ms with two).  The LDS panels (33 KB narrow, 66 KB
    // wide per workgroup) allow both.
    constexpr int kRowBytes = W * (int)sizeof(typename R::vec);
    const int per_cu = (UPDATE && !WIDE && kRowBytes >= 160) ? 1 : 2;
    if (!a.queue) return hipErrorInvalidValue;
    const Geometry g = queue_geometry(num_cu, grid_cap, per_cu, kRowBytes + (UPDATE ? 32 : 0),
                                      UPDATE ? Traffic::Update : Traffic::ReadOnly,
                                      // (buffers that are not 16-byte aligned go through the one-element path,
                                      // which is spread over the whole grid: no tile count, no short-shard form)
                                      a.vec_ok ? (a.P / 4 + kBlock - 1) / kBlock : -1);
    *grid_out = g.grid;
    hipLaunchKernelGGL(kern, dim3(g.grid), dim3(kBlock), 0, s, a.params, a.momentum, a.rows, a.cf, a.P, a.vec_ok,
                       g.span_g, g.span_k, a.publish, a.publish_dtype == STAR_BF16 ? 1 : 0, a.partials, a.queue,
                       g.claim);
    return hipGetLastError();
}

template <int W>
hipError_t launch_mfma_w(int dtype, bool update, const AffArgs& a, int num_cu, int grid_cap, int* grid_out,
                         hipStream_t s) {
    constexpr bool WIDE = W > 16;
    if (dtype == STAR_F32) {
        if (update) return launch_mfma_t<W, RowF32, true, WIDE>(a, num_cu, grid_cap, grid_out, s);
        return launch_mfma_t<W, RowF32, false, WIDE>(a, num_cu, grid_cap, grid_out, s);
    }
    if (update) return launch_mfma_t<W, RowBf16x4, true, WIDE>(a, num_cu, grid_cap, grid_out, s);
    return launch_mfma_t<W, RowBf16x4, false, WIDE>(a, num_cu, grid_cap, grid_out, s);
}

}  // namespace

hipError_t launch_affine_mfma(int Wp, int dtype, bool update, const AffArgs& a, int num_cu, int grid_cap,
                              int* grid_out, hipStream_t s) {
    switch (Wp) {
#define X(N) case N: return launch_mfma_w<N>(dtype, update, a, num_cu, grid_cap, grid_out, s);
        STAR_FOR_EACH_W(X)
#undef X
        default: return hipErrorInvalidValue;
    }
}

}  // namespace star
