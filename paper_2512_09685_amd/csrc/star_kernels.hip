// gfx950 kernels for the group-synchronous parameter update.
//
// Layout: every buffer is a flat array of P elements, cut into "chunks" of VEC
// consecutive elements.  A wave works on 64 consecutive chunks, so it reads 64
// consecutive 16-byte pieces of each row: whole cache lines, every byte used
// once.  Workgroups are mapped to chunks in "spans": G consecutive workgroups
// sweep one contiguous span of G*K tiles together (tile = 256 chunks), each
// taking every G-th tile, so that at any moment the running workgroups touch a
// narrow, advancing window of every row (DRAM pages stay open) while each
// workgroup still lives for K tiles (one norm reduction per K tiles).  Each
// gradient row, params and momentum are read once per call; params and
// momentum are written once.  All state of an element lives in registers
// between the load and the store.
//
// Two evaluations of the U updates of a call (Section 1 items (2), (4);
// Section 4.2 of the paper define the updates):
//   seq_kernel  walks the updates one by one with the W gradients of the
//               element held in registers; group tables sit in LDS.
//   aff_kernel  applies the U updates as one affine map of (p, v, g_0..g_W-1)
//               whose coefficients the host composed in double precision.
// Per-group norms: seq_kernel accumulates gbar_u^2 per thread (LDS slots),
// aff_kernel accumulates the pairwise products of the rows (Gram matrix);
// both end with a wave64 DPP reduction and write one partial per block.
#include <hip/hip_runtime.h>

#include "star_device.h"

namespace star {

// ================================================================= affine kernel
template <int W>
__device__ __forceinline__ void gram_step(float (&acc)[W * (W + 1) / 2], const float (&g)[W]) {
    int e = 0;
#pragma unroll
    for (int a = 0; a < W; ++a)
#pragma unroll
        for (int b = a; b < W; ++b) {
            acc[e] = __builtin_fmaf(g[a], g[b], acc[e]);
            ++e;
        }
}

// KCH: chunks a thread loads together per tile when the tiles come from the queue (a tile is then
// KCH * 256 chunks).  More than one only for the Gram matrix alone on very few rows: a thread that loads 8
// to 32 bytes per tile keeps too little in flight (1 fp32 row: 0.40 of the HBM peak), whatever the claim.
// ONE_WAVE: the launch runs one wave per SIMD (the half-size workgroups of the update on 24 and more bf16 rows:
// two of 128 threads per compute unit).  Telling the compiler so lets it spend registers on issuing a tile's 34
// loads together instead of saving them for an occupancy the launch never uses: 32 bf16 rows, 138 M elements,
// 1.84 against 1.89-1.91 ms.  The limit is enforced by the hardware too, so only launches that take their tiles
// from the queue use these instantiations (a short shard with one tile per workgroup needs many workgroups per
// unit: 0.52 against 0.71 of the HBM peak on 12 M elements), and 8 or 16 rows, which run one wave per SIMD as
// well, measured 1-2 % slower with it.
template <int W, class R, bool UPDATE, bool GRAM, int KCH = 1, bool ONE_WAVE = false>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(1, ONE_WAVE ? 1 : 8)))
void aff_kernel(float* __restrict__ params, float* __restrict__ momentum,
                                                     const RowPtrs rows, const AffCoef cf, const int64_t P,
                                                     const int vec_ok, const int span_g, const int span_k,
                                                     void* __restrict__ publish, const int publish_bf16,
                                                     double* __restrict__ partials, TileQueue* __restrict__ queue,
                                                     const int claim) {
    constexpr int VEC = R::VEC;
    constexpr int NG = W * (W + 1) / 2;
    float acc[GRAM ? NG : 1];
#pragma unroll
    for (int e = 0; e < (GRAM ? NG : 1); ++e) acc[e] = 0.0f;
    // Second-level sums, one private LDS slot per thread and pair.  The register
    // accumulators are folded into them every kGramFold tiles, so no fp32 chain
    // of products is longer than 4*kGramFold terms: long chains of squares of
    // short-mantissa (bf16) values round down systematically, about 1e-9 per
    // term, because the low bits of a square are not uniformly distributed.
    // With few rows (up to kFewRows) there are few pairs: the slots are double and take the sums after
    // every chunk, which makes them independent of the order of the tiles (to 1e-16), so that this
    // variant can take its tiles from the queue like the plain one; and it has the registers for it.
    constexpr bool kFew = GRAM && gram_few_rows_form(W, std::is_same<R, RowF32>::value, UPDATE);
    typedef typename std::conditional<kFew, double, float>::type fold_t;
    __shared__ fold_t fold[GRAM ? NG * kBlock : 1];
    if constexpr (GRAM) {
#pragma unroll
        for (int e = 0; e < NG; ++e) fold[e * kBlock + threadIdx.x] = (fold_t)0;
    }
    auto fold_now = [&]() {
        if constexpr (GRAM) {
#pragma unroll
            for (int e = 0; e < NG; ++e) {
                fold[e * kBlock + threadIdx.x] += (fold_t)acc[e];
                acc[e] = 0.0f;
            }
        }
    };

    // the Gram variants are always launched with kBlock threads (their LDS slots are laid out for that);
    // the plain one also runs with half-size workgroups
    const int threads = GRAM ? kBlock : (int)blockDim.x;
    const Span span = make_span(span_g, span_k, threads);
    const int64_t nchunk = vec_ok ? P / VEC : 0;

    // one chunk: VEC elements of every row, the update, the pairwise products
    auto process = [&](const int64_t c) {
        typename R::vec g[W];
#pragma unroll
        for (int w = 0; w < W; ++w) g[w] = R::load(rows.p[w], c);
        float pe[VEC], ve[VEC];
        if constexpr (UPDATE) {
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                const f32x4 pq = load_state(params, c * (VEC / 4) + q);
                const f32x4 vq = load_state(momentum, c * (VEC / 4) + q);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    pe[4 * q + k] = pq[k];
                    ve[4 * q + k] = vq[k];
                }
            }
        }
        static_for<0, VEC>([&](auto kc) {
            constexpr int K = decltype(kc)::value;
            float ge[W];
            static_for<0, W>([&](auto wc) {
                constexpr int Wi = decltype(wc)::value;
                ge[Wi] = R::template get<K>(g[Wi]);
            });
            if constexpr (UPDATE) aff_step<W>(pe[K], ve[K], ge, cf);
            if constexpr (GRAM) gram_step<W>(acc, ge);
        });
        if constexpr (UPDATE) {
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                f32x4 pq = {pe[4 * q], pe[4 * q + 1], pe[4 * q + 2], pe[4 * q + 3]};
                f32x4 vq = {ve[4 * q], ve[4 * q + 1], ve[4 * q + 2], ve[4 * q + 3]};
                store_state(pq, params, c * (VEC / 4) + q);
                store_state(vq, momentum, c * (VEC / 4) + q);
                if (publish) publish_chunk(pq, publish, publish_bf16, c * (VEC / 4) + q);
            }
        }
    };
    bool queued = false;
    if constexpr (!GRAM || kFew) {
        // without the register-heavy Gram accumulators the kernel affords a second copy of the chunk
        // code: tiles from the queue for long shards, a fixed assignment for short ones
        if (claim > 0) {
            queued = true;
            if constexpr (KCH > 1) {
                static_assert(GRAM && !UPDATE, "several chunks per thread: Gram matrix alone");
                const int64_t width = (int64_t)threads * KCH;
                const int64_t ntile = (nchunk + width - 1) / width;
                for_each_claimed_tile(queue, ntile, claim, [&](const int64_t tile) {
                    typename R::vec g[KCH][W];
#pragma unroll
                    for (int j = 0; j < KCH; ++j) {   // all loads of the tile first
                        const int64_t c = tile * width + (int64_t)j * threads + threadIdx.x;
#pragma unroll
                        for (int w = 0; w < W; ++w) g[j][w] = c < nchunk ? R::load(rows.p[w], c) : typename R::vec{};
                    }
#pragma unroll
                    for (int j = 0; j < KCH; ++j) {   // a chunk beyond the end holds zeros and adds nothing
                        static_for<0, VEC>([&](auto kc) {
                            constexpr int K = decltype(kc)::value;
                            float ge[W];
                            static_for<0, W>([&](auto wc) {
                                constexpr int Wi = decltype(wc)::value;
                                ge[Wi] = R::template get<K>(g[j][Wi]);
                            });
                            gram_step<W>(acc, ge);
                        });
                        fold_now();   // per chunk, as with one chunk per tile: the sums do not depend on KCH
                    }
                });
            } else {
                const int64_t ntile = (nchunk + threads - 1) / threads;
                for_each_claimed_tile(queue, ntile, claim, [&](const int64_t tile) {
                    const int64_t c = tile * threads + threadIdx.x;
                    if (c < nchunk) {
                        process(c);
                        if constexpr (kFew) fold_now();
                    }
                });
            }
        }
    }
    if (!queued) {
        int64_t c = span.first;
        for (int k = 0; k < span.K && c < nchunk; ++k, c += span.step) {
            if constexpr (GRAM && !kFew) {
                if ((k & (kGramFold - 1)) == kGramFold - 1) fold_now();
            }
            process(c);
            if constexpr (kFew) fold_now();
        }
    }
    // elements not covered by whole chunks (the ragged end, or everything when
    // some buffer is not 16-byte aligned): same arithmetic, one element at a time
    const int64_t nrest = P - nchunk * VEC;
    int64_t r = span.first;
    for (int k = 0; k < span.K && r < nrest; ++k, r += span.step) {
        const int64_t j = nchunk * VEC + r;
        float ge[W];
#pragma unroll
        for (int w = 0; w < W; ++w) ge[w] = R::load1(rows.p[w], j);
        if constexpr (UPDATE) {
            float pe = params[j], ve = momentum[j];
            aff_step<W>(pe, ve, ge, cf);
            params[j] = pe;
            momentum[j] = ve;
            if (publish) publish_element(pe, publish, publish_bf16, j);
        }
        if constexpr (GRAM) gram_step<W>(acc, ge);
    }

    if constexpr (GRAM) {
        __shared__ fold_t wave_part[kBlock / 64][NG];
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int e = 0; e < NG; ++e) {
            const fold_t s = wave_sum_to_lane63((fold_t)acc[e] + fold[e * kBlock + threadIdx.x]);
            if (lane == 63) wave_part[wave][e] = s;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < NG; e += kBlock) {
            double s = 0.0;
#pragma unroll
            for (int q = 0; q < kBlock / 64; ++q) s += (double)wave_part[q][e];
            partials[(int64_t)e * gridDim.x + blockIdx.x] = s;
        }
    }
}

// ================================================================= step-by-step kernel
// LDS: (norms) nacc[U][kBlock] | wave_part[4][U], both double | coef[U][W] | lr[U] | mask[U]
// nacc holds one running sum of gbar^2 per thread and update.  It is double because the tiles a
// thread sees depend on the queue: each chunk's fp32 sum of four squares is formed in a fixed order,
// and added in double the order of the chunks matters only at 1e-16.
template <int W, bool UPDATE, bool NORMS>
__device__ __forceinline__ void seq_steps(float (&g)[W][4], float (&p)[4], float (&v)[4],
                                          const float* s_coef, const float* s_lr, const uint32_t* s_mask,
                                          double* s_nacc, const int U, const float mu, const float wd) {
    // Running compensation of p over the updates of a launch (Kahan): p moves by increments far smaller
    // than itself, and U plain roundings of p would add up like sqrt(U) half-ulps (U = 300: beyond 1e-6).
    // With the lost low part carried along, p ends within an ulp of the exactly accumulated value for any
    // U.  A single update keeps the plain fused step (nothing to carry).
    float lost[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int u = 0; u < U; ++u) {
        const uint32_t m = __builtin_amdgcn_readfirstlane(s_mask[u]);
        float gb[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int w = 0; w < W; ++w) {  // ascending worker id; the test is uniform over the wave
            if (m & (1u << w)) {
                const float c = s_coef[u * W + w];
#pragma unroll
                for (int k = 0; k < 4; ++k) gb[k] = __builtin_fmaf(c, g[w][k], gb[k]);
            }
        }
        if constexpr (NORMS) {
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) s = __builtin_fmaf(gb[k], gb[k], s);  // unused slots hold 0
            s_nacc[u * kBlock + threadIdx.x] += (double)s;
        }
        if constexpr (UPDATE) {
            const float lr = s_lr[u];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float d = __builtin_fmaf(wd, p[k], gb[k]);   // d = gbar + wd p
                v[k] = __builtin_fmaf(mu, v[k], d);                // v = mu v + d
                if (U == 1) {
                    p[k] = __builtin_fmaf(-lr, v[k], p[k]);        // p = p - lr v
                } else {
                    const float y = __builtin_fmaf(-lr, v[k], -lost[k]);   // the step, less what the last sum dropped
                    const float t = p[k] + y;
                    lost[k] = (t - p[k]) - y;
                    p[k] = t;
                }
            }
        }
    }
}

// COLLAPSED (with UPDATE and NORMS): the norms are accumulated update by update as usual, the update itself is
// applied once, as the affine map `cf` of the whole stream.  For wide fp32 rows with norms and a short stream:
// the Gram matrix of 17 to 32 fp32 rows costs 1536 matrix flops per element whatever the stream, the direct
// sums y_u + 1 multiply-adds per update.
template <int W, class R, bool UPDATE, bool NORMS, bool COLLAPSED = false>
__global__ __launch_bounds__(kBlock) void seq_kernel(float* __restrict__ params, float* __restrict__ momentum,
                                                     const RowPtrs rows, const float* __restrict__ t_coef,
                                                     const float* __restrict__ t_lr,
                                                     const uint32_t* __restrict__ t_mask, const int U,
                                                     const float mu, const float wd, const int64_t P,
                                                     const int vec_ok, const int span_g, const int span_k,
                                                     void* __restrict__ publish, const int publish_bf16,
                                                     double* __restrict__ partials, TileQueue* __restrict__ queue,
                                                     const int claim, const InlineTables inl, const AffCoef cf) {
    static_assert(R::VEC == 4, "the step-by-step kernel works on 4-element chunks");
    static_assert(!COLLAPSED || (UPDATE && NORMS), "the collapsed update rides on the norm walk");
    extern __shared__ double lds[];
    double* s_nacc = lds;
    double* s_wave = s_nacc + (NORMS ? U * kBlock : 0);
    float* s_coef = reinterpret_cast<float*>(s_wave + (NORMS ? (kBlock / 64) * U : 0));
    float* s_lr = s_coef + U * W;
    uint32_t* s_mask = reinterpret_cast<uint32_t*>(s_lr + U);
    if (t_coef) {
        for (int i = threadIdx.x; i < U * W; i += kBlock) s_coef[i] = t_coef[i];
        for (int i = threadIdx.x; i < U; i += kBlock) {
            s_lr[i] = t_lr[i];
            s_mask[i] = t_mask[i];
        }
    } else {  // small tables ride in the kernel arguments
        for (int i = threadIdx.x; i < U * W; i += kBlock) s_coef[i] = inl.coef[i];
        for (int i = threadIdx.x; i < U; i += kBlock) {
            s_lr[i] = inl.lr[i];
            s_mask[i] = inl.mask[i];
        }
    }
    if constexpr (NORMS)
        for (int u = 0; u < U; ++u) s_nacc[u * kBlock + threadIdx.x] = 0.0;
    __syncthreads();

    const Span span = make_span(span_g, span_k);
    const int64_t nchunk = vec_ok ? P / 4 : 0;

    auto process = [&](const int64_t c) {
        typename R::vec raw[W];
#pragma unroll
        for (int w = 0; w < W; ++w) raw[w] = R::load(rows.p[w], c);
        float p[4] = {0, 0, 0, 0}, v[4] = {0, 0, 0, 0};
        if constexpr (UPDATE) {
            const f32x4 pv = load_state(params, c);
            const f32x4 vv = load_state(momentum, c);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                p[k] = pv[k];
                v[k] = vv[k];
            }
        }
        float g[W][4];
        static_for<0, W>([&](auto wc) {
            constexpr int Wi = decltype(wc)::value;
            static_for<0, 4>([&](auto kc) {
                constexpr int K = decltype(kc)::value;
                g[Wi][K] = R::template get<K>(raw[Wi]);
            });
        });
        if constexpr (COLLAPSED) {
            seq_steps<W, false, true>(g, p, v, s_coef, s_lr, s_mask, s_nacc, U, mu, wd);
            static_for<0, 4>([&](auto kc) {
                constexpr int K = decltype(kc)::value;
                float ge[W];
#pragma unroll
                for (int w = 0; w < W; ++w) ge[w] = g[w][K];
                aff_step<W>(p[K], v[K], ge, cf);
            });
        } else {
            seq_steps<W, UPDATE, NORMS>(g, p, v, s_coef, s_lr, s_mask, s_nacc, U, mu, wd);
        }
        if constexpr (UPDATE) {
            f32x4 pv, vv;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                pv[k] = p[k];
                vv[k] = v[k];
            }
            store_state(pv, params, c);
            store_state(vv, momentum, c);
            if (publish) publish_chunk(pv, publish, publish_bf16, c);
        }
    };
    if (claim > 0) {   // tiles from the queue
        const int64_t ntile = (nchunk + kBlock - 1) / kBlock;
        for_each_claimed_tile(queue, ntile, claim, [&](const int64_t tile) {
            const int64_t c = tile * kBlock + threadIdx.x;
            if (c < nchunk) process(c);
        });
    } else {
        int64_t c = span.first;
        for (int k = 0; k < span.K && c < nchunk; ++k, c += span.step) process(c);
    }
    const int64_t nrest = P - nchunk * 4;
    int64_t r = span.first;
    for (int k = 0; k < span.K && r < nrest; ++k, r += span.step) {
        const int64_t j = nchunk * 4 + r;
        float g[W][4];
#pragma unroll
        for (int w = 0; w < W; ++w) {
            g[w][0] = R::load1(rows.p[w], j);
            g[w][1] = g[w][2] = g[w][3] = 0.0f;
        }
        float p[4] = {0, 0, 0, 0}, v[4] = {0, 0, 0, 0};
        if constexpr (UPDATE) {
            p[0] = params[j];
            v[0] = momentum[j];
        }
        if constexpr (COLLAPSED) {
            seq_steps<W, false, true>(g, p, v, s_coef, s_lr, s_mask, s_nacc, U, mu, wd);
            float ge[W];
#pragma unroll
            for (int w = 0; w < W; ++w) ge[w] = g[w][0];
            aff_step<W>(p[0], v[0], ge, cf);
        } else {
            seq_steps<W, UPDATE, NORMS>(g, p, v, s_coef, s_lr, s_mask, s_nacc, U, mu, wd);
        }
        if constexpr (UPDATE) {
            params[j] = p[0];
            momentum[j] = v[0];
            if (publish) publish_element(p[0], publish, publish_bf16, j);
        }
    }

    if constexpr (NORMS) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        for (int u = 0; u < U; ++u) {
            const double s = wave_sum_to_lane63(s_nacc[u * kBlock + threadIdx.x]);
            if (lane == 63) s_wave[wave * U + u] = s;
        }
        __syncthreads();
        for (int u = threadIdx.x; u < U; u += kBlock) {
            double s = 0.0;
#pragma unroll
            for (int q = 0; q < kBlock / 64; ++q) s += s_wave[q * U + u];
            partials[(int64_t)u * gridDim.x + blockIdx.x] = s;
        }
    }
}

// ================================================================= finishing kernels
__global__ __launch_bounds__(kBlock) void reduce_kernel(const double* __restrict__ partials, const int grid,
                                                        double* __restrict__ sums_out,
                                                        float* __restrict__ sqrt_out) {
    __shared__ double s_wave[kBlock / 64];
    const int e = blockIdx.x;
    double s = 0.0;
    for (int b = threadIdx.x; b < grid; b += kBlock) s += partials[(int64_t)e * grid + b];
    // fixed order: within a wave by the cross-lane moves, then the waves in turn (these kernels last a
    // few microseconds, most of it latency, so one barrier instead of a tree of eight)
    s = wave_sum_to_lane63(s);
    if ((threadIdx.x & 63) == 63) s_wave[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int q = 0; q < kBlock / 64; ++q) t += s_wave[q];
        if (sums_out) sums_out[e] = t;
        if (sqrt_out) sqrt_out[e] = (float)sqrt(t);
    }
}

// One workgroup per update u: n_u^2 = sum over pairs (a <= b) of c_a c_b Gamma_ab (off-diagonal pairs twice),
// each thread one pair, then a fixed-order tree sum in double.
__global__ __launch_bounds__(kBlock) void gram_norms_kernel(const double* __restrict__ gamma,
                                                            const double* __restrict__ coef, const int U,
                                                            const int W, float* __restrict__ norms_out) {
    __shared__ double s_wave[kBlock / 64];
    const int u = blockIdx.x;
    const double* c = coef + (int64_t)u * W;
    const int ng = W * (W + 1) / 2;
    double s = 0.0;
    for (int e = threadIdx.x; e < ng; e += kBlock) {
        const double g = gamma[e];   // requested together with the coefficients: one memory latency, not two
        int a = 0, rem = e;
        while (rem >= W - a) {
            rem -= W - a;
            ++a;
        }
        const int b = a + rem;
        const double ca = c[a], cb = c[b];
        // rows outside the group take no part: a non-finite entry of a worker that is not a member (0 * inf)
        // must not reach this group's norm
        if (ca == 0.0 || cb == 0.0) continue;
        const double t = ca * cb * g;
        s += (a == b) ? t : 2.0 * t;
    }
    s = wave_sum_to_lane63(s);
    if ((threadIdx.x & 63) == 63) s_wave[threadIdx.x >> 6] = s;
    __syncthreads();
    // a tiny negative sum (rounding of a quadratic form that is zero) gives 0; a non-finite one stays
    // non-finite, so that a bad gradient report shows in the norms of the groups it is part of
    if (threadIdx.x == 0 && u < U) {
        double t = 0.0;
#pragma unroll
        for (int q = 0; q < kBlock / 64; ++q) t += s_wave[q];
        norms_out[u] = (float)sqrt(t < 0.0 && t > -1e300 ? 0.0 : t);
    }
}

// Packed upper triangle (row-major, a <= b) -> full symmetric W x W matrix; a zero
// matrix when gamma is null (empty shard).
// The packed triangle is over Wp >= W rows (the kernels' padded row count); W x W entries are copied out.
__global__ __launch_bounds__(kBlock) void gram_unpack_kernel(const double* __restrict__ gamma, const int Wp,
                                                             const int W, double* __restrict__ out) {
    const int i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= W * W) return;
    const int r = i / W, c = i % W;
    const int a = r < c ? r : c, b = r < c ? c : r;
    out[i] = gamma ? gamma[a * Wp - a * (a - 1) / 2 + (b - a)] : 0.0;
}

__global__ __launch_bounds__(kBlock) void fill_kernel(float* __restrict__ dst, const int64_t n, const float value) {
    const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) dst[i] = value;
}

// ================================================================= launchers
int padded_rows(int Wc) {
    if (Wc <= 16) return Wc < 1 ? 1 : Wc;
    return (Wc + 3) / 4 * 4;
}

namespace {

size_t seq_lds_bytes(int W, int U, bool norms) {
    return sizeof(float) * ((size_t)U * W + 2 * (size_t)U) +
           (norms ? sizeof(double) * ((size_t)(kBlock / 64) * U + (size_t)U * kBlock) : 0);
}

template <int W, class R, bool UPDATE, bool NORMS, bool COLLAPSED = false>
hipError_t launch_seq_t(const SeqArgs& a, int num_cu, int grid_cap, int* grid_out, hipStream_t s) {
    auto kern = seq_kernel<W, R, UPDATE, NORMS, COLLAPSED>;
    const size_t lds = seq_lds_bytes(W, a.U, NORMS);
    // one or two updates are bound by memory and take their tiles from the queue; longer streams are bound
    // by arithmetic and latency and keep the fixed assignment with as many waves as fit
    const int thread_bytes = W * (int)sizeof(typename R::vec) + (UPDATE ? 32 : 0);
    // the collapsed form does so little arithmetic per update that it is bound by memory for any stream it is used for
    const bool queued = a.queue && a.vec_ok && (COLLAPSED || seq_takes_queue(a.U));
    // (the collapsed form's norm walk -- LDS reads and a wave-uniform branch per row and update -- needs a second
    // workgroup per unit to hide under the memory time: 20 to 32 fp32 rows, 8 updates, 0.68-0.71 of the HBM peak with
    // two against 0.43-0.45 with one)
    const int per_cu = COLLAPSED ? 2 : queue_workgroups_per_cu(thread_bytes, UPDATE);
    const Geometry g = queued ? queue_geometry(num_cu, grid_cap, per_cu, thread_bytes)
                              : pick_geometry(a.P, 4, a.vec_ok != 0, NORMS, num_cu, grid_cap, thread_bytes, 4,
                                              COLLAPSED ? 2 : 1);   // (short shards as well: 25-30 % faster with two)
    *grid_out = g.grid;
    hipLaunchKernelGGL(kern, dim3(g.grid), dim3(kBlock), lds, s, a.params, a.momentum, a.rows, a.coef, a.lr, a.mask,
                       a.U, a.mu, a.wd, a.P, a.vec_ok, g.span_g, g.span_k, a.publish, a.publish_dtype == STAR_BF16 ? 1 : 0,
                       a.partials, a.queue, g.claim, a.coef ? InlineTables() : *a.inl, a.cf ? *a.cf : AffCoef());
    return hipGetLastError();
}

template <int W, class R, bool UPDATE, bool GRAM>
hipError_t launch_aff_t(const AffArgs& a, int num_cu, int grid_cap, int* grid_out, hipStream_t s) {
    // the Gram matrix alone on very few rows: enough chunks per thread for about 64 bytes in flight
    constexpr int kRowBytes = W * (int)sizeof(typename R::vec);
    // (134 M elements, 1 / 2 / 3 fp32 rows: 0.69 / 0.78 / 0.79 of the HBM peak against 0.40 / 0.66 / 0.78 with one
    // chunk; 1 / 2 / 3 bf16 rows with 4 / 4 / 2 chunks: 0.44 / 0.66 / 0.65 against 0.22 / 0.36 / 0.48)
    constexpr int KCH = (GRAM && !UPDATE && W <= kFewRows && kRowBytes < 64)
                            ? (kRowBytes <= 8 ? 8 : (kRowBytes <= 16 ? 4 : 2)) : 1;
    const bool queued = aff_takes_queue(GRAM, W, std::is_same<R, RowF32>::value, UPDATE) && a.queue && a.vec_ok;
    if constexpr (KCH > 1) {
        if (queued) {
            const int thread_bytes = kRowBytes * KCH;
            const Geometry g = queue_geometry(num_cu, grid_cap, 2, thread_bytes, Traffic::ReadOnly);
            *grid_out = g.grid;
            hipLaunchKernelGGL((aff_kernel<W, R, UPDATE, GRAM, KCH>), dim3(g.grid), dim3(g.threads), 0, s, a.params,
                               a.momentum, a.rows, a.cf, a.P, a.vec_ok, g.span_g, g.span_k, a.publish,
                               a.publish_dtype == STAR_BF16 ? 1 : 0, a.partials, a.queue, g.claim);
            return hipGetLastError();
        }
    }
    auto kern = aff_kernel<W, R, UPDATE, GRAM>;
    // long shards without the Gram accumulators: long-lived workgroups, tiles from the queue
    const int thread_bytes = W * (int)sizeof(typename R::vec) + (UPDATE ? 32 : 0);
    Geometry g = queued ? queue_geometry(num_cu, grid_cap, queue_workgroups_per_cu(thread_bytes, UPDATE), thread_bytes,
                                         UPDATE ? Traffic::Update : Traffic::ReadOnly)
                        : pick_geometry(a.P, R::VEC, a.vec_ok != 0, GRAM, num_cu, grid_cap);
    // 24 and more bf16 rows: twice as many workgroups of half the size (tiles of 1 KB per row) measured
    // 3-4 % faster (32 rows, 138 M elements: 1.92 against 1.98 ms); with 16 rows the same is 15 % slower,
    // and fp32 rows do not care.  With these half-size tiles claims of 4 (4 KB of every row, 8 KB of the
    // state) are the fastest: 1-4 % ahead of 3 on every box and shard length tried (32 rows, 138 M
    // elements: 1.81 against 1.89 ms; 24 rows 1.43 against 1.53 ms), 5 to 12 fall off again.
    if constexpr (std::is_same<R, RowBf16x4>::value && W >= 24 && UPDATE && !GRAM) {
        if (queued) {
            g.threads = kBlock / 2;
            g.grid = g.span_g = std::min(2 * g.grid, grid_cap);
            g.claim = 4;
            *grid_out = g.grid;
            hipLaunchKernelGGL((aff_kernel<W, R, UPDATE, GRAM, 1, true>), dim3(g.grid), dim3(g.threads), 0, s, a.params,
                               a.momentum, a.rows, a.cf, a.P, a.vec_ok, g.span_g, g.span_k, a.publish,
                               a.publish_dtype == STAR_BF16 ? 1 : 0, a.partials, a.queue, g.claim);
            return hipGetLastError();
        }
    }
    *grid_out = g.grid;
    hipLaunchKernelGGL(kern, dim3(g.grid), dim3(g.threads), 0, s, a.params, a.momentum, a.rows, a.cf, a.P, a.vec_ok,
                       g.span_g, g.span_k, a.publish, a.publish_dtype == STAR_BF16 ? 1 : 0, a.partials, a.queue,
                       g.claim);
    return hipGetLastError();
}

template <int W>
hipError_t launch_seq_w(int dtype, bool update, bool norms, const SeqArgs& a, int num_cu, int grid_cap,
                        int* grid_out, hipStream_t s) {
    if (a.cf) {   // collapsed update with direct norms: built for wide fp32 rows only
        if constexpr (W > 16) {
            if (dtype == STAR_F32 && update && norms)
                return launch_seq_t<W, RowF32, true, true, true>(a, num_cu, grid_cap, grid_out, s);
        }
        return hipErrorInvalidValue;
    }
    if (dtype == STAR_F32) {
        if (update && norms) return launch_seq_t<W, RowF32, true, true>(a, num_cu, grid_cap, grid_out, s);
        if (update) return launch_seq_t<W, RowF32, true, false>(a, num_cu, grid_cap, grid_out, s);
        return launch_seq_t<W, RowF32, false, true>(a, num_cu, grid_cap, grid_out, s);
    }
    if (update && norms) return launch_seq_t<W, RowBf16x4, true, true>(a, num_cu, grid_cap, grid_out, s);
    if (update) return launch_seq_t<W, RowBf16x4, true, false>(a, num_cu, grid_cap, grid_out, s);
    return launch_seq_t<W, RowBf16x4, false, true>(a, num_cu, grid_cap, grid_out, s);
}

template <int W>
hipError_t launch_aff_w(int dtype, bool update, bool gram, const AffArgs& a, int num_cu, int grid_cap,
                        int* grid_out, hipStream_t s) {
    if constexpr (W <= 16) {
        if (gram) {
            if (dtype == STAR_F32) {
                if (update) return launch_aff_t<W, RowF32, true, true>(a, num_cu, grid_cap, grid_out, s);
                return launch_aff_t<W, RowF32, false, true>(a, num_cu, grid_cap, grid_out, s);
            }
            if (update) return launch_aff_t<W, RowBf16x4, true, true>(a, num_cu, grid_cap, grid_out, s);
            return launch_aff_t<W, RowBf16x4, false, true>(a, num_cu, grid_cap, grid_out, s);
        }
    }
    if (gram || !update) return hipErrorInvalidValue;
    if (dtype == STAR_F32) return launch_aff_t<W, RowF32, true, false>(a, num_cu, grid_cap, grid_out, s);
    return launch_aff_t<W, RowBf16x4, true, false>(a, num_cu, grid_cap, grid_out, s);
}

}  // namespace

int seq_max_updates(int Wp, bool norms) {
    // stay inside 64 KB of LDS per workgroup
    const size_t budget = 60 * 1024;
    int u = 1;
    while (u < 256 && seq_lds_bytes(Wp, u + 1, norms) <= budget) ++u;
    return u;
}

hipError_t launch_seq(int Wp, int dtype, bool update, bool norms, const SeqArgs& a, int num_cu, int grid_cap,
                      int* grid_out, hipStream_t s) {
    if (!update && !norms) return hipErrorInvalidValue;
    if (a.U < 1 || a.U > seq_max_updates(Wp, norms)) return hipErrorInvalidValue;
    switch (Wp) {
#define X(N) case N: return launch_seq_w<N>(dtype, update, norms, a, num_cu, grid_cap, grid_out, s);
        STAR_FOR_EACH_W(X)
#undef X
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_affine(int Wp, int dtype, bool update, bool gram, const AffArgs& a, int num_cu, int grid_cap,
                         int* grid_out, hipStream_t s) {
    if (!update && !gram) return hipErrorInvalidValue;
    switch (Wp) {
#define X(N) case N: return launch_aff_w<N>(dtype, update, gram, a, num_cu, grid_cap, grid_out, s);
        STAR_FOR_EACH_W(X)
#undef X
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_reduce(const double* partials, int n_out, int grid, double* sums_out, float* sqrt_out,
                         hipStream_t s) {
    if (n_out < 1) return hipSuccess;
    hipLaunchKernelGGL(reduce_kernel, dim3(n_out), dim3(kBlock), 0, s, partials, grid, sums_out, sqrt_out);
    return hipGetLastError();
}

hipError_t launch_gram_norms(const double* gamma, const double* coef, int U, int Wp, float* norms_out,
                             hipStream_t s) {
    if (U < 1) return hipSuccess;
    hipLaunchKernelGGL(gram_norms_kernel, dim3(U), dim3(kBlock), 0, s, gamma, coef, U, Wp,
                       norms_out);
    return hipGetLastError();
}

hipError_t launch_gram_unpack(const double* gamma, int Wp, int W, double* out, hipStream_t s) {
    hipLaunchKernelGGL(gram_unpack_kernel, dim3((W * W + kBlock - 1) / kBlock), dim3(kBlock), 0, s, gamma, Wp, W, out);
    return hipGetLastError();
}

hipError_t launch_fill(float* dst, int64_t n, float value, hipStream_t s) {
    if (n < 1) return hipSuccess;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, dst, n, value);
    return hipGetLastError();
}

}  // namespace star
