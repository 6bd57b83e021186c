// gfx950 kernel for aggregation without the optimizer step: for every group u,
//     out_u[j] = sum_{w in G_u} c_{u,w} g_w[j]
// -- what a parent aggregates from its children and itself before it
// broadcasts in the all-reduce architecture (Section 4.2, "All-reduce
// architecture"), and what a tree node forwards upward (Section 4.4.2).
//
// Same layout and mapping as the update kernels: a thread owns chunks of 4
// elements, holds the W gradients of the chunk in registers, walks the groups
// with a wave-uniform member test (tables in LDS), fp32 FMA chain in ascending
// worker id.  Every row is read once, every output written once (fp32, or bf16
// rounded to nearest even).  Optional per-group norms as in the update kernel.
#include "star_device.h"

namespace star {

// LDS: out pointers [U] (8 bytes each) | coef[U][W] | mask[U] | (norms) wave[4][U] | nacc[U][kBlock]
template <int W, class R>
__global__ __launch_bounds__(kBlock) void reduce_rows_kernel(const RowPtrs rows, const float* __restrict__ t_coef,
                                                             const uint32_t* __restrict__ t_mask,
                                                             void* const* __restrict__ t_out, const int U,
                                                             const int out_bf16, const int64_t P, const int vec_ok,
                                                             const int norms, const int span_g, const int span_k,
                                                             double* __restrict__ partials,
                                                             TileQueue* __restrict__ queue, const int claim,
                                                             const InlineTables inl) {
    extern __shared__ uint64_t lds64[];
    // out pointers | (norms) running sums of gbar^2 per thread and group, and per wave, in double (the
    // tiles a thread sees depend on the queue; see the step-by-step kernel) | coefficients | masks
    uint64_t* s_out = lds64;
    double* s_nacc = reinterpret_cast<double*>(s_out + U);
    double* s_wave = s_nacc + (norms ? U * kBlock : 0);
    float* s_coef = reinterpret_cast<float*>(s_wave + (norms ? (kBlock / 64) * U : 0));
    uint32_t* s_mask = reinterpret_cast<uint32_t*>(s_coef + U * W);
    if (t_coef) {
        for (int i = threadIdx.x; i < U * W; i += kBlock) s_coef[i] = t_coef[i];
        for (int i = threadIdx.x; i < U; i += kBlock) {
            s_mask[i] = t_mask[i];
            s_out[i] = reinterpret_cast<uint64_t>(t_out[i]);
        }
    } else {  // small tables ride in the kernel arguments
        for (int i = threadIdx.x; i < U * W; i += kBlock) s_coef[i] = inl.coef[i];
        for (int i = threadIdx.x; i < U; i += kBlock) {
            s_mask[i] = inl.mask[i];
            s_out[i] = reinterpret_cast<uint64_t>(inl.out[i]);
        }
    }
    if (norms)
        for (int u = 0; u < U; ++u) s_nacc[u * kBlock + threadIdx.x] = 0.0;
    __syncthreads();

    const Span span = make_span(span_g, span_k);
    const int64_t nchunk = vec_ok ? P / 4 : 0;

    // one pass over the groups for the element(s) held in g; `store` writes gbar of group u
    auto walk = [&](float (&g)[W][4], auto&& store) {
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
            if (norms) {
                float s = 0.0f;
#pragma unroll
                for (int k = 0; k < 4; ++k) s = __builtin_fmaf(gb[k], gb[k], s);  // unused slots hold 0
                s_nacc[u * kBlock + threadIdx.x] += (double)s;
            }
            const uint64_t o = s_out[u];
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)o);
            const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(o >> 32));
            store(reinterpret_cast<void*>(((uint64_t)hi << 32) | lo), gb);
        }
    };

    auto process = [&](const int64_t c) {
        typename R::vec raw[W];
#pragma unroll
        for (int w = 0; w < W; ++w) raw[w] = R::load(rows.p[w], c);
        float g[W][4];
        static_for<0, W>([&](auto wc) {
            constexpr int Wi = decltype(wc)::value;
            static_for<0, 4>([&](auto kc) {
                constexpr int K = decltype(kc)::value;
                g[Wi][K] = R::template get<K>(raw[Wi]);
            });
        });
        walk(g, [&](void* out, const float (&gb)[4]) {
            const f32x4 x = {gb[0], gb[1], gb[2], gb[3]};
            publish_chunk(x, out, out_bf16, c);
        });
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
        walk(g, [&](void* out, const float (&gb)[4]) {
            publish_element(gb[0], out, out_bf16, j);
        });
    }

    if (norms) {
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

namespace {

size_t reduce_lds_bytes(int W, int U, bool norms) {
    return sizeof(uint64_t) * (size_t)U + sizeof(float) * ((size_t)U * W + (size_t)U) +
           (norms ? sizeof(double) * ((size_t)(kBlock / 64) * U + (size_t)U * kBlock) : 0);
}

template <int W, class R>
hipError_t launch_reduce_t(const ReduceArgs& a, int num_cu, int grid_cap, int* grid_out, hipStream_t s) {
    auto kern = reduce_rows_kernel<W, R>;
    const size_t lds = reduce_lds_bytes(W, a.U, a.norms != 0);
    const bool queued = a.queue && a.vec_ok;
    const Geometry g = queued ? queue_geometry(num_cu, grid_cap, queue_workgroups_per_cu(0, false),
                                               W * (int)sizeof(typename R::vec) + 16, Traffic::Reduce)
                              // (with norms: long-lived workgroups, and at least two of them per unit whatever
                                              // the tile weighs -- 32 bf16 rows, 16 groups, 32 Mi elements: one per unit 1.72 ms)
                              : pick_geometry(a.P, 4, a.vec_ok != 0, a.norms != 0, num_cu, grid_cap,
                                              W * (int)sizeof(typename R::vec), 4, 2);
    *grid_out = g.grid;
    hipLaunchKernelGGL(kern, dim3(g.grid), dim3(kBlock), lds, s, a.rows, a.coef, a.mask, a.out, a.U,
                       a.out_dtype == STAR_BF16 ? 1 : 0, a.P, a.vec_ok, a.norms, g.span_g, g.span_k, a.partials,
                       a.queue, g.claim, a.coef ? InlineTables() : *a.inl);
    return hipGetLastError();
}

}  // namespace

int reduce_max_updates(int Wp, bool norms) {
    const size_t budget = 60 * 1024;  // stay inside 64 KB of LDS per workgroup
    int u = 1;
    while (u < 256 && reduce_lds_bytes(Wp, u + 1, norms) <= budget) ++u;
    return u;
}

hipError_t launch_group_reduce(int Wp, int dtype, const ReduceArgs& a, int num_cu, int grid_cap, int* grid_out,
                               hipStream_t s) {
    if (a.U < 1 || a.U > reduce_max_updates(Wp, a.norms != 0)) return hipErrorInvalidValue;
    switch (Wp) {
#define X(N)                                                                                         \
    case N:                                                                                          \
        return dtype == STAR_F32 ? launch_reduce_t<N, RowF32>(a, num_cu, grid_cap, grid_out, s)      \
                                 : launch_reduce_t<N, RowBf16x4>(a, num_cu, grid_cap, grid_out, s);
        STAR_FOR_EACH_W(X)
#undef X
        default: return hipErrorInvalidValue;
    }
}

}  // namespace star
