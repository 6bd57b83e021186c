// Host-side planning for the group-synchronous update: argument checks,
// canonical groups, coefficient tables, the collapsed affine map and the
// arithmetic cost of each evaluation.  Pure host code (no HIP).
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "star.h"

namespace star {

struct Plan {
    int32_t W = 0;   // workers as given by the caller
    int32_t U = 0;   // updates
    int32_t Wc = 0;  // rows referenced by at least one group ("compact" rows)
    int32_t row_of[STAR_MAX_WORKERS] = {};  // compact index -> worker id, ascending

    // Dense per-update tables over compact rows (row-major [U][Wc]).
    // coef is c_{u,w} (0 for non-members), mask has bit k set when compact row k
    // is a member of update u, lr is the effective rate of update u
    // (per-update or global rate, times y_u/W under the scaling rule of
    // Section 4.3.1).
    std::vector<double> coef;
    std::vector<uint32_t> mask;
    std::vector<double> lr;
    std::vector<int32_t> ysize;
    bool negative_coef = false;   // some coefficient is below zero (possible with STAR_W_EXPLICIT only)

    double mu = 0, wd = 0;

    // The U updates as one affine map (p_U, v_U) = M (p_0, v_0) + B g,
    // B row-major [2][Wc]; composed in double.
    double M[4] = {1, 0, 0, 1};
    std::vector<double> B;

    // fused multiply-adds per element of the two evaluations
    double fma_seq = 0, fma_affine = 0;
};

// Checks the stream and the hyper-parameters and fills `plan`.  `hp` may be
// null when only norms are planned (then `wmode_only` gives the weighting and
// no affine map is built).  On error returns the status and a message.
star_status build_plan(int32_t W, const star_updates* upd, const star_hparams* hp, int32_t wmode_only,
                       bool want_norms, Plan* plan, std::string* err);

// Largest Wc for which the pairwise-product (Gram) route to the norms is built: on the vector
// ALUs (accumulators in registers) and on the matrix cores.
constexpr int kMaxValuGramW = 16;
constexpr int kMaxGramW = 32;

enum class Route { Seq, Affine };

// Picks the evaluation: the literal kernel for a single update on fp32 rows,
// the collapsed one otherwise.  `grad_bytes` is the size of a gradient element,
// `forced` a star_kernel.
Route choose_route(const Plan& plan, int grad_bytes, int forced);

}  // namespace star
