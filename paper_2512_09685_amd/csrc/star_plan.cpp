// Host-side planning: see star_plan.h.
#include "star_plan.h"

#include <algorithm>
#include <cmath>
#include <cstdio>

namespace star {

namespace {

star_status fail(std::string* err, star_status s, const char* fmt, long a = 0, long b = 0, long c = 0) {
    if (err) {
        char buf[256];
        std::snprintf(buf, sizeof buf, fmt, a, b, c);
        *err = buf;
    }
    return s;
}

}  // namespace

star_status build_plan(int32_t W, const star_updates* upd, const star_hparams* hp, int32_t wmode_only,
                       bool want_norms, Plan* plan, std::string* err) {
    if (!upd) return fail(err, STAR_ERR_NULL, "updates struct is NULL");
    if (W < 1 || W > STAR_MAX_WORKERS) return fail(err, STAR_ERR_SHAPE, "W=%ld outside [1,%ld]", W, STAR_MAX_WORKERS);
    if (upd->U < 0) return fail(err, STAR_ERR_SHAPE, "U=%ld is negative", upd->U);
    const int32_t U = upd->U;
    const int32_t wmode = hp ? hp->wmode : wmode_only;
    if (wmode != STAR_W_MEAN && wmode != STAR_W_STALE && wmode != STAR_W_EXPLICIT)
        return fail(err, STAR_ERR_HPARAM, "unknown weighting mode %ld", wmode);
    if (hp) {
        if (!std::isfinite(hp->lr) || !std::isfinite(hp->momentum) || !std::isfinite(hp->weight_decay))
            return fail(err, STAR_ERR_HPARAM, "lr, momentum and weight decay must be finite");
    }
    if (U > 0) {
        if (!upd->offsets || !upd->members) return fail(err, STAR_ERR_NULL, "offsets or members is NULL");
        if (wmode == STAR_W_EXPLICIT && !upd->coeff)
            return fail(err, STAR_ERR_NULL, "explicit weighting needs a coefficient array");
        if (upd->offsets[0] != 0) return fail(err, STAR_ERR_GROUP, "offsets[0] must be 0");
    }

    plan->W = W;
    plan->U = U;
    plan->negative_coef = false;
    plan->mu = hp ? (double)hp->momentum : 0.0;
    plan->wd = hp ? (double)hp->weight_decay : 0.0;

    // pass 1: group shapes, ids, duplicates; which rows are referenced
    uint32_t used = 0;
    for (int32_t u = 0; u < U; ++u) {
        const int64_t lo = upd->offsets[u], hi = upd->offsets[u + 1];
        if (hi <= lo) return fail(err, STAR_ERR_GROUP, "group %ld is empty or offsets decrease", u);
        if (hi - lo > W) return fail(err, STAR_ERR_GROUP, "group %ld lists more members than workers", u);
        uint32_t seen = 0;
        for (int64_t m = lo; m < hi; ++m) {
            const int32_t id = upd->members[m];
            if (id < 0 || id >= W) return fail(err, STAR_ERR_GROUP, "group %ld: worker id %ld outside [0,%ld)", u, id, W);
            if (seen & (1u << id)) return fail(err, STAR_ERR_GROUP, "group %ld lists worker %ld twice", u, id);
            seen |= 1u << id;
            if (wmode == STAR_W_STALE && upd->staleness && upd->staleness[m] < 0)
                return fail(err, STAR_ERR_HPARAM, "group %ld: negative staleness", u);
            if (wmode == STAR_W_EXPLICIT && !std::isfinite(upd->coeff[m]))
                return fail(err, STAR_ERR_HPARAM, "group %ld: non-finite coefficient", u);
        }
        used |= seen;
        if (hp && upd->lr && !std::isfinite(upd->lr[u]))
            return fail(err, STAR_ERR_HPARAM, "update %ld: non-finite learning rate", u);
    }

    // compact rows, ascending worker id (keeps the summation order "ascending id")
    int32_t compact_of[STAR_MAX_WORKERS];
    int32_t Wc = 0;
    for (int32_t w = 0; w < W; ++w) {
        compact_of[w] = -1;
        if (used & (1u << w)) {
            compact_of[w] = Wc;
            plan->row_of[Wc++] = w;
        }
    }
    plan->Wc = Wc;

    // pass 2: dense tables
    plan->coef.assign((size_t)U * std::max(Wc, 1), 0.0);
    plan->mask.assign(U, 0u);
    plan->lr.assign(U, 0.0);
    plan->ysize.assign(U, 0);
    double fma_seq = 0;
    for (int32_t u = 0; u < U; ++u) {
        const int64_t lo = upd->offsets[u], hi = upd->offsets[u + 1];
        const int32_t y = (int32_t)(hi - lo);
        plan->ysize[u] = y;
        for (int64_t m = lo; m < hi; ++m) {
            double c;
            if (wmode == STAR_W_EXPLICIT) {
                c = (double)upd->coeff[m];
            } else {
                double a = 1.0;
                if (wmode == STAR_W_STALE && upd->staleness) a = 1.0 / (1.0 + (double)upd->staleness[m]);
                c = a / (double)y;
            }
            const int32_t k = compact_of[upd->members[m]];
            if (c < 0.0) plan->negative_coef = true;
            plan->coef[(size_t)u * Wc + k] = c;
            plan->mask[u] |= 1u << k;
        }
        if (hp) {
            double lr = upd->lr ? (double)upd->lr[u] : (double)hp->lr;
            if (hp->scale_lr_by_group) lr *= (double)y / (double)W;
            plan->lr[u] = lr;
        }
        fma_seq += y + (hp ? 3 : 0) + (want_norms ? 1 : 0);
    }
    plan->fma_seq = fma_seq;
    // beyond 16 rows the Gram matrix is formed on the matrix cores: 128 instructions of 64 cycles per
    // 256 elements and wave, about what 260 vector multiply-adds per element would take
    const double gram_cost = Wc <= kMaxValuGramW ? 0.5 * Wc * (Wc + 1) : 260.0;
    plan->fma_affine = (hp ? 2.0 * Wc + 4.0 : 0.0) + (want_norms ? gram_cost : 0.0);

    // the collapsed map: x = (p, v);  x' = A_u x + b_u gbar_u,
    //   A_u = [[1 - lr wd, -lr mu], [wd, mu]],  b_u = (-lr, 1),  gbar_u = c_u . g
    plan->M[0] = 1; plan->M[1] = 0; plan->M[2] = 0; plan->M[3] = 1;
    plan->B.assign((size_t)2 * std::max(Wc, 1), 0.0);
    if (hp) {
        double* B0 = plan->B.data();
        double* B1 = B0 + Wc;
        const double mu = plan->mu, wd = plan->wd;
        for (int32_t u = 0; u < U; ++u) {
            const double lr = plan->lr[u];
            const double a00 = 1.0 - lr * wd, a01 = -lr * mu, a10 = wd, a11 = mu;
            const double m00 = a00 * plan->M[0] + a01 * plan->M[2], m01 = a00 * plan->M[1] + a01 * plan->M[3];
            const double m10 = a10 * plan->M[0] + a11 * plan->M[2], m11 = a10 * plan->M[1] + a11 * plan->M[3];
            plan->M[0] = m00; plan->M[1] = m01; plan->M[2] = m10; plan->M[3] = m11;
            const double* c = &plan->coef[(size_t)u * Wc];
            for (int32_t k = 0; k < Wc; ++k) {
                const double b0 = a00 * B0[k] + a01 * B1[k] - lr * c[k];
                const double b1 = a10 * B0[k] + a11 * B1[k] + c[k];
                B0[k] = b0;
                B1[k] = b1;
            }
        }
    }
    return STAR_OK;
}

Route choose_route(const Plan& plan, int grad_bytes, int forced) {
    static_assert(STAR_MAX_WORKERS <= kMaxGramW, "every admissible row count has a Gram kernel");
    if (forced == STAR_KERNEL_SEQ) return Route::Seq;
    if (forced == STAR_KERNEL_AFFINE || forced == STAR_KERNEL_AFFINE_MFMA) return Route::Affine;
    // A single update has nothing to collapse, and on fp32 rows the literal kernel does the least work for
    // it (no Gram matrix behind the norm, one finishing kernel fewer: 0.82 against 0.95 ms on 110 M
    // elements with the norm, the same time without).  On bf16 rows, and from two updates on, the
    // collapsed form is ahead: both forms are bound by the same bytes, and the literal kernel's inner loop
    // (LDS coefficient reads, a wave-uniform branch per row and update) stops hiding under the memory time
    // at the low occupancy the large shards run best at -- a single update on bf16 rows 4 % behind, two
    // updates 1.40 against 1.49 ms in its favour on 16 fp32 rows but 12.4 against 9.6 ms on 16 bf16 rows,
    // behind everywhere from three updates on.
    return (plan.U <= 1 && grad_bytes == 4) ? Route::Seq : Route::Affine;
}

}  // namespace star
