/*
 * CPU oracle for the group-synchronous parameter update of STAR
 * (arXiv 2512.09685).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded
 * statement of what the update computes, used only to check the GPU library
 * and to time a CPU baseline.  It shares no code with the GPU library and the
 * GPU library never calls it.
 *
 * What is computed, and where the paper defines it:
 *   - A parameter server keeps one copy of the parameters and adds up the
 *     gradient copies of the workers that feed an update, then updates the
 *     parameters (Section 1: SSGD waits for all workers, ASGD updates on any
 *     one worker; Section 2, the parameter-server description).
 *   - STAR's x-order modes use the gradients of x workers, or of one cluster
 *     of workers, for each update (Section 1 item (2); Section 4.2).  The set
 *     of workers behind one update is the "worker group" (Section 1 item (4)).
 *   - After a mode switch the learning rate is scaled with the number of
 *     gradient reports y in the update, r_new = (y/N) r_SSGD (Section 4.3.1,
 *     "Scaling learning rate after switching").
 *   - The paper implements this in PyTorch (Section 5.1, Implementation) and
 *     does not print the optimizer; the reading taken here is PyTorch's SGD:
 *         d = gbar + wd * p;   v = mu * v + d;   p = p - lr * v
 *     with gbar the group's (weighted) mean gradient, dampening 0, no
 *     Nesterov, weight decay coupled into the gradient.
 *   - Per-group gradient norm: ||gbar_u||_2 over the shard, before weight
 *     decay (the gradient-norm progress signal of Sections 4.3.1 and 7).
 *
 * Member weight a_{u,m}:  MEAN: 1;  STALE: 1/(1+s_{u,m}) (not renormalised);
 * EXPLICIT: coefficient given directly (then no 1/y factor is applied).
 * gbar_u[j] = sum over listed members m of  coef(u,m) * g_{member}[j],
 * coef = a/y for MEAN and STALE.
 *
 * Parity pins (tests/test_oracle_pins.py): hand-computed cases exact in
 * binary, closed forms, SSGD / ASGD special cases written independently,
 * torch.optim.SGD in float64, linearity, permutation and batch-split
 * invariants, exhaustive tiny cases in rational arithmetic.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_W_MEAN = 0, ORACLE_W_STALE = 1, ORACLE_W_EXPLICIT = 2 };

typedef struct {
    int32_t U;
    const int32_t *offsets;   /* [U+1] */
    const int32_t *members;   /* [offsets[U]] */
    const int32_t *staleness; /* same length, or NULL */
    const float *coeff;       /* same length, EXPLICIT only */
    const float *lr;          /* [U] or NULL */
} oracle_updates;

typedef struct {
    float lr, momentum, weight_decay;
    int32_t wmode;
    int32_t scale_lr_by_group;
} oracle_hparams;

/* value of element j of a gradient row, exactly, as a double */
static double grad_at(const void *row, int dtype, int64_t j)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)row)[j];
    uint32_t bits = (uint32_t)((const uint16_t *)row)[j] << 16; /* bf16 = top half of a float */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double member_coef(const oracle_updates *up, int wmode, int32_t idx, int32_t y)
{
    if (wmode == ORACLE_W_EXPLICIT)
        return (double)up->coeff[idx];
    double a = 1.0;
    if (wmode == ORACLE_W_STALE && up->staleness)
        a = 1.0 / (1.0 + (double)up->staleness[idx]);
    return a / (double)y;
}

static double update_lr(const oracle_updates *up, const oracle_hparams *hp, int32_t u, int32_t y, int32_t W)
{
    double lr = up->lr ? (double)up->lr[u] : (double)hp->lr;
    if (hp->scale_lr_by_group)
        lr *= (double)y / (double)W; /* r_new = (M_new / M) r, M_new = y M / N */
    return lr;
}

static int check_stream(const oracle_updates *up, int32_t W)
{
    if (up->U < 0) return 2;
    if (up->U > 0 && (!up->offsets || !up->members)) return 1;
    for (int32_t u = 0; u < up->U; ++u) {
        int32_t lo = up->offsets[u], hi = up->offsets[u + 1];
        if (hi <= lo) return 3;
        for (int32_t m = lo; m < hi; ++m) {
            if (up->members[m] < 0 || up->members[m] >= W) return 3;
            for (int32_t k = lo; k < m; ++k)
                if (up->members[k] == up->members[m]) return 3;
        }
    }
    return 0;
}

/*
 * Exact mode.  params / momentum are double arrays holding the state; all
 * arithmetic is double; nothing is rounded inside the call.  norms_out may be
 * NULL, else receives U doubles.  Returns 0, or a nonzero code for a
 * malformed stream (no state is touched then).
 */
int oracle_group_update_f64(double *params, double *momentum, const void *const *rows, int grad_dtype,
                            int64_t P, int32_t W, const oracle_updates *up, const oracle_hparams *hp,
                            double *norms_out)
{
    int rc = check_stream(up, W);
    if (rc) return rc;
    const double mu = (double)hp->momentum, wd = (double)hp->weight_decay;
    for (int32_t u = 0; u < up->U; ++u) {
        const int32_t lo = up->offsets[u];
        const int32_t y = up->offsets[u + 1] - lo;
        const double lr = update_lr(up, hp, u, y, W);
        double sumsq = 0.0;
        for (int64_t j = 0; j < P; ++j) {
            double gbar = 0.0;
            for (int32_t m = 0; m < y; ++m)
                gbar += member_coef(up, hp->wmode, lo + m, y) * grad_at(rows[up->members[lo + m]], grad_dtype, j);
            sumsq += gbar * gbar;
            double d = gbar + wd * params[j];
            momentum[j] = mu * momentum[j] + d;
            params[j] = params[j] - lr * momentum[j];
        }
        if (norms_out) norms_out[u] = sqrt(sumsq);
    }
    return 0;
}

/*
 * Call-boundary wrapper: the state a parameter server stores between calls is
 * fp32.  Promote to double, run the exact update, round to nearest fp32 once.
 * scratch must hold 2*P doubles.
 */
int oracle_group_update(float *params, float *momentum, const void *const *rows, int grad_dtype, int64_t P,
                        int32_t W, const oracle_updates *up, const oracle_hparams *hp, double *norms_out,
                        double *scratch)
{
    double *p = scratch, *v = scratch + P;
    for (int64_t j = 0; j < P; ++j) {
        p[j] = (double)params[j];
        v[j] = (double)momentum[j];
    }
    int rc = oracle_group_update_f64(p, v, rows, grad_dtype, P, W, up, hp, norms_out);
    if (rc) return rc;
    for (int64_t j = 0; j < P; ++j) {
        params[j] = (float)p[j];
        momentum[j] = (float)v[j];
    }
    return 0;
}

/* Norms alone: n_u = sqrt(sum_j gbar_u[j]^2). */
int oracle_group_norms(const void *const *rows, int grad_dtype, int64_t P, int32_t W, const oracle_updates *up,
                       int32_t wmode, double *norms_out)
{
    int rc = check_stream(up, W);
    if (rc) return rc;
    for (int32_t u = 0; u < up->U; ++u) {
        const int32_t lo = up->offsets[u];
        const int32_t y = up->offsets[u + 1] - lo;
        double sumsq = 0.0;
        for (int64_t j = 0; j < P; ++j) {
            double gbar = 0.0;
            for (int32_t m = 0; m < y; ++m)
                gbar += member_coef(up, wmode, lo + m, y) * grad_at(rows[up->members[lo + m]], grad_dtype, j);
            sumsq += gbar * gbar;
        }
        norms_out[u] = sqrt(sumsq);
    }
    return 0;
}

/*
 * Aggregation without the optimizer step (the sum a parent forms from its
 * children's gradients and its own in the all-reduce architecture, Section 4.2;
 * the sum a tree node forwards upward, Section 4.4.2):
 *     out[u*P + j] = sum over listed members m of coef(u,m) * g_member[j].
 * norms_out (may be NULL) receives || out_u ||_2.
 */
int oracle_group_reduce(double *out, const void *const *rows, int grad_dtype, int64_t P, int32_t W,
                        const oracle_updates *up, int32_t wmode, double *norms_out)
{
    int rc = check_stream(up, W);
    if (rc) return rc;
    for (int32_t u = 0; u < up->U; ++u) {
        const int32_t lo = up->offsets[u];
        const int32_t y = up->offsets[u + 1] - lo;
        double sumsq = 0.0;
        for (int64_t j = 0; j < P; ++j) {
            double gbar = 0.0;
            for (int32_t m = 0; m < y; ++m)
                gbar += member_coef(up, wmode, lo + m, y) * grad_at(rows[up->members[lo + m]], grad_dtype, j);
            out[(int64_t)u * P + j] = gbar;
            sumsq += gbar * gbar;
        }
        if (norms_out) norms_out[u] = sqrt(sumsq);
    }
    return 0;
}

/*
 * Gram matrix of the gradient rows: out[a*W + b] = sum_j g_a[j] g_b[j].  The
 * squared norm of any weighted sum of rows is the quadratic form of its
 * coefficients in this matrix; it also feeds the noise-scale estimate (the
 * gradient-norm signal of Sections 4.3.1 and 7).
 */
int oracle_gram(double *out, const void *const *rows, int grad_dtype, int64_t P, int32_t W)
{
    for (int32_t a = 0; a < W; ++a)
        for (int32_t b = 0; b < W; ++b) {
            double s = 0.0;
            for (int64_t j = 0; j < P; ++j)
                s += grad_at(rows[a], grad_dtype, j) * grad_at(rows[b], grad_dtype, j);
            out[(int64_t)a * W + b] = s;
        }
    return 0;
}

/*
 * Stepwise-fp32 mode: what a literal fp32 parameter server produces.  Every
 * product and sum is rounded to fp32 (this file is compiled with
 * -ffp-contract=off, so no fused multiply-add), members are taken in
 * ascending worker id, state is fp32 after every update.  Used to report how
 * far a plain fp32 server sits from the exact result, and as the timed CPU
 * baseline; parity is judged against the exact mode above.
 */
int oracle_group_update_f32step(float *params, float *momentum, const void *const *rows, int grad_dtype,
                                int64_t P, int32_t W, const oracle_updates *up, const oracle_hparams *hp,
                                double *norms_out)
{
    int rc = check_stream(up, W);
    if (rc) return rc;
    if (W > 64) return 2;
    const float mu = hp->momentum, wd = hp->weight_decay;
    for (int32_t u = 0; u < up->U; ++u) {
        const int32_t lo = up->offsets[u];
        const int32_t y = up->offsets[u + 1] - lo;
        const float lr = (float)update_lr(up, hp, u, y, W);
        float c[64];
        int present[64];
        for (int32_t w = 0; w < W; ++w) present[w] = 0;
        for (int32_t m = 0; m < y; ++m) {
            c[up->members[lo + m]] = (float)member_coef(up, hp->wmode, lo + m, y);
            present[up->members[lo + m]] = 1;
        }
        double sumsq = 0.0;
        for (int64_t j = 0; j < P; ++j) {
            float gbar = 0.0f;
            for (int32_t w = 0; w < W; ++w)
                if (present[w]) gbar = gbar + c[w] * (float)grad_at(rows[w], grad_dtype, j);
            sumsq += (double)gbar * (double)gbar;
            float d = gbar + wd * params[j];
            momentum[j] = mu * momentum[j] + d;
            params[j] = params[j] - lr * momentum[j];
        }
        if (norms_out) norms_out[u] = sqrt(sumsq);
    }
    return 0;
}
