/*
 * CPU oracle for one batched Leader-SGD step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain statement of what the method computes, written
 * from the paper (arXiv 1905.10395).  It is used by the tests, by the smoke
 * check and by the CPU-baseline leg of the benchmark, and by nothing else.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Conventions
 *   - State (x, m, Z, g, losses) is stored in fp32, the same bytes the GPU
 *     holds.  Every sum, dot product and update expression is evaluated in
 *     fp64 and rounded once to fp32 where it is stored.
 *   - Workers are rows of x[W, ld]; group j owns rows [off[j], off[j+1]).
 *   - Z[(G+1), ld] holds the leader copies kept between communications
 *     (Algorithm 1, the leader variables set at initialisation and at each
 *     communication; supplement B.1, communication periods):
 *     rows 0..G-1 local leaders, row G the global leader.
 *
 * Pins (tests/test_oracle_*.py): zero pull coefficients reduce to SGD; the
 * leader's own pull vanishes; the affine form X+ = (1-eta*lam)X + eta*lam*Z -
 * eta*grad of the matrix-completion supplement; several leaders collapse to
 * one (Section 3, first paragraph); fixed-leader limit on a diagonal
 * quadratic and the bound of Theorem 2; monotone leader value (Lemma
 * "leader_descent"); the sinc example's optimum -0.2172 (supplement Table 1);
 * grad F = (XX^T - M)X for the dense PSD problem; finite differences;
 * brute-force argmin and hand-computed near-tie gaps; momentum together with
 * pulls against a library momentum-SGD fed the gradient of Eq. 2's objective
 * with the leader copies held fixed (and, for the grad-only mode, fed g alone
 * with the pulls as a plain step beside it), over stale periods; Algorithm
 * 1's communication pull as two successive single-leader interpolations;
 * window mean and column mean against numpy; the elastic-averaging comparison
 * method against its printed optimum on the sinc example (-0.0912), its
 * conserved sum, and the spurious stationary point of the supplement's
 * proposition on EASGD.
 *
 * Fixed by declaration, the paper being silent (the arithmetic of each choice
 * is pinned as above, the choice itself is not the paper's): that momentum is
 * heavy ball on the full direction by default, the bf16 rounding points of
 * the MLP workload, the loss normalisation c of the matrix-completion batch.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_NESTEROV            1
#define ORACLE_LEADER_EXEMPT       2
#define ORACLE_PULL_UNSCALED       4
#define ORACLE_MOMENTUM_GRAD_ONLY  8

/* ------------------------------------------------------------------ */
/* Leader selection: Eq. 1/2 argmin definitions; the steps of Algorithm 1
 * that pick the best worker of each group and of all groups.  Ties go to
 * the lowest index; NaN counts as +infinity.                            */
/* ------------------------------------------------------------------ */
static double sel_value(float v) { return isnan(v) ? INFINITY : (double)v; }

static void argmin_range(const float* losses, int lo, int hi, int32_t* idx, double* gap)
{
    int best = lo;
    double bv = sel_value(losses[lo]);
    for (int i = lo + 1; i < hi; ++i) {
        double v = sel_value(losses[i]);
        if (v < bv) { bv = v; best = i; }
    }
    *idx = best;
    if (gap) {
        double second = INFINITY;
        for (int i = lo; i < hi; ++i)
            if (i != best) { double v = sel_value(losses[i]); if (v < second) second = v; }
        if (second == bv) *gap = 0.0;                          /* a tie, also between infinities          */
        else if (isinf(second) || isinf(bv)) *gap = INFINITY;  /* no finite runner-up, or a best of -inf  */
        else { double den = fabs(bv) > 1e-30 ? fabs(bv) : 1e-30; *gap = (second - bv) / den; }
    }
}

/* lead[G], glead[1] are updated only for refreshed groups / a global refresh.
 * gaps (optional, [G+1]) receives (second best - best)/|best| per refreshed
 * selection, used by tests to detect legitimate near-ties.             */
void lsgd_oracle_select_leaders(const float* losses, int W, int G, const int32_t* off,
                                const uint8_t* refresh_local, int refresh_global,
                                int32_t* lead, int32_t* glead, double* gaps)
{
    for (int j = 0; j < G; ++j) {
        if (refresh_local && !refresh_local[j]) continue;
        argmin_range(losses, off[j], off[j + 1], &lead[j], gaps ? &gaps[j] : 0);
    }
    if (refresh_global) argmin_range(losses, 0, W, glead, gaps ? &gaps[G] : 0);
}

/* ------------------------------------------------------------------ */
/* Pull update.  Supplement B.1: x+ = x - eta*(g + lam*(x - z)); with two
 * leaders (Eq. 2 / Eq. 3) the pulls add.  Leader copies are taken from
 * the pre-update parameters at a refresh, kept otherwise.              */
/* ------------------------------------------------------------------ */
void lsgd_oracle_pull_update(float* x, float* m, const float* g, float* Z,
                             int W, int64_t P, int64_t ld, int G, const int32_t* off,
                             const int32_t* lead, int32_t glead,
                             const uint8_t* refresh_local, int refresh_global,
                             float eta_f, float lamL_f, float lamG_f, float mu_f,
                             int flags, float wd_f)
{
    const double eta = eta_f, mu = mu_f, wd = wd_f;
    double lamL = lamL_f, lamG = lamG_f;
    if (flags & ORACLE_PULL_UNSCALED) { lamL = lamL / eta; lamG = lamG / eta; } /* Eq. 3 as printed */

    /* step 2: copy the selected leaders' current parameters */
    for (int j = 0; j < G; ++j)
        if (lamL_f != 0.0f && (!refresh_local || refresh_local[j]))
            memcpy(Z + (int64_t)j * ld, x + (int64_t)lead[j] * ld, sizeof(float) * (size_t)P);
    if (lamG_f != 0.0f && refresh_global)
        memcpy(Z + (int64_t)G * ld, x + (int64_t)glead * ld, sizeof(float) * (size_t)P);

    /* step 3: every worker moves, all from pre-update values (Z holds the leaders') */
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < W; ++i) {
        int j = 0;
        while (!(off[j] <= i && i < off[j + 1])) ++j;
        double cL = lamL, cG = lamG;
        if (flags & ORACLE_LEADER_EXEMPT) {
            if (i == lead[j]) cL = 0.0;
            if (i == glead) cG = 0.0;
        }
        const float* zL = Z + (int64_t)j * ld;
        const float* zG = Z + (int64_t)G * ld;
        float* xi = x + (int64_t)i * ld;
        float* mi = m ? m + (int64_t)i * ld : 0;
        const float* gi = g + (int64_t)i * ld;
        for (int64_t p = 0; p < P; ++p) {
            double xv = xi[p];
            double gv = gi[p];
            if (wd_f != 0.0f) gv += wd * xv;
            double pull = 0.0;
            if (lamL_f != 0.0f) pull += cL * (xv - (double)zL[p]);
            if (lamG_f != 0.0f) pull += cG * (xv - (double)zG[p]);
            double step;
            if (mu_f == 0.0f) {
                step = gv + pull;
            } else if (flags & ORACLE_MOMENTUM_GRAD_ONLY) {
                double mv = mu * (double)mi[p] + gv;
                mi[p] = (float)mv;
                mv = (double)mi[p];
                step = ((flags & ORACLE_NESTEROV) ? gv + mu * mv : mv) + pull;
            } else {
                double d = gv + pull;
                double mv = mu * (double)mi[p] + d;
                mi[p] = (float)mv;
                mv = (double)mi[p];
                step = (flags & ORACLE_NESTEROV) ? d + mu * mv : mv;
            }
            xi[p] = (float)(xv - eta * step);
        }
    }
}

/* ------------------------------------------------------------------ */
/* Communication step of Algorithm 1: after re-selecting leaders, every worker
 * of a re-selected group is pulled to its local leader, x <- x - lam (x - x~^j),
 * and at a global communication to the global leader, x <- x - lam_G (x - x~).
 * No gradient, no learning rate, momentum untouched.  Both pulls use the
 * leaders' parameters as they were when selected (copied to Z first); a
 * leader's pull to itself is zero.                                      */
/* ------------------------------------------------------------------ */
void lsgd_oracle_leader_pull(float* x, float* Z, int W, int64_t P, int64_t ld, int G, const int32_t* off,
                             const int32_t* lead, int32_t glead, const uint8_t* refresh_local, int refresh_global,
                             float lamL_f, float lamG_f)
{
    for (int j = 0; j < G; ++j)
        if (!refresh_local || refresh_local[j])
            memcpy(Z + (int64_t)j * ld, x + (int64_t)lead[j] * ld, sizeof(float) * (size_t)P);
    if (refresh_global)
        memcpy(Z + (int64_t)G * ld, x + (int64_t)glead * ld, sizeof(float) * (size_t)P);
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < W; ++i) {
        int j = 0;
        while (!(off[j] <= i && i < off[j + 1])) ++j;
        const double cL = (!refresh_local || refresh_local[j]) ? (double)lamL_f : 0.0;
        const double cG = refresh_global ? (double)lamG_f : 0.0;
        const float* zL = Z + (int64_t)j * ld;
        const float* zG = Z + (int64_t)G * ld;
        float* xi = x + (int64_t)i * ld;
        for (int64_t p = 0; p < P; ++p) {
            double y = (double)xi[p];
            if (cL != 0.0) y = y - cL * (y - (double)zL[p]);
            if (cG != 0.0) y = y - cG * (y - (double)zG[p]);
            xi[p] = (float)y;
        }
    }
}

/* Selection loss smoothed over the last K minibatches (Section 4.1: the leader is
 * chosen from the average training loss over the last 10 / 64 batches).
 * window[K][W] is a ring: slot t % K receives the new losses; out = mean of
 * the min(t+1, K) newest slots.                                          */
void lsgd_oracle_smooth_losses(float* window, int K, int64_t t, const float* losses, int W, float* out)
{
    memcpy(window + (t % K) * W, losses, sizeof(float) * (size_t)W);
    const int64_t n = (t + 1 < K) ? t + 1 : K;
    for (int i = 0; i < W; ++i) {
        double s = 0.0;
        for (int64_t q = 0; q < n; ++q) s += (double)window[q * W + i];
        out[i] = (float)(s / (double)n);
    }
}

/* Center variable reported at test time (Section 4.1): the average of all workers' parameters. */
void lsgd_oracle_center(const float* x, int W, int64_t P, int64_t ld, float* out)
{
    for (int64_t p = 0; p < P; ++p) {
        double s = 0.0;
        for (int i = 0; i < W; ++i) s += (double)x[(int64_t)i * ld + p];
        out[p] = (float)(s / (double)W);
    }
}

/* Elastic averaging (EAGD / EASGD), the method the paper compares with, in the form the supplement
 * writes it beside LGD ("Low-Rank Matrix Completion Experiments"): every worker takes the same pulled
 * step with the center in the leader's place, X+ = (1 - eta lam) X + eta lam Xc - eta grad, i.e.
 * lsgd_oracle_pull_update with Z's global row holding the center and no local term; and the center
 * moves to   Xc+ = (1 - p eta lam) Xc + p eta lam * (1/p) sum_i X^i   with p = W workers.
 * Both formulas are read at the same time step: the mean is over the workers' parameters BEFORE
 * their own update, so this function runs first (it only changes the center).  The pre-update
 * center is returned in old_center for the workers' step.                                    */
void lsgd_oracle_easgd_center(const float* x, int W, int64_t P, int64_t ld, float* center, float* old_center,
                              float eta_f, float lam_f)
{
    const double a = (double)W * (double)eta_f * (double)lam_f;
    for (int64_t p = 0; p < P; ++p) {
        double s = 0.0;
        for (int i = 0; i < W; ++i) s += (double)x[(int64_t)i * ld + p];
        const double mean = s / (double)W;
        const double c = (double)center[p];
        old_center[p] = center[p];
        center[p] = (float)((1.0 - a) * c + a * mean);
    }
}

/* ------------------------------------------------------------------ */
/* Matrix completion on observed entries.  Worker row = [U (m x r) | V (n x r)],
 * both row-major.  For batch entries k with (a_k, b_k, M_k):
 *   e_k = <U[a_k], V[b_k]> - M_k ; loss = c * sum e_k^2 ;
 *   dU[a] = 2c * sum_{k: a_k=a} e_k V[b_k] ; dV[b] = 2c * sum_{k: b_k=b} e_k U[a_k].
 * With every entry observed, U = V = X and c = 1/2 ... the problem family of
 * the supplement's "Low-Rank Matrix Completion Experiments".           */
/* ------------------------------------------------------------------ */
void lsgd_oracle_mc_grad_loss(const float* x, int W, int64_t ld, int m, int n, int r,
                              const int32_t* rows, const int32_t* cols, const float* vals,
                              int64_t n_obs, const int32_t* batch_idx, int64_t B, float c_f,
                              float* g, float* losses)
{
    const int64_t P = (int64_t)(m + n) * r;
    const double c = c_f;
    const int64_t nb = batch_idx ? B : n_obs;
    #pragma omp parallel for schedule(static)
    for (int i = 0; i < W; ++i) {
        const float* U = x + (int64_t)i * ld;
        const float* V = U + (int64_t)m * r;
        double* acc = (double*)calloc((size_t)P, sizeof(double));
        double* aU = acc;
        double* aV = acc + (int64_t)m * r;
        double loss = 0.0;
        for (int64_t k = 0; k < nb; ++k) {
            int64_t s = batch_idx ? batch_idx[(int64_t)i * B + k] : k;
            int a = rows[s], b = cols[s];
            double dot = 0.0;
            for (int q = 0; q < r; ++q) dot += (double)U[(int64_t)a * r + q] * (double)V[(int64_t)b * r + q];
            double e = dot - (double)vals[s];
            loss += e * e;
            for (int q = 0; q < r; ++q) {
                aU[(int64_t)a * r + q] += e * (double)V[(int64_t)b * r + q];
                aV[(int64_t)b * r + q] += e * (double)U[(int64_t)a * r + q];
            }
        }
        float* gi = g + (int64_t)i * ld;
        for (int64_t p = 0; p < P; ++p) gi[p] = (float)(2.0 * c * acc[p]);
        for (int64_t p = P; p < ld; ++p) gi[p] = 0.0f;
        losses[i] = (float)(c * loss);
        free(acc);
    }
}

/* ------------------------------------------------------------------ */
/* MLP classifier, softmax cross-entropy, mixed precision.
 * Worker row = [W_1 (d1 x d0 row-major) | b_1 | W_2 | b_2 | ...].
 * Rounding points (round-to-nearest-even to bf16): the inputs X (already
 * stored as bf16), weight operands, stored activations h_k = relu(z_k), and
 * back-propagated deltas used as matrix operands.  Biases, logits, softmax,
 * loss, dW, db stay fp32 (fp64 accumulation here).                     */
/* ------------------------------------------------------------------ */
static float bf16_round(float v)
{
    uint32_t u; memcpy(&u, &v, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return v;           /* inf / nan unchanged */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    u &= 0xFFFF0000u;
    float o; memcpy(&o, &u, 4);
    return o;
}
static float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16; float o; memcpy(&o, &u, 4); return o;
}

/* min_abs_preact (optional, [W, B]): for every sample the smallest |z| over all hidden units of all hidden
 * layers, i.e. how far the sample is from switching a ReLU mask.  A by-product of the forward pass for the
 * tests; it takes no part in the arithmetic.
 * Threads: over workers when there are at least as many workers as threads, otherwise over the independent
 * outputs inside one worker (batch rows, or weight rows for dW); every sum keeps its order either way.   */
void lsgd_oracle_mlp_grad_loss(const float* x, int W, int64_t ld, int n_layers, const int32_t* dims,
                               const uint16_t* X, const int32_t* y, int B,
                               float* g, float* losses, float* min_abs_preact)
{
    const int L = n_layers;
    int64_t P = 0;
    for (int k = 0; k < L; ++k) P += (int64_t)dims[k + 1] * dims[k] + dims[k + 1];
    const int over_workers = W >= omp_get_max_threads();

    #pragma omp parallel for schedule(dynamic, 1) if(over_workers)
    for (int i = 0; i < W; ++i) {
        const float* xi = x + (int64_t)i * ld;
        float* gi = g + (int64_t)i * ld;
        /* per-layer buffers */
        float** Wq = (float**)malloc(sizeof(float*) * L);     /* bf16-rounded weights  */
        const float** bias = (const float**)malloc(sizeof(float*) * L);
        float** h = (float**)malloc(sizeof(float*) * (L + 1)); /* h[0]=input, h[k] bf16 activations */
        float** z = (float**)malloc(sizeof(float*) * (L + 1)); /* fp32 pre-activations  */
        int64_t* woff = (int64_t*)malloc(sizeof(int64_t) * L);
        int64_t o = 0;
        for (int k = 0; k < L; ++k) {
            int64_t nw = (int64_t)dims[k + 1] * dims[k];
            woff[k] = o;
            Wq[k] = (float*)malloc(sizeof(float) * nw);
            for (int64_t t = 0; t < nw; ++t) Wq[k][t] = bf16_round(xi[o + t]);
            bias[k] = xi + o + nw;
            o += nw + dims[k + 1];
        }
        h[0] = (float*)malloc(sizeof(float) * (size_t)B * dims[0]);
        z[0] = 0;
        for (int64_t t = 0; t < (int64_t)B * dims[0]; ++t)
            h[0][t] = bf16_bits_to_float(X[(int64_t)i * B * dims[0] + t]);

        /* forward */
        for (int k = 0; k < L; ++k) {
            int din = dims[k], dout = dims[k + 1];
            z[k + 1] = (float*)malloc(sizeof(float) * (size_t)B * dout);
            h[k + 1] = (float*)malloc(sizeof(float) * (size_t)B * dout);
            #pragma omp parallel for schedule(static) if(!over_workers)
            for (int b = 0; b < B; ++b)
                for (int q = 0; q < dout; ++q) {
                    double acc = 0.0;
                    const float* hr = h[k] + (int64_t)b * din;
                    const float* wr = Wq[k] + (int64_t)q * din;
                    for (int p = 0; p < din; ++p) acc += (double)hr[p] * (double)wr[p];
                    float zz = (float)(acc + (double)bias[k][q]);
                    z[k + 1][(int64_t)b * dout + q] = zz;
                    h[k + 1][(int64_t)b * dout + q] = (k + 1 < L) ? bf16_round(zz > 0.0f ? zz : 0.0f) : zz;
                }
        }
        if (min_abs_preact)
            for (int b = 0; b < B; ++b) {
                float mn = INFINITY;
                for (int k = 1; k < L; ++k)
                    for (int q = 0; q < dims[k]; ++q) {
                        float a = fabsf(z[k][(int64_t)b * dims[k] + q]);
                        if (a < mn) mn = a;
                    }
                min_abs_preact[(int64_t)i * B + b] = mn;
            }
        /* loss and output delta */
        int C = dims[L];
        double loss = 0.0;
        float* delta = (float*)malloc(sizeof(float) * (size_t)B * C);
        for (int b = 0; b < B; ++b) {
            const float* lg = z[L] + (int64_t)b * C;
            double mx = lg[0];
            for (int q = 1; q < C; ++q) if ((double)lg[q] > mx) mx = lg[q];
            double se = 0.0;
            for (int q = 0; q < C; ++q) se += exp((double)lg[q] - mx);
            double lse = mx + log(se);
            int yb = y[(int64_t)i * B + b];
            loss += lse - (double)lg[yb];
            for (int q = 0; q < C; ++q) {
                double pq = exp((double)lg[q] - lse);
                double d = (pq - (q == yb ? 1.0 : 0.0)) / (double)B;
                delta[(int64_t)b * C + q] = bf16_round((float)d);
            }
        }
        losses[i] = (float)(loss / (double)B);

        /* backward */
        for (int k = L - 1; k >= 0; --k) {
            int din = dims[k], dout = dims[k + 1];
            int64_t nw = (int64_t)din * dout;
            double* acc = (double*)calloc((size_t)nw, sizeof(double));
            double* accb = (double*)calloc((size_t)dout, sizeof(double));
            /* dW[q][p] = sum_b delta[b][q] h[b][p], db[q] = sum_b delta[b][q]; b ascending in every sum */
            #pragma omp parallel for schedule(static) if(!over_workers)
            for (int q = 0; q < dout; ++q) {
                double* ar = acc + (int64_t)q * din;
                for (int b = 0; b < B; ++b) {
                    double d = delta[(int64_t)b * dout + q];
                    accb[q] += d;
                    if (d == 0.0) continue;
                    const float* hr = h[k] + (int64_t)b * din;
                    for (int p = 0; p < din; ++p) ar[p] += d * (double)hr[p];
                }
            }
            for (int64_t t = 0; t < nw; ++t) gi[woff[k] + t] = (float)acc[t];
            for (int q = 0; q < dout; ++q) gi[woff[k] + nw + q] = (float)accb[q];
            free(acc); free(accb);
            if (k > 0) {
                float* nd = (float*)malloc(sizeof(float) * (size_t)B * din);
                #pragma omp parallel for schedule(static) if(!over_workers)
                for (int b = 0; b < B; ++b)
                    for (int p = 0; p < din; ++p) {
                        double s = 0.0;
                        for (int q = 0; q < dout; ++q)
                            s += (double)delta[(int64_t)b * dout + q] * (double)Wq[k][(int64_t)q * din + p];
                        float sv = (float)s;
                        nd[(int64_t)b * din + p] = (z[k][(int64_t)b * din + p] > 0.0f) ? bf16_round(sv) : 0.0f;
                    }
                free(delta);
                delta = nd;
            }
        }
        for (int64_t p = P; p < ld; ++p) gi[p] = 0.0f;
        free(delta);
        for (int k = 0; k < L; ++k) free(Wq[k]);
        for (int k = 0; k <= L; ++k) { free(h[k]); if (z[k]) free(z[k]); }
        free(Wq); free(bias); free(h); free(z); free(woff);
    }
}

/* Loss only (forward pass in the same arithmetic), for finite-difference pins
 * on a model whose weights/activations are exactly bf16-representable.   */
float lsgd_oracle_bf16_round(float v) { return bf16_round(v); }
