/*
 * CPU oracle for the BiGLA token mixer and the 2D gating locality injection.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 statement of
 * what the hot path computes.  It shares no code with the HIP library and is
 * linked, loaded or executed only by the tests, the smoke check and the
 * cpu_baseline leg of the benchmark.
 *
 * Every routine is the paper's definition written out directly:
 *   - bigla_ref_f64         : the two recurrences of Eq. (BiGLA), Section 4.2.1,
 *                             run token by token, then averaged.
 *   - locality_gate_ref_f64 : Section 4.2.2 (depthwise 3x3 convolution on the
 *                             patch grid, sigmoid gate, convex blend).
 *   - gate_producer_ref_f64 : the direction-wise forget gates, first two lines
 *                             of Eq. (BiGLA) with the low-rank gate of Section 3,
 *                             returned as log-gates.
 *   - bigla_bwd_ref_f64     : the gradient of bigla_ref_f64 with respect to all five
 *                             inputs, by the chain rule on the same two recurrences
 *                             (the paper trains through them, Section 5, but prints no
 *                             gradient formulas): adjoint states run against each
 *                             recurrence's direction.
 * No blocking, chunking, fusion or reordering is applied.
 *
 * Pins (tests/test_oracle_pins.py): explicit-product quadratic form by brute
 * force, the all-gates-one reduction to plain bidirectional linear attention,
 * the closed forms for vanishing and constant gates, the reversal symmetry,
 * the kill-one-direction causal check, trilinearity, a hand-worked L=2 case,
 * and for the convolution a library conv2d plus closed-form kernels; for the
 * gradient, central finite differences of bigla_ref_f64 in all five inputs and the
 * closed forms of the gates-closed and gates-open limits.
 *
 * Layout everywhere: dense row-major, innermost index = feature.
 *   q, k, g_fwd, g_bwd : [B, H, L, dk]      v, out : [B, H, L, dv]
 * g_* are LOG gates: alpha = exp(g) in (0, 1].
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* One (batch, head) slab.  S is a dk x dv scratch matrix, o_dir an L x dv scratch. */
static void bigla_slab(const double *q, const double *k, const double *v,
                       const double *g_fwd, const double *g_bwd, double *out,
                       int L, int dk, int dv, double *S, double *o_fwd)
{
    /* forward direction: S_t = diag(alpha_fwd_t) S_{t-1} + k_t^T v_t ; o_t = q_t S_t */
    memset(S, 0, sizeof(double) * (size_t)dk * dv);
    for (int t = 0; t < L; ++t) {
        for (int c = 0; c < dk; ++c) {
            const double alpha = exp(g_fwd[(size_t)t * dk + c]);
            const double kc = k[(size_t)t * dk + c];
            for (int j = 0; j < dv; ++j)
                S[(size_t)c * dv + j] = alpha * S[(size_t)c * dv + j] + kc * v[(size_t)t * dv + j];
        }
        for (int j = 0; j < dv; ++j) {
            double acc = 0.0;
            for (int c = 0; c < dk; ++c)
                acc += q[(size_t)t * dk + c] * S[(size_t)c * dv + j];
            o_fwd[(size_t)t * dv + j] = acc;
        }
    }
    /* backward direction: S_t = diag(alpha_bwd_t) S_{t+1} + k_t^T v_t ; o_t = q_t S_t */
    memset(S, 0, sizeof(double) * (size_t)dk * dv);
    for (int t = L - 1; t >= 0; --t) {
        for (int c = 0; c < dk; ++c) {
            const double alpha = exp(g_bwd[(size_t)t * dk + c]);
            const double kc = k[(size_t)t * dk + c];
            for (int j = 0; j < dv; ++j)
                S[(size_t)c * dv + j] = alpha * S[(size_t)c * dv + j] + kc * v[(size_t)t * dv + j];
        }
        for (int j = 0; j < dv; ++j) {
            double acc = 0.0;
            for (int c = 0; c < dk; ++c)
                acc += q[(size_t)t * dk + c] * S[(size_t)c * dv + j];
            /* o_t = (o_fwd_t + o_bwd_t) / 2 */
            out[(size_t)t * dv + j] = 0.5 * (o_fwd[(size_t)t * dv + j] + acc);
        }
    }
}

/*
 * BiGLA forward, Section 4.2.1, Eq. (BiGLA).  Both states start from zero
 * (before the first token for the forward scan, after the last token for the
 * backward scan).  Returns 0, or -1 on a bad argument / allocation failure.
 * nthreads <= 0 means "all cores"; slabs (b, h) are independent units.
 */
int bigla_ref_f64(const double *q, const double *k, const double *v,
                  const double *g_fwd, const double *g_bwd, double *out,
                  int B, int H, int L, int dk, int dv, int nthreads)
{
    if (!q || !k || !v || !g_fwd || !g_bwd || !out) return -1;
    if (B <= 0 || H <= 0 || L <= 0 || dk <= 0 || dv <= 0) return -1;
    const long slabs = (long)B * H;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *S = (double *)malloc(sizeof(double) * (size_t)dk * dv);
        double *of = (double *)malloc(sizeof(double) * (size_t)L * dv);
        if (!S || !of) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        } else {
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
            for (long s = 0; s < slabs; ++s) {
                const size_t ok = (size_t)s * L * dk, ov = (size_t)s * L * dv;
                bigla_slab(q + ok, k + ok, v + ov, g_fwd + ok, g_bwd + ok, out + ov, L, dk, dv, S, of);
            }
        }
        free(S);
        free(of);
    }
    return failed ? -1 : 0;
}

/*
 * Gradient of one direction of one slab.  With s_t the state column of value dimension j
 * (s_t = alpha_t * s_{t-1} + k_t v_t[j], walking in direction `step` = +1 or -1 from the
 * direction's first token) and o_t[j] = q_t . s_t, the adjoint of s_t is
 *     a_t = q_t do_t[j] + alpha_{t+step} * a_{t+step}        (zero beyond the last token)
 * and the chain rule gives
 *     dq_t += s_t do_t[j],  dk_t += a_t v_t[j],  dv_t[j] += k_t . a_t,
 *     dalpha_t += a_t * s_{t-step}  (nothing before the first token),  dg_t = alpha_t dalpha_t.
 * do = d_out / 2 (the average of the two directions).  Columns j are independent, so the states
 * of one column at every token (L x dk) are kept and the adjoint runs back over them.
 */
static void bigla_bwd_direction(const double *q, const double *k, const double *v, const double *g,
                                const double *d_out, double *dq, double *dk_, double *dv_, double *dg,
                                int L, int dk, int dv, int step, double *states, double *a, double *dalpha)
{
    const int first = step > 0 ? 0 : L - 1;
    memset(dalpha, 0, sizeof(double) * (size_t)L * dk);
    for (int j = 0; j < dv; ++j) {
        /* states of column j at every token */
        for (int n = 0; n < L; ++n) {
            const int t = first + n * step;
            for (int c = 0; c < dk; ++c) {
                const double prev = n == 0 ? 0.0 : states[(size_t)(t - step) * dk + c];
                states[(size_t)t * dk + c] = exp(g[(size_t)t * dk + c]) * prev + k[(size_t)t * dk + c] * v[(size_t)t * dv + j];
            }
        }
        /* adjoint, from the direction's last token back to its first */
        for (int c = 0; c < dk; ++c) a[c] = 0.0;
        for (int n = L - 1; n >= 0; --n) {
            const int t = first + n * step;
            const double dot = 0.5 * d_out[(size_t)t * dv + j];
            double kv = 0.0;
            for (int c = 0; c < dk; ++c) {
                const double decay = n == L - 1 ? 0.0 : exp(g[(size_t)(t + step) * dk + c]);
                a[c] = q[(size_t)t * dk + c] * dot + decay * a[c];
                dq[(size_t)t * dk + c] += states[(size_t)t * dk + c] * dot;
                dk_[(size_t)t * dk + c] += a[c] * v[(size_t)t * dv + j];
                kv += k[(size_t)t * dk + c] * a[c];
                if (n > 0) dalpha[(size_t)t * dk + c] += a[c] * states[(size_t)(t - step) * dk + c];
            }
            dv_[(size_t)t * dv + j] += kv;
        }
    }
    for (size_t i = 0; i < (size_t)L * dk; ++i) dg[i] = exp(g[i]) * dalpha[i];
}

/*
 * BiGLA backward: given d_out = dLoss/d_out [B,H,L,dv], the gradients of the loss with respect
 * to q, k, g_fwd, g_bwd [B,H,L,dk] and v [B,H,L,dv] of bigla_ref_f64.  Returns 0, or -1 on a bad
 * argument / allocation failure.
 */
int bigla_bwd_ref_f64(const double *q, const double *k, const double *v, const double *g_fwd,
                      const double *g_bwd, const double *d_out, double *dq, double *dk_, double *dv_,
                      double *dg_fwd, double *dg_bwd, int B, int H, int L, int dk, int dv, int nthreads)
{
    if (!q || !k || !v || !g_fwd || !g_bwd || !d_out || !dq || !dk_ || !dv_ || !dg_fwd || !dg_bwd) return -1;
    if (B <= 0 || H <= 0 || L <= 0 || dk <= 0 || dv <= 0) return -1;
    const long slabs = (long)B * H;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel num_threads(nthreads)
#endif
    {
        double *states = (double *)malloc(sizeof(double) * (size_t)L * dk);
        double *dalpha = (double *)malloc(sizeof(double) * (size_t)L * dk);
        double *a = (double *)malloc(sizeof(double) * (size_t)dk);
        if (!states || !dalpha || !a) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        } else {
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
            for (long s = 0; s < slabs; ++s) {
                const size_t ok = (size_t)s * L * dk, ov = (size_t)s * L * dv;
                memset(dq + ok, 0, sizeof(double) * (size_t)L * dk);
                memset(dk_ + ok, 0, sizeof(double) * (size_t)L * dk);
                memset(dv_ + ov, 0, sizeof(double) * (size_t)L * dv);
                bigla_bwd_direction(q + ok, k + ok, v + ov, g_fwd + ok, d_out + ov, dq + ok, dk_ + ok, dv_ + ov,
                                    dg_fwd + ok, L, dk, dv, +1, states, a, dalpha);
                bigla_bwd_direction(q + ok, k + ok, v + ov, g_bwd + ok, d_out + ov, dq + ok, dk_ + ok, dv_ + ov,
                                    dg_bwd + ok, L, dk, dv, -1, states, a, dalpha);
            }
        }
        free(states);
        free(dalpha);
        free(a);
    }
    return failed ? -1 : 0;
}

/* Number of threads bigla_ref_f64 / locality_gate_ref_f64 use for nthreads <= 0. */
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * 2D gating locality injection, Section 4.2.2:
 *   O_local = DWConv3x3(X)              (stride 1, zero padding 1, cross-correlation,
 *                                        one 3x3 filter per channel c = h*dv + j)
 *   G       = sigmoid(z)
 *   O       = G * O_local + (1 - G) * O_global
 * x, z, o_global, out : [B, H, Hg*Wg, dv] with token index t = y*Wg + x_pos;
 * w : [H*dv, 3, 3]; bias : [H*dv] or NULL.
 */
int locality_gate_ref_f64(const double *x, const double *w, const double *bias,
                          const double *z, const double *o_global, double *out,
                          int B, int H, int Hg, int Wg, int dv, int nthreads)
{
    if (!x || !w || !z || !o_global || !out) return -1;
    if (B <= 0 || H <= 0 || Hg <= 0 || Wg <= 0 || dv <= 0) return -1;
    const long slabs = (long)B * H;
    const int L = Hg * Wg;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (long s = 0; s < slabs; ++s) {
        const int h = (int)(s % H);
        const size_t base = (size_t)s * L * dv;
        for (int y = 0; y < Hg; ++y)
            for (int xp = 0; xp < Wg; ++xp)
                for (int j = 0; j < dv; ++j) {
                    const int c = h * dv + j;
                    double local = bias ? bias[c] : 0.0;
                    for (int dy = -1; dy <= 1; ++dy)
                        for (int dx = -1; dx <= 1; ++dx) {
                            const int yy = y + dy, xx = xp + dx;
                            if (yy < 0 || yy >= Hg || xx < 0 || xx >= Wg) continue; /* zero pad */
                            local += w[(size_t)c * 9 + (dy + 1) * 3 + (dx + 1)] *
                                     x[base + ((size_t)yy * Wg + xx) * dv + j];
                        }
                    const size_t o = base + ((size_t)y * Wg + xp) * dv + j;
                    const double gate = 1.0 / (1.0 + exp(-z[o]));
                    out[o] = gate * local + (1.0 - gate) * o_global[o];
                }
    }
    return 0;
}

/* log(sigmoid(z)) without overflow: min(z, 0) - log(1 + exp(-|z|)), the same function. */
static double log_sigmoid(double z)
{
    return (z < 0.0 ? z : 0.0) - log1p(exp(-fabs(z)));
}

/*
 * Direction-wise forget gates, Eq. (BiGLA) lines 1-2 (Section 4.2.1) with the low-rank gate of
 * Section 3:
 *   z_t     = (x_t W1) W2 + b               in R^{2*H*dk}
 *   alpha_t = sigmoid(z_t)^(1/tau)
 *   split   : entries [0, H*dk) are the forward gates, [H*dk, 2*H*dk) the backward gates;
 *             inside each half head h owns entries [h*dk, (h+1)*dk)
 * Returned as LOG gates g = log(alpha) = log(sigmoid(z)) / tau  (<= 0).
 *   x : [B, L, D]   w1 : [D, rank]   w2 : [rank, 2*H*dk]   bias : [2*H*dk] or NULL
 *   g_fwd, g_bwd : [B, H, L, dk]
 * The product is evaluated in the printed order: first the rank-wide x_t W1, then times W2.
 */
int gate_producer_ref_f64(const double *x, const double *w1, const double *w2, const double *bias,
                          double *g_fwd, double *g_bwd, int B, int H, int L, int D, int rank, int dk,
                          double tau, int nthreads)
{
    if (!x || !w1 || !w2 || !g_fwd || !g_bwd) return -1;
    if (B <= 0 || H <= 0 || L <= 0 || D <= 0 || rank <= 0 || dk <= 0 || !(tau > 0.0)) return -1;
    const long tokens = (long)B * L;
    const int half = H * dk, width = 2 * half;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel
#else
    (void)nthreads;
#endif
    {
        double *low = (double *)malloc(sizeof(double) * (size_t)rank);
        if (!low) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        } else {
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
            for (long n = 0; n < tokens; ++n) {
                const long b = n / L, t = n % L;
                const double *xt = x + (size_t)n * D;
                for (int r = 0; r < rank; ++r) {
                    double acc = 0.0;
                    for (int i = 0; i < D; ++i) acc += xt[i] * w1[(size_t)i * rank + r];
                    low[r] = acc;
                }
                for (int c = 0; c < width; ++c) {
                    double z = bias ? bias[c] : 0.0;
                    for (int r = 0; r < rank; ++r) z += low[r] * w2[(size_t)r * width + c];
                    const int dir = c / half, h = (c % half) / dk, j = c % dk;
                    double *g = dir == 0 ? g_fwd : g_bwd;
                    g[(((size_t)b * H + h) * L + t) * dk + j] = log_sigmoid(z) / tau;
                }
            }
        }
        free(low);
    }
    return failed ? -1 : 0;
}
