/*
 * Rodimus DDTS recurrence -- fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the GPU library must compute.  Nothing in the product path may call,
 * link or import it; only tests/, the smoke check and the benchmark's
 * "cpu_baseline" leg do.  It shares no code with the HIP kernels.
 *
 * What it computes (paper, Sec. 3.1.3 "The Overall Rodimus Block", the state
 * recurrence of the block, with the general gated transition of Sec. 3.1.1 in
 * its second, factored form and the value-side transition gate fixed to one):
 *
 *     S_t = diag(alpha_t) S_{t-1} + (k_t)^T (beta_t .* v_t),   o_t = q_t S_t
 *
 * per (batch b, head h) independently, t = 1..T, S_0 given (or zero), with
 * alpha_t = exp(log_alpha_t) a 1 x dk row acting on the rows of the dk x dv
 * state, beta_t a 1 x dv input gate on the value, and the key-side input gate
 * (g^tau in the paper) already folded into k_t by the caller.  The output uses
 * the state AFTER the update, exactly as the recurrence is printed.  The
 * feed-through term of the block output (d_t .* x'_t) is outside this function.
 *
 * All arithmetic is IEEE double.  Inputs arrive as float: every bf16 and fp32
 * value the GPU receives is exactly representable in float, so the oracle sees
 * the same numbers the GPU sees and input rounding is not counted as error.
 *
 * Layouts (innermost index contiguous):
 *     q, k, log_alpha : [B, T, H, dk]      v, beta, o : [B, T, H, dv]
 *     S0, S_T         : [B, H, dk, dv]
 * The decode step uses the same layouts with T dropped ([N, H, ...]).
 *
 * The value gate may instead arrive as its pre-activation z_beta (flag
 * `beta_is_preactivation`): then beta_t = sigmoid(z_beta_t) (Sec. 3.1.2, the
 * input gate on the value side) is evaluated here in double, so that the
 * oracle again starts from the very bits the GPU receives.
 *
 * There is no blocking, fusion or reordering: the loops below are the
 * recurrence as written.  OpenMP only distributes the independent (b, h)
 * recurrences over host threads.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int rodimus_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double sigmoid_d(double z) { return z >= 0.0 ? 1.0 / (1.0 + exp(-z)) : exp(z) / (1.0 + exp(z)); }

/* One time step of one (b, h) recurrence, in place on S (dk x dv, row-major). */
static void ddts_update_general(double *S, const float *q, const float *k, const float *v,
                                const float *log_alpha, const float *log_beta_t, const float *beta, int beta_is_preactivation,
                                double *o, int dk, int dv, double *gated_v);

static void ddts_update(double *S, const float *q, const float *k, const float *v,
                        const float *log_alpha, const float *beta, int beta_is_preactivation,
                        double *o, int dk, int dv, double *gated_v)
{
    ddts_update_general(S, q, k, v, log_alpha, NULL, beta, beta_is_preactivation, o, dk, dv, gated_v);
}

/* The general gated transition of Sec. 3.1.1 (first equation of the section): the state is decayed along both of its
   dimensions, S_t = (alpha_t^T beta_t) .* S_{t-1} + k_t^T (beta_hat_t .* v_t), with beta_t = exp(log_beta_t) a 1 x dv row
   (log_beta_t == NULL: beta_t = 1, the choice the paper makes for the block). */
static void ddts_update_general(double *S, const float *q, const float *k, const float *v,
                                const float *log_alpha, const float *log_beta_t, const float *beta, int beta_is_preactivation,
                                double *o, int dk, int dv, double *gated_v)
{
    /* gated value: beta_t .* v_t   (beta == NULL means the all-ones gate;
       with the flag set the array holds z_beta and beta_t = sigmoid(z_beta_t)) */
    for (int j = 0; j < dv; ++j) {
        double gate = 1.0;
        if (beta) gate = beta_is_preactivation ? sigmoid_d((double)beta[j]) : (double)beta[j];
        gated_v[j] = gate * (double)v[j];
    }

    /* S_t = diag(alpha_t) S_{t-1} + k_t^T (beta_t .* v_t) */
    for (int r = 0; r < dk; ++r) {
        const double alpha = exp((double)log_alpha[r]);   /* exp(-inf) == 0 */
        const double kr = (double)k[r];
        double *Srow = S + (size_t)r * dv;
        for (int j = 0; j < dv; ++j) {
            const double decay = log_beta_t ? alpha * exp((double)log_beta_t[j]) : alpha;
            Srow[j] = decay * Srow[j] + kr * gated_v[j];
        }
    }

    /* o_t = q_t S_t  (the updated state) */
    for (int j = 0; j < dv; ++j) {
        double acc = 0.0;
        for (int r = 0; r < dk; ++r)
            acc += (double)q[r] * S[(size_t)r * dv + j];
        o[j] = acc;
    }
}

/*
 * Sequential scan over T tokens.
 *   beta may be NULL (all ones); S0 may be NULL (zero state); S_T may be NULL.
 *   beta_is_preactivation != 0: `beta` holds z_beta and the gate is sigmoid(z_beta).
 * Returns 0 on success, 1 on bad arguments, 2 on allocation failure.
 */
int rodimus_oracle_scan(const float *q, const float *k, const float *v,
                        const float *log_alpha, const float *beta,
                        const double *S0, double *o, double *S_T,
                        int B, int T, int H, int dk, int dv, int beta_is_preactivation)
{
    if (!q || !k || !v || !log_alpha || !o) return 1;
    if (B < 0 || T < 0 || H < 0 || dk <= 0 || dv <= 0) return 1;
    int failed = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *S = (double *)malloc(sizeof(double) * (size_t)dk * dv);
            double *gv = (double *)malloc(sizeof(double) * (size_t)dv);
            if (!S || !gv) {
                free(S); free(gv);
#pragma omp atomic write
                failed = 1;
                continue;
            }
            const size_t state_off = ((size_t)b * H + h) * (size_t)dk * dv;
            for (size_t e = 0; e < (size_t)dk * dv; ++e)
                S[e] = S0 ? S0[state_off + e] : 0.0;

            for (int t = 0; t < T; ++t) {
                const size_t row = ((size_t)b * T + t) * H + h;
                ddts_update(S, q + row * dk, k + row * dk, v + row * dv,
                            log_alpha + row * dk, beta ? beta + row * dv : NULL, beta_is_preactivation,
                            o + row * dv, dk, dv, gv);
            }
            if (S_T)
                for (size_t e = 0; e < (size_t)dk * dv; ++e)
                    S_T[state_off + e] = S[e];
            free(S); free(gv);
        }
    }
    return failed ? 2 : 0;
}

/*
 * One recurrent decode step for N independent sequences: S is updated in place
 * to S' and o = q S'.   Layouts [N, H, dk], [N, H, dv], S [N, H, dk, dv].
 */
int rodimus_oracle_step(const float *q, const float *k, const float *v,
                        const float *log_alpha, const float *beta,
                        double *S, double *o, int N, int H, int dk, int dv, int beta_is_preactivation)
{
    if (!q || !k || !v || !log_alpha || !S || !o) return 1;
    if (N < 0 || H < 0 || dk <= 0 || dv <= 0) return 1;
    int failed = 0;

#pragma omp parallel for schedule(static)
    for (long s = 0; s < (long)N * H; ++s) {
        double *gv = (double *)malloc(sizeof(double) * (size_t)dv);
        if (!gv) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        ddts_update(S + (size_t)s * dk * dv, q + (size_t)s * dk, k + (size_t)s * dk,
                    v + (size_t)s * dv, log_alpha + (size_t)s * dk,
                    beta ? beta + (size_t)s * dv : NULL, beta_is_preactivation, o + (size_t)s * dv, dk, dv, gv);
        free(gv);
    }
    return failed ? 2 : 0;
}

/*
 * DDTS gate front-end (paper Sec. 3.1.2 "Design of alpha, alpha-hat and beta-hat", and the pre-processing of
 * Sec. 3.1.3), row by row.  A row is one (token, head).  From the pre-activations z_g, z_tau (1 x dk) and z_beta
 * (1 x dv) and the raw q, k (1 x dk):
 *
 *     g         = softplus(z_g)                      selection gate
 *     tau       = sigmoid(z_tau)                     temperature gate
 *     log_alpha = -g .* tau                          (alpha = exp(-g .* tau), the decay gate)
 *     alpha_hat = g ^ tau                            input gate on the key side
 *     k_out     = alpha_hat .* k / max(||k||_2, eps) k normalised (L2 over the row, eps = 1e-12), gate folded in
 *     q_out     = q / sqrt(dk)
 *     beta      = sigmoid(z_beta)                    input gate on the value side
 *
 * These are exactly the arguments the recurrence above takes (second, factored form of the transition in Sec. 3.1.1).
 * The paper says k is "normalized" without naming the norm; L2 with the usual epsilon guard is the reading taken.
 * z_beta / beta may be NULL together.  Everything in double; no reordering.
 */
static double softplus_d(double z) { return z > 0.0 ? z + log1p(exp(-z)) : log1p(exp(z)); }

int rodimus_oracle_ddts_gates(const float *z_g, const float *z_tau, const float *z_beta,
                              const float *q, const float *k,
                              double *log_alpha, double *beta, double *q_out, double *k_out,
                              long M, int dk, int dv)
{
    if (!z_g || !z_tau || !q || !k || !log_alpha || !q_out || !k_out) return 1;
    if ((z_beta == NULL) != (beta == NULL)) return 1;
    if (M < 0 || dk <= 0 || dv < 0) return 1;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < M; ++r) {
        const size_t o = (size_t)r * dk;
        double norm2 = 0.0;
        for (int n = 0; n < dk; ++n) norm2 += (double)k[o + n] * (double)k[o + n];
        const double norm = sqrt(norm2);
        const double inv = 1.0 / (norm > 1e-12 ? norm : 1e-12);
        for (int n = 0; n < dk; ++n) {
            const double g = softplus_d((double)z_g[o + n]);
            const double tau = sigmoid_d((double)z_tau[o + n]);
            log_alpha[o + n] = -g * tau;
            k_out[o + n] = pow(g, tau) * (double)k[o + n] * inv;
            q_out[o + n] = (double)q[o + n] / sqrt((double)dk);
        }
        if (z_beta)
            for (int j = 0; j < dv; ++j) beta[(size_t)r * dv + j] = sigmoid_d((double)z_beta[(size_t)r * dv + j]);
    }
    return 0;
}

/*
 * Backward pass of the sequential scan: reverse-mode differentiation of the recurrence above, step by step
 * (training use of the block, paper Sec. 3.1.3; the recurrence is the one printed there).  Given the
 * cotangents do_t of the outputs and dS_T of the final state (NULL = zero), with
 *
 *     S_t = diag(a_t) S_{t-1} + k_t^T u_t,   u_t = beta_t .* v_t,   a_t = exp(log_alpha_t),   o_t = q_t S_t
 *
 * the total cotangent of S_t is  G_t = q_t^T do_t + diag(a_{t+1}) G_{t+1}  (G_{T+1} taken so that the carried term at
 * t = T is dS_T), and
 *
 *     dq_t = do_t S_t^T              dk_t = u_t G_t^T              du_t = k_t G_t
 *     dv_t = beta_t .* du_t          dbeta_t = v_t .* du_t
 *     dlog_alpha_t = a_t .* rowsum(G_t .* S_{t-1})                 dS_0 = diag(a_1) G_1
 *
 * The states S_t are needed in reverse order: they are kept at every `segment`-th step during a forward sweep and
 * recomputed inside a segment (the same arithmetic as the forward oracle, so nothing is approximated).
 * beta == NULL means the all-ones gate (dbeta is then not written and may be NULL).  Any output pointer may be NULL.
 * Returns 0 on success, 1 on bad arguments, 2 on allocation failure.
 */
static int scan_bwd_impl(const float *q, const float *k, const float *v,
                         const float *log_alpha, const float *beta, int beta_is_preactivation, const double *S0,
                         const double *d_o, const double *dS_T,
                         double *dq, double *dk, double *dv, double *dlog_alpha, double *dbeta, double *dS0,
                         int B, int T, int H, int dk_, int dv_)
{
    const int n = dk_, m = dv_, segment = 64;
    if (!q || !k || !v || !log_alpha || !d_o) return 1;
    if (B < 0 || T < 0 || H < 0 || n <= 0 || m <= 0) return 1;
    int failed = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const size_t sz = (size_t)n * m;
            const int nseg = (T + segment - 1) / segment;
            double *ck = (double *)malloc(sizeof(double) * sz * (size_t)(nseg + 1));      /* state entering each segment */
            double *sb = (double *)malloc(sizeof(double) * sz * (size_t)(segment + 1));   /* states inside one segment  */
            double *G = (double *)malloc(sizeof(double) * sz);
            double *u = (double *)malloc(sizeof(double) * (size_t)m);
            double *du = (double *)malloc(sizeof(double) * (size_t)m);
            double *otmp = (double *)malloc(sizeof(double) * (size_t)m);
            if (!ck || !sb || !G || !u || !du || !otmp) {
                free(ck); free(sb); free(G); free(u); free(du); free(otmp);
#pragma omp atomic write
                failed = 1;
                continue;
            }
            const size_t state_off = ((size_t)b * H + h) * sz;
            /* forward sweep: remember the state entering every segment */
            for (size_t e = 0; e < sz; ++e) ck[e] = S0 ? S0[state_off + e] : 0.0;
            for (int s = 0; s < nseg; ++s) {
                double *cur = ck + (size_t)(s + 1) * sz;
                for (size_t e = 0; e < sz; ++e) cur[e] = ck[(size_t)s * sz + e];
                const int t1 = (s + 1) * segment < T ? (s + 1) * segment : T;
                for (int t = s * segment; t < t1; ++t) {
                    const size_t row = ((size_t)b * T + t) * H + h;
                    ddts_update(cur, q + row * n, k + row * n, v + row * m, log_alpha + row * n,
                                beta ? beta + row * m : NULL, beta_is_preactivation, otmp, n, m, u);
                }
            }
            /* reverse sweep */
            for (size_t e = 0; e < sz; ++e) G[e] = dS_T ? dS_T[state_off + e] : 0.0;     /* carried term diag(a_{t+1}) G_{t+1} */
            for (int s = nseg - 1; s >= 0; --s) {
                const int t0 = s * segment, t1 = (s + 1) * segment < T ? (s + 1) * segment : T;
                for (size_t e = 0; e < sz; ++e) sb[e] = ck[(size_t)s * sz + e];
                for (int t = t0; t < t1; ++t) {             /* sb[i+1] = S_t for t = t0 + i */
                    const size_t row = ((size_t)b * T + t) * H + h;
                    double *nxt = sb + (size_t)(t - t0 + 1) * sz;
                    for (size_t e = 0; e < sz; ++e) nxt[e] = sb[(size_t)(t - t0) * sz + e];
                    ddts_update(nxt, q + row * n, k + row * n, v + row * m, log_alpha + row * n,
                                beta ? beta + row * m : NULL, beta_is_preactivation, otmp, n, m, u);
                }
                for (int t = t1 - 1; t >= t0; --t) {
                    const size_t row = ((size_t)b * T + t) * H + h;
                    const double *St = sb + (size_t)(t - t0 + 1) * sz, *Sp = sb + (size_t)(t - t0) * sz;
                    const float *qt = q + row * n, *kt = k + row * n, *vt = v + row * m, *lt = log_alpha + row * n;
                    const float *bt = beta ? beta + row * m : NULL;
                    const double *dot = d_o + row * m;
                    /* G_t = carried + q_t^T do_t */
                    for (int r = 0; r < n; ++r)
                        for (int j = 0; j < m; ++j) G[(size_t)r * m + j] += (double)qt[r] * dot[j];
                    for (int j = 0; j < m; ++j) {
                        /* the gate's value; with the flag set the array holds z_beta and the gate is sigmoid(z_beta) */
                        double gate = 1.0;
                        if (bt) gate = beta_is_preactivation ? sigmoid_d((double)bt[j]) : (double)bt[j];
                        u[j] = gate * (double)vt[j];
                        double acc = 0.0;
                        for (int r = 0; r < n; ++r) acc += (double)kt[r] * G[(size_t)r * m + j];
                        du[j] = acc;
                        if (dv) dv[row * m + j] = gate * acc;
                        /* cotangent of the gate, v .* du; of its pre-activation: times sigmoid'(z) = gate (1 - gate) */
                        if (dbeta && bt) dbeta[row * m + j] = (double)vt[j] * acc * (beta_is_preactivation ? gate * (1.0 - gate) : 1.0);
                    }
                    for (int r = 0; r < n; ++r) {
                        const double a = exp((double)lt[r]);
                        double accq = 0.0, acck = 0.0, acca = 0.0;
                        for (int j = 0; j < m; ++j) {
                            accq += St[(size_t)r * m + j] * dot[j];
                            acck += G[(size_t)r * m + j] * u[j];
                            acca += G[(size_t)r * m + j] * Sp[(size_t)r * m + j];
                        }
                        if (dq) dq[row * n + r] = accq;
                        if (dk) dk[row * n + r] = acck;
                        if (dlog_alpha) dlog_alpha[row * n + r] = a * acca;
                        for (int j = 0; j < m; ++j) G[(size_t)r * m + j] *= a;       /* carried to step t-1 */
                    }
                }
            }
            if (dS0)
                for (size_t e = 0; e < sz; ++e) dS0[state_off + e] = G[e];
            free(ck); free(sb); free(G); free(u); free(du); free(otmp);
        }
    }
    return failed ? 2 : 0;
}

int rodimus_oracle_scan_bwd(const float *q, const float *k, const float *v,
                            const float *log_alpha, const float *beta, const double *S0,
                            const double *d_o, const double *dS_T,
                            double *dq, double *dk, double *dv, double *dlog_alpha, double *dbeta, double *dS0,
                            int B, int T, int H, int dk_, int dv_)
{
    return scan_bwd_impl(q, k, v, log_alpha, beta, 0, S0, d_o, dS_T, dq, dk, dv, dlog_alpha, dbeta, dS0, B, T, H, dk_, dv_);
}

/* The same with the value gate given as its pre-activation (Sec. 3.1.2: beta_hat = sigmoid(z_beta)): `z_beta` in place of
 * beta, and dz_beta = (v .* du) .* beta_hat (1 - beta_hat) in place of dbeta. */
int rodimus_oracle_scan_bwd_zbeta(const float *q, const float *k, const float *v,
                                  const float *log_alpha, const float *z_beta, const double *S0,
                                  const double *d_o, const double *dS_T,
                                  double *dq, double *dk, double *dv, double *dlog_alpha, double *dz_beta, double *dS0,
                                  int B, int T, int H, int dk_, int dv_)
{
    if (!z_beta) return 1;
    return scan_bwd_impl(q, k, v, log_alpha, z_beta, 1, S0, d_o, dS_T, dq, dk, dv, dlog_alpha, dz_beta, dS0, B, T, H, dk_, dv_);
}

/*
 * Output stage of the block around the recurrence (paper Sec. 3.1.3): the feed-through term of the block's state-space
 * form, o_t = q_t S_t + d .* x'_t with d a learnable weight per value channel (here one row per head) and x'_t the
 * short-convolved input, followed by the output gate of the Gated Linear Unit the block is merged into,
 * y_t = o_t .* act(z_t).  The paper cites the GLU of Dauphin et al. (sigmoid gate) and describes the block as akin to
 * the Mamba series (SiLU gate) without printing the activation: both are offered (act = 0: sigmoid(z), 1: z * sigmoid(z)).
 *   o        [rows, H, dv] double (rows = B*T), the recurrence output
 *   x_prime  [rows, H, dv] float or NULL (no feed-through);  d [H, dv] float (required with x_prime)
 *   z_gate   [rows, H, dv] float or NULL (no output gate)
 * Everything in double, element by element.
 */
int rodimus_oracle_block_output(const double *o, const float *x_prime, const float *d, const float *z_gate,
                                double *y, long rows, int H, int dv, int act)
{
    if (!o || !y || rows < 0 || H < 0 || dv <= 0) return 1;
    if (x_prime && !d) return 1;
    if (act != 0 && act != 1) return 1;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r)
        for (int h = 0; h < H; ++h)
            for (int j = 0; j < dv; ++j) {
                const size_t e = ((size_t)r * H + h) * dv + j;
                double val = o[e];
                if (x_prime) val += (double)d[(size_t)h * dv + j] * (double)x_prime[e];
                if (z_gate) {
                    const double z = (double)z_gate[e];
                    val *= act == 0 ? sigmoid_d(z) : z * sigmoid_d(z);
                }
                y[e] = val;
            }
    return 0;
}

/*
 * ShortConv of the block (paper Sec. 3.1.3): the block's input x_t is passed through a short convolution to give x'_t,
 * which feeds the gates and the feed-through term.  The paper names the operator and points to the recurrent models
 * that use it without printing it; the reading taken is the one of those models: a causal depthwise convolution over
 * time of width W (each channel has its own W taps and a bias), optionally followed by SiLU,
 *     x'_t[c] = act( bias[c] + sum_{j=0..W-1} w[c][j] * x_{t-(W-1)+j}[c] ),
 * where inputs before the call's first token come from `state_in` (the last W-1 inputs of the previous call, oldest
 * first) or are zero.  `state_out` receives the last W-1 inputs seen so far (for a decode step: T = 1).
 *   x          [B, T, C] float           w [C, W] float       bias [C] float or NULL
 *   state_in   [B, W-1, C] float or NULL  y [B, T, C] double   state_out [B, W-1, C] double or NULL
 *   act = 0: none, 1: SiLU (z * sigmoid(z)).
 * Everything in double, tap by tap in the order j = 0..W-1.
 */
int rodimus_oracle_short_conv(const float *x, const float *w, const float *bias, const float *state_in,
                              double *y, double *state_out, int B, int T, int C, int W, int act)
{
    if (B < 0 || T < 0 || C < 0 || W < 1) return 1;
    if (act != 0 && act != 1) return 1;
    if ((size_t)B * T * C > 0 && (!x || !y)) return 1;
    if (C > 0 && !w) return 1;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c) {
            /* input at time s of this (b, c): s in [-(W-1), T) */
#define XIN(s) ((s) >= 0 ? (double)x[((size_t)b * T + (s)) * C + c] \
                         : (state_in ? (double)state_in[((size_t)b * (W - 1) + (W - 1 + (s))) * C + c] : 0.0))
            for (int t = 0; t < T; ++t) {
                double acc = bias ? (double)bias[c] : 0.0;
                for (int j = 0; j < W; ++j) acc += (double)w[(size_t)c * W + j] * XIN(t - (W - 1) + j);
                y[((size_t)b * T + t) * C + c] = act == 1 ? acc * sigmoid_d(acc) : acc;
            }
            if (state_out)
                for (int j = 0; j < W - 1; ++j) state_out[((size_t)b * (W - 1) + j) * C + c] = XIN(T - (W - 1) + j);
#undef XIN
        }
    return 0;
}

/*
 * The block's recurrence taken straight from its pre-activations (paper Sec. 3.1.3, the state-space form of the
 * overall block, with the gates of Sec. 3.1.2 and the pre-processing of q and k stated after it):
 *
 *     g = softplus(z_g),  tau = sigmoid(z_tau),  beta_hat = sigmoid(z_beta)
 *     S_t = diag(exp(-g .* tau)) S_{t-1} + (g^tau .* khat_t)^T (beta_hat .* v_t),   o_t = (q_t / sqrt(dk)) S_t
 *     khat_t = k_t / max(||k_t||_2, 1e-12)
 *
 * One token of one (b, h), in place on S; z_beta may be NULL (beta_hat = 1).  Everything in double, written out from
 * the equation (it does not go through rodimus_oracle_ddts_gates or ddts_update above, which the tests compare it with).
 */
static void block_update(double *S, const float *q, const float *k, const float *v, const float *z_g, const float *z_tau,
                         const float *z_beta, double *o, int dk, int dv)
{
    double norm2 = 0.0;
    for (int r = 0; r < dk; ++r) norm2 += (double)k[r] * (double)k[r];
    double norm = sqrt(norm2);
    if (norm < 1e-12) norm = 1e-12;
    for (int r = 0; r < dk; ++r) {
        const double g = softplus_d((double)z_g[r]);
        const double tau = sigmoid_d((double)z_tau[r]);
        const double decay = exp(-g * tau);
        const double write = pow(g, tau) * ((double)k[r] / norm);
        double *Srow = S + (size_t)r * dv;
        for (int j = 0; j < dv; ++j) {
            const double bv = (z_beta ? sigmoid_d((double)z_beta[j]) : 1.0) * (double)v[j];
            Srow[j] = decay * Srow[j] + write * bv;
        }
    }
    const double scale = 1.0 / sqrt((double)dk);
    for (int j = 0; j < dv; ++j) {
        double acc = 0.0;
        for (int r = 0; r < dk; ++r) acc += (double)q[r] * scale * S[(size_t)r * dv + j];
        o[j] = acc;
    }
}

/* Sequential scan of the block from pre-activations.  Layouts as rodimus_oracle_scan, z_g, z_tau [B,T,H,dk],
 * z_beta [B,T,H,dv] or NULL. */
int rodimus_oracle_scan_gated(const float *q, const float *k, const float *v, const float *z_g, const float *z_tau,
                              const float *z_beta, const double *S0, double *o, double *S_T,
                              int B, int T, int H, int dk, int dv)
{
    if (!q || !k || !v || !z_g || !z_tau || !o) return 1;
    if (B < 0 || T < 0 || H < 0 || dk <= 0 || dv <= 0) return 1;
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *S = (double *)malloc(sizeof(double) * (size_t)dk * dv);
            if (!S) {
#pragma omp atomic write
                failed = 1;
                continue;
            }
            const size_t state_off = ((size_t)b * H + h) * (size_t)dk * dv;
            for (size_t e = 0; e < (size_t)dk * dv; ++e) S[e] = S0 ? S0[state_off + e] : 0.0;
            for (int t = 0; t < T; ++t) {
                const size_t row = ((size_t)b * T + t) * H + h;
                block_update(S, q + row * dk, k + row * dk, v + row * dv, z_g + row * dk, z_tau + row * dk,
                             z_beta ? z_beta + row * dv : NULL, o + row * dv, dk, dv);
            }
            if (S_T)
                for (size_t e = 0; e < (size_t)dk * dv; ++e) S_T[state_off + e] = S[e];
            free(S);
        }
    }
    return failed ? 2 : 0;
}

/*
 * Backward pass of rodimus_oracle_scan_gated: reverse-mode differentiation of the block's recurrence (Sec. 3.1.3) through
 * the gates of Sec. 3.1.2 and the pre-processing of q and k, step by step in double.  Per step, with
 *
 *     g = softplus(z_g)   tau = sigmoid(z_tau)   a = exp(-g tau)   w = g^tau   n = max(||k||_2, 1e-12)
 *     khat = w .* k / n   qhat = q / sqrt(dk)    s = sigmoid(z_beta)   u = s .* v
 *     S_t = diag(a) S_{t-1} + khat^T u           o_t = qhat S_t
 *
 * and G_t = qhat_t^T do_t + diag(a_{t+1}) G_{t+1} the cotangent of S_t (the carried term at t = T is dS_T):
 *
 *     dqhat = do S_t^T      dkhat = u G_t^T      du = khat G_t      da = rowsum(G_t .* S_{t-1})
 *     dq = dqhat / sqrt(dk)
 *     dv = s .* du          dz_beta = v .* du .* s (1 - s)
 *     dw = dkhat .* k / n
 *     dk = dkhat .* w / n - k (sum_r dkhat_r w_r k_r) / n^3       (second term only while ||k|| is above the guard)
 *     dg   = -da a tau + dw tau g^(tau - 1)
 *     dtau = -da a g   + dw w ln g
 *     dz_g = dg sigmoid(z_g)       dz_tau = dtau tau (1 - tau)
 *
 * (g > 0 always; where g underflows to 0 in double, w = 0 and the dw terms are taken as 0.)  The states are recomputed
 * per segment of 64 steps as in the backward pass above.  z_beta == NULL means the all-ones value gate (dz_beta is then
 * not written).  Any output pointer may be NULL.  Returns 0 on success, 1 on bad arguments, 2 on allocation failure.
 */
int rodimus_oracle_scan_gated_bwd(const float *q, const float *k, const float *v, const float *z_g, const float *z_tau,
                                  const float *z_beta, const double *S0, const double *d_o, const double *dS_T,
                                  double *dq, double *dk, double *dv, double *dz_g, double *dz_tau, double *dz_beta, double *dS0,
                                  int B, int T, int H, int dk_, int dv_)
{
    const int n = dk_, m = dv_, segment = 64;
    if (!q || !k || !v || !z_g || !z_tau || !d_o) return 1;
    if (B < 0 || T < 0 || H < 0 || n <= 0 || m <= 0) return 1;
    int failed = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const size_t sz = (size_t)n * m;
            const int nseg = (T + segment - 1) / segment;
            double *ck = (double *)malloc(sizeof(double) * sz * (size_t)(nseg + 1));      /* state entering each segment */
            double *sb = (double *)malloc(sizeof(double) * sz * (size_t)(segment + 1));   /* states inside one segment  */
            double *G = (double *)malloc(sizeof(double) * sz);
            double *u = (double *)malloc(sizeof(double) * (size_t)m);
            double *otmp = (double *)malloc(sizeof(double) * (size_t)m);
            double *dkhat = (double *)malloc(sizeof(double) * (size_t)n);
            if (!ck || !sb || !G || !u || !otmp || !dkhat) {
                free(ck); free(sb); free(G); free(u); free(otmp); free(dkhat);
#pragma omp atomic write
                failed = 1;
                continue;
            }
            const size_t state_off = ((size_t)b * H + h) * sz;
            /* forward sweep: remember the state entering every segment */
            for (size_t e = 0; e < sz; ++e) ck[e] = S0 ? S0[state_off + e] : 0.0;
            for (int s = 0; s < nseg; ++s) {
                double *cur = ck + (size_t)(s + 1) * sz;
                for (size_t e = 0; e < sz; ++e) cur[e] = ck[(size_t)s * sz + e];
                const int t1 = (s + 1) * segment < T ? (s + 1) * segment : T;
                for (int t = s * segment; t < t1; ++t) {
                    const size_t row = ((size_t)b * T + t) * H + h;
                    block_update(cur, q + row * n, k + row * n, v + row * m, z_g + row * n, z_tau + row * n,
                                 z_beta ? z_beta + row * m : NULL, otmp, n, m);
                }
            }
            /* reverse sweep */
            for (size_t e = 0; e < sz; ++e) G[e] = dS_T ? dS_T[state_off + e] : 0.0;     /* carried term diag(a_{t+1}) G_{t+1} */
            const double qscale = 1.0 / sqrt((double)n);
            for (int s = nseg - 1; s >= 0; --s) {
                const int t0 = s * segment, t1 = (s + 1) * segment < T ? (s + 1) * segment : T;
                for (size_t e = 0; e < sz; ++e) sb[e] = ck[(size_t)s * sz + e];
                for (int t = t0; t < t1; ++t) {             /* sb[i+1] = S_t for t = t0 + i */
                    const size_t row = ((size_t)b * T + t) * H + h;
                    double *nxt = sb + (size_t)(t - t0 + 1) * sz;
                    for (size_t e = 0; e < sz; ++e) nxt[e] = sb[(size_t)(t - t0) * sz + e];
                    block_update(nxt, q + row * n, k + row * n, v + row * m, z_g + row * n, z_tau + row * n,
                                 z_beta ? z_beta + row * m : NULL, otmp, n, m);
                }
                for (int t = t1 - 1; t >= t0; --t) {
                    const size_t row = ((size_t)b * T + t) * H + h;
                    const double *St = sb + (size_t)(t - t0 + 1) * sz, *Sp = sb + (size_t)(t - t0) * sz;
                    const float *qt = q + row * n, *kt = k + row * n, *vt = v + row * m;
                    const float *zgt = z_g + row * n, *ztt = z_tau + row * n, *zbt = z_beta ? z_beta + row * m : NULL;
                    const double *dot = d_o + row * m;
                    double norm2 = 0.0;
                    for (int r = 0; r < n; ++r) norm2 += (double)kt[r] * (double)kt[r];
                    const int guarded = !(sqrt(norm2) > 1e-12);
                    const double norm = guarded ? 1e-12 : sqrt(norm2);
                    /* G_t = carried + qhat_t^T do_t */
                    for (int r = 0; r < n; ++r)
                        for (int j = 0; j < m; ++j) G[(size_t)r * m + j] += (double)qt[r] * qscale * dot[j];
                    /* value side: du = khat G_t */
                    for (int j = 0; j < m; ++j) {
                        const double sg = zbt ? sigmoid_d((double)zbt[j]) : 1.0;
                        u[j] = sg * (double)vt[j];
                        double acc = 0.0;
                        for (int r = 0; r < n; ++r) {
                            const double w = pow(softplus_d((double)zgt[r]), sigmoid_d((double)ztt[r]));
                            acc += w * ((double)kt[r] / norm) * G[(size_t)r * m + j];
                        }
                        if (dv) dv[row * m + j] = sg * acc;
                        if (dz_beta && zbt) dz_beta[row * m + j] = (double)vt[j] * acc * sg * (1.0 - sg);
                    }
                    /* key side */
                    double through_norm = 0.0;                   /* sum_r dkhat_r w_r k_r */
                    for (int r = 0; r < n; ++r) {
                        double acc = 0.0;
                        for (int j = 0; j < m; ++j) acc += G[(size_t)r * m + j] * u[j];
                        dkhat[r] = acc;
                        through_norm += acc * pow(softplus_d((double)zgt[r]), sigmoid_d((double)ztt[r])) * (double)kt[r];
                    }
                    for (int r = 0; r < n; ++r) {
                        const double g = softplus_d((double)zgt[r]), tau = sigmoid_d((double)ztt[r]);
                        const double a = exp(-g * tau), w = pow(g, tau);
                        double accq = 0.0, acca = 0.0;
                        for (int j = 0; j < m; ++j) {
                            accq += St[(size_t)r * m + j] * dot[j];
                            acca += G[(size_t)r * m + j] * Sp[(size_t)r * m + j];
                        }
                        if (dq) dq[row * n + r] = accq * qscale;
                        double dk_r = dkhat[r] * w / norm;
                        if (!guarded) dk_r -= (double)kt[r] * through_norm / (norm * norm * norm);
                        if (dk) dk[row * n + r] = dk_r;
                        const double dw = dkhat[r] * (double)kt[r] / norm;
                        double dg = -acca * a * tau, dtau = -acca * a * g;
                        if (g > 0.0) {
                            dg += dw * tau * pow(g, tau - 1.0);
                            dtau += dw * w * log(g);
                        }
                        if (dz_g) dz_g[row * n + r] = dg * sigmoid_d((double)zgt[r]);
                        if (dz_tau) dz_tau[row * n + r] = dtau * tau * (1.0 - tau);
                        for (int j = 0; j < m; ++j) G[(size_t)r * m + j] *= a;       /* carried to step t-1 */
                    }
                }
            }
            if (dS0)
                for (size_t e = 0; e < sz; ++e) dS0[state_off + e] = G[e];
            free(ck); free(sb); free(G); free(u); free(otmp); free(dkhat);
        }
    }
    return failed ? 2 : 0;
}

/* One decode step of the same for N sequences, S [N,H,dk,dv] updated in place. */
int rodimus_oracle_step_gated(const float *q, const float *k, const float *v, const float *z_g, const float *z_tau,
                              const float *z_beta, double *S, double *o, int N, int H, int dk, int dv)
{
    if (!q || !k || !v || !z_g || !z_tau || !S || !o) return 1;
    if (N < 0 || H < 0 || dk <= 0 || dv <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (long s = 0; s < (long)N * H; ++s)
        block_update(S + (size_t)s * dk * dv, q + (size_t)s * dk, k + (size_t)s * dk, v + (size_t)s * dv,
                     z_g + (size_t)s * dk, z_tau + (size_t)s * dk, z_beta ? z_beta + (size_t)s * dv : NULL,
                     o + (size_t)s * dv, dk, dv);
    return 0;
}

/*
 * The recurrence with the general transition of Sec. 3.1.1: as rodimus_oracle_scan / rodimus_oracle_step with one more
 * input, log_beta_t [B,T,H,dv] / [N,H,dv] (<= 0), the logarithm of the transition gate along the value dimension.
 * `beta` stays the input gate on the value (values, not pre-activations).
 */
int rodimus_oracle_scan_general(const float *q, const float *k, const float *v, const float *log_alpha,
                                const float *log_beta_t, const float *beta, const double *S0, double *o, double *S_T,
                                int B, int T, int H, int dk, int dv)
{
    if (!q || !k || !v || !log_alpha || !log_beta_t || !o) return 1;
    if (B < 0 || T < 0 || H < 0 || dk <= 0 || dv <= 0) return 1;
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *S = (double *)malloc(sizeof(double) * (size_t)dk * dv);
            double *gv = (double *)malloc(sizeof(double) * (size_t)dv);
            if (!S || !gv) {
                free(S); free(gv);
#pragma omp atomic write
                failed = 1;
                continue;
            }
            const size_t state_off = ((size_t)b * H + h) * (size_t)dk * dv;
            for (size_t e = 0; e < (size_t)dk * dv; ++e) S[e] = S0 ? S0[state_off + e] : 0.0;
            for (int t = 0; t < T; ++t) {
                const size_t row = ((size_t)b * T + t) * H + h;
                ddts_update_general(S, q + row * dk, k + row * dk, v + row * dv, log_alpha + row * dk, log_beta_t + row * dv,
                                    beta ? beta + row * dv : NULL, 0, o + row * dv, dk, dv, gv);
            }
            if (S_T)
                for (size_t e = 0; e < (size_t)dk * dv; ++e) S_T[state_off + e] = S[e];
            free(S); free(gv);
        }
    }
    return failed ? 2 : 0;
}

int rodimus_oracle_step_general(const float *q, const float *k, const float *v, const float *log_alpha,
                                const float *log_beta_t, const float *beta, double *S, double *o, int N, int H, int dk, int dv)
{
    if (!q || !k || !v || !log_alpha || !log_beta_t || !S || !o) return 1;
    if (N < 0 || H < 0 || dk <= 0 || dv <= 0) return 1;
    int failed = 0;
#pragma omp parallel for schedule(static)
    for (long s = 0; s < (long)N * H; ++s) {
        double *gv = (double *)malloc(sizeof(double) * (size_t)dv);
        if (!gv) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        ddts_update_general(S + (size_t)s * dk * dv, q + (size_t)s * dk, k + (size_t)s * dk, v + (size_t)s * dv,
                            log_alpha + (size_t)s * dk, log_beta_t + (size_t)s * dv, beta ? beta + (size_t)s * dv : NULL, 0,
                            o + (size_t)s * dv, dk, dv, gv);
        free(gv);
    }
    return failed ? 2 : 0;
}
