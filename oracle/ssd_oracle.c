/*
 * TEST INFRASTRUCTURE ONLY -- fp64 CPU oracle for the selective state-space scan.
 *
 * Nothing in the product path may call this file; it exists so that tests, the smoke
 * check and the benchmark's cpu_baseline leg have an independent answer to compare with.
 * It shares no code with the HIP kernels.
 *
 * What it computes is the plain definition, token by token, with no chunking, blocking
 * or fusion (paper Sec. 3.1, Eq. 1: h_t = A_t h_{t-1} + B_t x_t, y_t = C_t h_t), in the
 * concrete Mamba-2 form used by the build: A_t = exp(dt_t * A_head) * I, the input matrix
 * is dt_t * B_t, and the output has a skip term D_head * x_t:
 *
 *     alpha_t        = exp(dt[b,t,h] * A[h])
 *     h_t[p,n]       = alpha_t * h_{t-1}[p,n] + dt[b,t,h] * x[b,t,h,p] * B[b,t,g,n]
 *     y[b,t,h,p]     = sum_n C[b,t,g,n] * h_t[p,n] + D[h] * x[b,t,h,p]
 *
 * with h_{-1} = init_state (zeros when NULL) and g the B/C group of head h.
 * boundary_states[b,k,h] is the state entering segment k (tokens k*segment ...), i.e.
 * the sequence-axis checkpoint of the paper's Sec. 3.3 (Alg. 1) under the reading that a
 * checkpoint holds the state needed to restart its segment.
 *
 * The backward routine is textbook reverse-mode differentiation of that loop (the
 * paper's Alg. 2 calls it Backward(x, h, grad_x, grad_h)).  It needs h_{t-1} while
 * walking backwards; instead of keeping every state it keeps one every `ckpt_every`
 * tokens and re-runs the very same forward loop inside each block, which reproduces the
 * stored trajectory bit for bit.
 *
 * Layouts (all row-major, all double):
 *   x, y, dy, dx : [Bt, L, H, P]      dt, ddt : [Bt, L, H]      A, D, dA, dD : [H]
 *   B, C, dB, dC : [Bt, L, G, N]      states  : [Bt, H, P, N]
 *   boundary_states : [Bt, L/segment, H, P, N]
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

static int group_of(int h, int H, int G, const int *head_group) {
    return head_group ? head_group[h] : h / (H / G);
}

/* One token of the recurrence for one (batch, head): updates h in place, writes y_t. */
static void step_forward(int P, int N, double alpha, double dt, double Dh, const double *xt,
                         const double *Bt, const double *Ct, double *h, double *yt) {
    for (int p = 0; p < P; ++p) {
        const double dtx = dt * xt[p];
        double acc = 0.0;
        double *hp = h + (size_t)p * N;
        for (int n = 0; n < N; ++n) {
            hp[n] = alpha * hp[n] + dtx * Bt[n];
            acc += Ct[n] * hp[n];
        }
        if (yt) yt[p] = acc + Dh * xt[p];
    }
}

/* Decay factor of token t: exp(dt_t A_h), or 0 where a new packed sequence starts (reset[b,t] != 0):
 * that token sees no state from the tokens before it. */
static double decay_of(const unsigned char *reset, size_t tok, double dt, double a_coef) {
    return (reset && reset[tok]) ? 0.0 : exp(dt * a_coef);
}

int ssd_oracle_fwd_packed(long Bt, long L, int H, int P, int G, int N, const double *x, const double *dt,
                          const double *A, const double *Bm, const double *Cm, const double *D,
                          const double *init_state, const int *head_group, const unsigned char *reset, double *y,
                          double *final_state, long segment, double *boundary_states) {
    if (Bt <= 0 || L < 0 || H <= 0 || P <= 0 || G <= 0 || N <= 0) return -1;
    if (!head_group && H % G != 0) return -1;
    if (boundary_states && (segment <= 0 || L % segment != 0)) return -1;
    const size_t PN = (size_t)P * N;
    const long nseg = boundary_states ? L / segment : 0;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long b = 0; b < Bt; ++b) {
        for (int h = 0; h < H; ++h) {
            double *st = (double *)malloc(PN * sizeof(double));
            if (!st) { fail = 1; continue; }
            if (init_state) memcpy(st, init_state + ((size_t)b * H + h) * PN, PN * sizeof(double));
            else memset(st, 0, PN * sizeof(double));
            const int g = group_of(h, H, G, head_group);
            for (long t = 0; t < L; ++t) {
                if (boundary_states && t % segment == 0)
                    memcpy(boundary_states + (((size_t)b * nseg + t / segment) * H + h) * PN, st,
                           PN * sizeof(double));
                const size_t tok = (size_t)b * L + t;
                step_forward(P, N, decay_of(reset, tok, dt[tok * H + h], A[h]), dt[tok * H + h], D[h],
                             x + (tok * H + h) * P, Bm + (tok * G + g) * N, Cm + (tok * G + g) * N, st,
                             y ? y + (tok * H + h) * P : NULL);
            }
            if (final_state) memcpy(final_state + ((size_t)b * H + h) * PN, st, PN * sizeof(double));
            free(st);
        }
    }
    return fail ? -2 : 0;
}

int ssd_oracle_fwd(long Bt, long L, int H, int P, int G, int N, const double *x, const double *dt,
                   const double *A, const double *Bm, const double *Cm, const double *D,
                   const double *init_state, const int *head_group, double *y,
                   double *final_state, long segment, double *boundary_states) {
    return ssd_oracle_fwd_packed(Bt, L, H, P, G, N, x, dt, A, Bm, Cm, D, init_state, head_group, NULL, y, final_state,
                                 segment, boundary_states);
}

int ssd_oracle_bwd_packed(long Bt, long L, int H, int P, int G, int N, const double *x, const double *dt,
                          const double *A, const double *Bm, const double *Cm, const double *D,
                          const double *init_state, const int *head_group, const unsigned char *reset,
                          const double *dy, const double *dfinal_state, double *dx, double *ddt, double *dA,
                          double *dB, double *dC, double *dD, double *dinit_state, long ckpt_every) {
    if (Bt <= 0 || L < 0 || H <= 0 || P <= 0 || G <= 0 || N <= 0) return -1;
    if (!head_group && H % G != 0) return -1;
    if (ckpt_every <= 0) ckpt_every = 256;
    const size_t PN = (size_t)P * N;
    const long nblk = (L + ckpt_every - 1) / ckpt_every;
    memset(dA, 0, (size_t)H * sizeof(double));
    memset(dD, 0, (size_t)H * sizeof(double));
    memset(dB, 0, (size_t)Bt * L * G * N * sizeof(double));
    memset(dC, 0, (size_t)Bt * L * G * N * sizeof(double));
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long b = 0; b < Bt; ++b) {
        for (int h = 0; h < H; ++h) {
            /* entering[k] = state before token k*ckpt_every; traj[i] = state before token blk0+i */
            double *entering = (double *)malloc((size_t)(nblk > 0 ? nblk : 1) * PN * sizeof(double));
            double *traj = (double *)malloc((size_t)(ckpt_every + 1) * PN * sizeof(double));
            double *lam = (double *)malloc(PN * sizeof(double));
            double *carry = (double *)malloc(PN * sizeof(double));
            double *dBh = (double *)calloc((size_t)(L > 0 ? L : 1) * N, sizeof(double));
            double *dCh = (double *)calloc((size_t)(L > 0 ? L : 1) * N, sizeof(double));
            if (!entering || !traj || !lam || !carry || !dBh || !dCh) {
                fail = 1;
                free(entering); free(traj); free(lam); free(carry); free(dBh); free(dCh);
                continue;
            }
            const int g = group_of(h, H, G, head_group);
            const double a_coef = A[h], Dh = D[h];
            /* pass 1: forward, keeping the state at every block start */
            if (init_state) memcpy(traj, init_state + ((size_t)b * H + h) * PN, PN * sizeof(double));
            else memset(traj, 0, PN * sizeof(double));
            for (long t = 0; t < L; ++t) {
                if (t % ckpt_every == 0) memcpy(entering + (t / ckpt_every) * PN, traj, PN * sizeof(double));
                const size_t tok = (size_t)b * L + t;
                step_forward(P, N, decay_of(reset, tok, dt[tok * H + h], a_coef), dt[tok * H + h], Dh,
                             x + (tok * H + h) * P, Bm + (tok * G + g) * N, Cm + (tok * G + g) * N, traj, NULL);
            }
            /* adjoint flowing into h_{L-1} from beyond the sequence */
            if (dfinal_state) memcpy(carry, dfinal_state + ((size_t)b * H + h) * PN, PN * sizeof(double));
            else memset(carry, 0, PN * sizeof(double));
            double dA_acc = 0.0, dD_acc = 0.0;
            for (long k = nblk - 1; k >= 0; --k) {
                const long t0 = k * ckpt_every;
                const long t1 = (t0 + ckpt_every < L) ? t0 + ckpt_every : L;
                /* re-run the block: traj[i] = h_{t0+i-1}, i = 0 .. t1-t0 */
                memcpy(traj, entering + k * PN, PN * sizeof(double));
                for (long t = t0; t < t1; ++t) {
                    double *nxt = traj + (size_t)(t - t0 + 1) * PN;
                    memcpy(nxt, traj + (size_t)(t - t0) * PN, PN * sizeof(double));
                    const size_t tok = (size_t)b * L + t;
                    step_forward(P, N, decay_of(reset, tok, dt[tok * H + h], a_coef), dt[tok * H + h], Dh,
                                 x + (tok * H + h) * P, Bm + (tok * G + g) * N, Cm + (tok * G + g) * N, nxt, NULL);
                }
                for (long t = t1 - 1; t >= t0; --t) {
                    const size_t tok = (size_t)b * L + t;
                    const double dtt = dt[tok * H + h];
                    const double alpha = decay_of(reset, tok, dtt, a_coef); /* 0 at a sequence start: da = 0 there too */
                    const double *xt = x + (tok * H + h) * P;
                    const double *dyt = dy + (tok * H + h) * P;
                    const double *Bt_ = Bm + (tok * G + g) * N;
                    const double *Ct_ = Cm + (tok * G + g) * N;
                    const double *h_prev = traj + (size_t)(t - t0) * PN;
                    const double *h_cur = traj + (size_t)(t - t0 + 1) * PN;
                    double *dBt = dBh + (size_t)t * N, *dCt = dCh + (size_t)t * N;
                    double *dxt = dx + (tok * H + h) * P;
                    double f = 0.0, da = 0.0;
                    for (int p = 0; p < P; ++p) {
                        double sx = 0.0;
                        for (int n = 0; n < N; ++n) {
                            const size_t i = (size_t)p * N + n;
                            const double l = carry[i] + dyt[p] * Ct_[n]; /* total adjoint of h_t */
                            lam[i] = l;
                            dCt[n] += dyt[p] * h_cur[i];
                            dBt[n] += dtt * xt[p] * l;
                            sx += Bt_[n] * l;
                            da += l * h_prev[i];
                        }
                        dxt[p] = dtt * sx + Dh * dyt[p];
                        f += xt[p] * sx;
                        dD_acc += dyt[p] * xt[p];
                    }
                    da *= alpha;
                    ddt[tok * H + h] = a_coef * da + f;
                    dA_acc += dtt * da;
                    for (size_t i = 0; i < PN; ++i) carry[i] = alpha * lam[i];
                }
            }
            if (dinit_state) memcpy(dinit_state + ((size_t)b * H + h) * PN, carry, PN * sizeof(double));
#pragma omp critical
            {
                dA[h] += dA_acc;
                dD[h] += dD_acc;
                for (long t = 0; t < L; ++t) {
                    double *o1 = dB + (((size_t)b * L + t) * G + g) * N;
                    double *o2 = dC + (((size_t)b * L + t) * G + g) * N;
                    for (int n = 0; n < N; ++n) {
                        o1[n] += dBh[(size_t)t * N + n];
                        o2[n] += dCh[(size_t)t * N + n];
                    }
                }
            }
            free(entering); free(traj); free(lam); free(carry); free(dBh); free(dCh);
        }
    }
    return fail ? -2 : 0;
}

int ssd_oracle_bwd(long Bt, long L, int H, int P, int G, int N, const double *x, const double *dt,
                   const double *A, const double *Bm, const double *Cm, const double *D,
                   const double *init_state, const int *head_group, const double *dy,
                   const double *dfinal_state, double *dx, double *ddt, double *dA, double *dB,
                   double *dC, double *dD, double *dinit_state, long ckpt_every) {
    return ssd_oracle_bwd_packed(Bt, L, H, P, G, N, x, dt, A, Bm, Cm, D, init_state, head_group, NULL, dy, dfinal_state,
                                 dx, ddt, dA, dB, dC, dD, dinit_state, ckpt_every);
}
