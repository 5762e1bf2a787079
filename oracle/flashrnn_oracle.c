/*
 * flashrnn_oracle.c -- plain fp64 CPU oracle for the head-wise RNN time-step loop.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what "correct" means for the GPU library; it is
 * used by the tests, by the smoke check and by the bench's cpu_baseline leg, and by nothing else.
 * It shares no code with the HIP path.  Everything is double precision, the loop over time is the
 * outermost loop, the recurrent product is a plain triple loop, and nothing is tiled, fused or
 * reordered beyond what the defining equations say.
 *
 * What is computed (paper sections in brackets):
 *   forward   g_t = x_t + R s0_{t-1} + b ;  s_t = P(s_{t-1}, g_t)          [Sec. 3, eq. (1),(2)]
 *   backward  dg_t = dP/dg * ds_t ; ds_{t-1} = dP/ds * ds_t (+ R^T dg_t for the hidden state)
 *                                                                          [Sec. 4, eq. (3),(4)]
 *             dx_t = dg_t ; db = sum_t dg_t ; dR = sum_t dg_t s0_{t-1}^T    [Sec. 4, eq. (5)-(7)]
 *             optional value-wise clipping of the R^T dg_t term per step    [Sec. 4.1]
 *   heads     R is block diagonal: NH independent heads of size D          [Sec. 4.2]
 *   cells     LSTM, GRU, sLSTM, Elman point-wise functions P                [App. A]
 *
 * Readings of the paper taken here (each one is listed again in the design notes):
 *   - eq. (4) and (7) are printed with the time index of dg / s0 shifted by one; because g_t depends
 *     on s0_{t-1} (eq. (1)) the chain rule gives  ds0_{t-1} += R^T dg_t  and  dR = sum_t dg_t s0_{t-1}^T.
 *   - gate order on the G axis: LSTM and sLSTM  i, f, z, o ; GRU  r, z, n.   State order h, c, n, m.
 *   - Elman network (App. A): one state, one gate, h_t = tanh(x_t + R h_{t-1} + b).
 *   - GRU4: the GRU exactly as App. A prints it, four gates in the printed order z, r, n, g, every one of them a full
 *     pre-activation x + R h_{t-1} + b:   h_t = sig(z) h_{t-1} + (1 - sig(z)) tanh(n + sig(r) tanh(g))
 *     (the appendix remarks that n does not depend on the previous state and g not on the input; a caller models that
 *     with a zero R slice / zero inputs for those gates).
 *   - sLSTM equations (App. A) have unbalanced parentheses; read as
 *       m_t = max(log sig(f) + m_{t-1}, i)
 *       c_t = exp(log sig(f) + m_{t-1} - m_t) c_{t-1} + exp(i - m_t) tanh(z)
 *       n_t = exp(log sig(f) + m_{t-1} - m_t) n_{t-1} + exp(i - m_t)
 *       h_t = sig(o) c_t / n_t
 *     The stabilizer m carries no gradient (it cancels in h); dstates0[m] = 0.
 *   - GRU: three gates r, z, n.  r and z are ordinary gates.  The recurrent part of gate n,
 *     yn = R_n h_{t-1} + b_n, is multiplied by sig(r) before it meets the input:
 *       h_t = sig(z) h_{t-1} + (1 - sig(z)) tanh(x_n + sig(r) * yn)
 *     (App. A prints a four-"gate" form with an inner tanh; the three-gate textbook form is the one
 *     the benchmark configuration names.)  Consequently dWx and the recurrent-side gradient differ in
 *     gate n:  dWx_n = d(pre-tanh),  dg_n = d(yn) = d(pre-tanh) * sig(r);  db and dR use dg.
 *
 * Layouts (row major):  Wx[T,B,G,NH,D]  R[NH,D,G,D] (first D = previous-state index, last D = unit)
 *                       b[NH,G,D]  states[T+1,S,B,NH,D]  dH[T,B,NH,D]  dWx like Wx  dR like R  db like b
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC flashrnn_oracle.c -o libflashrnn_oracle.so -lm
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { CELL_LSTM = 0, CELL_GRU = 1, CELL_SLSTM = 2, CELL_ELMAN = 3, CELL_GRU4 = 4 };

static int n_states(int cell) { return cell == CELL_LSTM ? 2 : cell == CELL_GRU ? 1 : cell == CELL_SLSTM ? 4 : cell == CELL_ELMAN ? 1 : cell == CELL_GRU4 ? 1 : -1; }
static int n_gates(int cell) { return cell == CELL_LSTM ? 4 : cell == CELL_GRU ? 3 : cell == CELL_SLSTM ? 4 : cell == CELL_ELMAN ? 1 : cell == CELL_GRU4 ? 4 : -1; }

int oracle_num_states(int cell) { return n_states(cell); }
int oracle_num_gates(int cell) { return n_gates(cell); }

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double sigm(double x) { return 1.0 / (1.0 + exp(-x)); }

/* log(sigmoid(x)) without overflow for either sign of x */
static double logsigm(double x) { return x >= 0.0 ? -log1p(exp(-x)) : x - log1p(exp(x)); }

/* y[g*D+e] = sum_d h[d] * R[n,d,g,e]  -- recurrent product of eq. (1) for one head, one batch row */
static void recurrent_product(int D, int G, const double* Rn, const double* h, double* y) {
    for (int j = 0; j < G * D; ++j) y[j] = 0.0;
    for (int d = 0; d < D; ++d) {
        const double hv = h[d];
        const double* Rrow = Rn + (size_t)d * G * D;
        for (int j = 0; j < G * D; ++j) y[j] += hv * Rrow[j];
    }
}

#define WX(t, bb, g, n, e) Wx[((((size_t)(t) * B + (bb)) * G + (g)) * NH + (n)) * D + (e)]
#define DWX(t, bb, g, n, e) dWx[((((size_t)(t) * B + (bb)) * G + (g)) * NH + (n)) * D + (e)]
#define ST(t, s, bb, n, e) states[((((size_t)(t) * S + (s)) * B + (bb)) * NH + (n)) * D + (e)]
#define BI(n, g, e) bias[((size_t)(n) * G + (g)) * D + (e)]

/*
 * Forward pass.  states0 may be NULL (all initial states zero).  states[0] receives the initial
 * states, states[t] the states after step t.  Returns 0, or -1 on a bad argument.
 */
int oracle_fwd(int cell, int T, int B, int NH, int D, const double* Wx, const double* R, const double* bias,
               const double* states0, double* states) {
    const int S = n_states(cell), G = n_gates(cell);
    if (S < 0 || T < 0 || B <= 0 || NH <= 0 || D <= 0 || !Wx || !R || !bias || !states) return -1;
    const size_t slab = (size_t)S * B * NH * D;
    if (states0) memcpy(states, states0, slab * sizeof(double));
    else memset(states, 0, slab * sizeof(double));

    for (int t = 1; t <= T; ++t) {
#pragma omp parallel
        {
            double* y = (double*)malloc(sizeof(double) * G * D);
#pragma omp for collapse(2) schedule(static)
            for (int bb = 0; bb < B; ++bb) {
                for (int n = 0; n < NH; ++n) {
                    recurrent_product(D, G, R + (size_t)n * D * G * D, &ST(t - 1, 0, bb, n, 0), y);
                    for (int e = 0; e < D; ++e) {
                        if (cell == CELL_LSTM) {
                            const double pi = WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e);
                            const double pf = WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e);
                            const double pz = WX(t - 1, bb, 2, n, e) + y[2 * D + e] + BI(n, 2, e);
                            const double po = WX(t - 1, bb, 3, n, e) + y[3 * D + e] + BI(n, 3, e);
                            const double c = sigm(pf) * ST(t - 1, 1, bb, n, e) + sigm(pi) * tanh(pz);
                            ST(t, 1, bb, n, e) = c;
                            ST(t, 0, bb, n, e) = sigm(po) * tanh(c);
                        } else if (cell == CELL_SLSTM) {
                            const double pi = WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e);
                            const double pf = WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e);
                            const double pz = WX(t - 1, bb, 2, n, e) + y[2 * D + e] + BI(n, 2, e);
                            const double po = WX(t - 1, bb, 3, n, e) + y[3 * D + e] + BI(n, 3, e);
                            const double m_prev = ST(t - 1, 3, bb, n, e);
                            const double lf = logsigm(pf);
                            const double m = fmax(lf + m_prev, pi);
                            const double fg = exp(lf + m_prev - m);
                            const double ig = exp(pi - m);
                            const double c = fg * ST(t - 1, 1, bb, n, e) + ig * tanh(pz);
                            const double nn = fg * ST(t - 1, 2, bb, n, e) + ig;
                            ST(t, 1, bb, n, e) = c;
                            ST(t, 2, bb, n, e) = nn;
                            ST(t, 3, bb, n, e) = m;
                            ST(t, 0, bb, n, e) = sigm(po) * c / nn;
                        } else if (cell == CELL_ELMAN) {
                            ST(t, 0, bb, n, e) = tanh(WX(t - 1, bb, 0, n, e) + y[e] + BI(n, 0, e));
                        } else if (cell == CELL_GRU4) {
                            const double z = sigm(WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e));
                            const double r = sigm(WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e));
                            const double pn = WX(t - 1, bb, 2, n, e) + y[2 * D + e] + BI(n, 2, e);
                            const double tg = tanh(WX(t - 1, bb, 3, n, e) + y[3 * D + e] + BI(n, 3, e));
                            ST(t, 0, bb, n, e) = z * ST(t - 1, 0, bb, n, e) + (1.0 - z) * tanh(pn + r * tg);
                        } else { /* GRU */
                            const double pr = WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e);
                            const double pz = WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e);
                            const double yn = y[2 * D + e] + BI(n, 2, e);
                            const double cand = tanh(WX(t - 1, bb, 2, n, e) + sigm(pr) * yn);
                            const double z = sigm(pz);
                            ST(t, 0, bb, n, e) = z * ST(t - 1, 0, bb, n, e) + (1.0 - z) * cand;
                        }
                    }
                }
            }
            free(y);
        }
    }
    return 0;
}

/*
 * Backward pass (BPTT).  Gate pre-activations are recomputed from Wx, R, bias and the stored states,
 * so nothing but the forward's `states` is needed.  dH[t-1] is the external gradient on h_t
 * (t = 1..T).  dstates_last (may be NULL) is an extra gradient on the final states [S,B,NH,D]
 * (its stabilizer slot is ignored).  Outputs: dWx, dR, db, dstates0.
 */
int oracle_bwd_clipped(int cell, int T, int B, int NH, int D, const double* Wx, const double* R, const double* bias,
                       const double* states, const double* dH, const double* dstates_last, double recurrent_clip,
                       double* dWx, double* dR, double* db, double* dstates0) {
    const int S = n_states(cell), G = n_gates(cell);
    if (S < 0 || T < 0 || B <= 0 || NH <= 0 || D <= 0) return -1;
    if (!Wx || !R || !bias || !states || !dH || !dWx || !dR || !db || !dstates0) return -1;
    const size_t BHD = (size_t)B * NH * D;
    /* carried state gradients ds[s][b][n][e]; recurrent-side gate gradients dg[b][g][n][e] */
    double* ds = (double*)calloc((size_t)S * BHD, sizeof(double));
    double* dg = (double*)calloc((size_t)G * BHD, sizeof(double));
    double* dh_prev = (double*)calloc(BHD, sizeof(double));
    if (!ds || !dg || !dh_prev) { free(ds); free(dg); free(dh_prev); return -2; }
    if (dstates_last) memcpy(ds, dstates_last, (size_t)S * BHD * sizeof(double));
    if (cell == CELL_SLSTM) memset(ds + 3 * BHD, 0, BHD * sizeof(double));
    memset(dR, 0, sizeof(double) * NH * D * G * D);
    memset(db, 0, sizeof(double) * NH * G * D);

#define DS(s, bb, n, e) ds[(((size_t)(s) * B + (bb)) * NH + (n)) * D + (e)]
#define DG(bb, g, n, e) dg[(((size_t)(bb) * G + (g)) * NH + (n)) * D + (e)]

    for (int t = T; t >= 1; --t) {
        /* (a) point-wise part: dg_t, dWx_t and the point-wise carries, eq. (3) and left term of eq. (4) */
#pragma omp parallel
        {
            double* y = (double*)malloc(sizeof(double) * G * D);
#pragma omp for collapse(2) schedule(static)
            for (int bb = 0; bb < B; ++bb) {
                for (int n = 0; n < NH; ++n) {
                    recurrent_product(D, G, R + (size_t)n * D * G * D, &ST(t - 1, 0, bb, n, 0), y);
                    for (int e = 0; e < D; ++e) {
                        const double dh = DS(0, bb, n, e) + dH[(((size_t)(t - 1) * B + bb) * NH + n) * D + e];
                        if (cell == CELL_LSTM) {
                            const double i = sigm(WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e));
                            const double f = sigm(WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e));
                            const double z = tanh(WX(t - 1, bb, 2, n, e) + y[2 * D + e] + BI(n, 2, e));
                            const double o = sigm(WX(t - 1, bb, 3, n, e) + y[3 * D + e] + BI(n, 3, e));
                            const double tc = tanh(ST(t, 1, bb, n, e));
                            const double dc = DS(1, bb, n, e) + dh * o * (1.0 - tc * tc);
                            const double di = dc * z * i * (1.0 - i);
                            const double df = dc * ST(t - 1, 1, bb, n, e) * f * (1.0 - f);
                            const double dz = dc * i * (1.0 - z * z);
                            const double dout = dh * tc * o * (1.0 - o);
                            DG(bb, 0, n, e) = di; DG(bb, 1, n, e) = df; DG(bb, 2, n, e) = dz; DG(bb, 3, n, e) = dout;
                            DWX(t - 1, bb, 0, n, e) = di; DWX(t - 1, bb, 1, n, e) = df;
                            DWX(t - 1, bb, 2, n, e) = dz; DWX(t - 1, bb, 3, n, e) = dout;
                            DS(1, bb, n, e) = dc * f;
                            DS(0, bb, n, e) = 0.0; /* h_{t-1} enters step t only through R */
                        } else if (cell == CELL_SLSTM) {
                            const double pi = WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e);
                            const double pf = WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e);
                            const double z = tanh(WX(t - 1, bb, 2, n, e) + y[2 * D + e] + BI(n, 2, e));
                            const double o = sigm(WX(t - 1, bb, 3, n, e) + y[3 * D + e] + BI(n, 3, e));
                            const double m_prev = ST(t - 1, 3, bb, n, e), m = ST(t, 3, bb, n, e);
                            const double c = ST(t, 1, bb, n, e), nn = ST(t, 2, bb, n, e);
                            const double fg = exp(logsigm(pf) + m_prev - m);
                            const double ig = exp(pi - m);
                            const double dc = DS(1, bb, n, e) + dh * o / nn;
                            const double dn = DS(2, bb, n, e) - dh * o * c / (nn * nn);
                            const double di = (dc * z + dn) * ig;
                            const double df = (dc * ST(t - 1, 1, bb, n, e) + dn * ST(t - 1, 2, bb, n, e)) * fg * sigm(-pf);
                            const double dz = dc * ig * (1.0 - z * z);
                            const double dout = dh * (c / nn) * o * (1.0 - o);
                            DG(bb, 0, n, e) = di; DG(bb, 1, n, e) = df; DG(bb, 2, n, e) = dz; DG(bb, 3, n, e) = dout;
                            DWX(t - 1, bb, 0, n, e) = di; DWX(t - 1, bb, 1, n, e) = df;
                            DWX(t - 1, bb, 2, n, e) = dz; DWX(t - 1, bb, 3, n, e) = dout;
                            DS(1, bb, n, e) = dc * fg;
                            DS(2, bb, n, e) = dn * fg;
                            DS(0, bb, n, e) = 0.0;
                        } else if (cell == CELL_GRU4) {
                            const double z = sigm(WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e));
                            const double r = sigm(WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e));
                            const double pn = WX(t - 1, bb, 2, n, e) + y[2 * D + e] + BI(n, 2, e);
                            const double tg = tanh(WX(t - 1, bb, 3, n, e) + y[3 * D + e] + BI(n, 3, e));
                            const double cand = tanh(pn + r * tg);
                            const double dpre = dh * (1.0 - z) * (1.0 - cand * cand);
                            const double dz = dh * (ST(t - 1, 0, bb, n, e) - cand) * z * (1.0 - z);
                            const double dr = dpre * tg * r * (1.0 - r);
                            const double dgg = dpre * r * (1.0 - tg * tg);
                            DG(bb, 0, n, e) = dz; DG(bb, 1, n, e) = dr; DG(bb, 2, n, e) = dpre; DG(bb, 3, n, e) = dgg;
                            DWX(t - 1, bb, 0, n, e) = dz; DWX(t - 1, bb, 1, n, e) = dr;
                            DWX(t - 1, bb, 2, n, e) = dpre; DWX(t - 1, bb, 3, n, e) = dgg;
                            DS(0, bb, n, e) = dh * z; /* direct path h_{t-1} -> h_t */
                        } else if (cell == CELL_ELMAN) {
                            const double h = tanh(WX(t - 1, bb, 0, n, e) + y[e] + BI(n, 0, e));
                            const double dpre = dh * (1.0 - h * h);
                            DWX(t - 1, bb, 0, n, e) = dpre;
                            DG(bb, 0, n, e) = dpre;
                            DS(0, bb, n, e) = 0.0; /* h_{t-1} enters step t only through R */
                        } else { /* GRU */
                            const double r = sigm(WX(t - 1, bb, 0, n, e) + y[0 * D + e] + BI(n, 0, e));
                            const double z = sigm(WX(t - 1, bb, 1, n, e) + y[1 * D + e] + BI(n, 1, e));
                            const double yn = y[2 * D + e] + BI(n, 2, e);
                            const double cand = tanh(WX(t - 1, bb, 2, n, e) + r * yn);
                            const double dpre = dh * (1.0 - z) * (1.0 - cand * cand);
                            const double dz = dh * (ST(t - 1, 0, bb, n, e) - cand) * z * (1.0 - z);
                            const double dr = dpre * yn * r * (1.0 - r);
                            DWX(t - 1, bb, 0, n, e) = dr; DWX(t - 1, bb, 1, n, e) = dz; DWX(t - 1, bb, 2, n, e) = dpre;
                            DG(bb, 0, n, e) = dr; DG(bb, 1, n, e) = dz; DG(bb, 2, n, e) = dpre * r;
                            DS(0, bb, n, e) = dh * z; /* direct path h_{t-1} -> h_t */
                        }
                    }
                }
            }
            free(y);
        }
        /* (b) recurrent part: dh_{t-1} += R dg_t (right term of eq. (4)); dR += h_{t-1} (x) dg_t; db += dg_t */
#pragma omp parallel for collapse(2) schedule(static)
        for (int n = 0; n < NH; ++n) {
            for (int d = 0; d < D; ++d) {
                const double* Rrow = R + ((size_t)n * D + d) * G * D;
                double* dRrow = dR + ((size_t)n * D + d) * G * D;
                for (int bb = 0; bb < B; ++bb) {
                    const double hp = ST(t - 1, 0, bb, n, d);
                    double acc = 0.0;
                    for (int g = 0; g < G; ++g)
                        for (int e = 0; e < D; ++e) {
                            const double v = DG(bb, g, n, e);
                            acc += Rrow[g * D + e] * v;
                            dRrow[g * D + e] += hp * v;
                        }
                    /* Sec. 4.1: the term that contains the recurrent matrix may be clipped, value by value, after
                       each time step (recurrent_clip < 0: not clipped; 0 cuts it to zero) */
                    dh_prev[((size_t)bb * NH + n) * D + d] = recurrent_clip >= 0.0 ? fmin(fmax(acc, -recurrent_clip), recurrent_clip) : acc;
                }
            }
        }
#pragma omp parallel for collapse(2) schedule(static)
        for (int n = 0; n < NH; ++n)
            for (int g = 0; g < G; ++g)
                for (int e = 0; e < D; ++e) {
                    double acc = 0.0;
                    for (int bb = 0; bb < B; ++bb) acc += DG(bb, g, n, e);
                    db[((size_t)n * G + g) * D + e] += acc;
                }
        for (size_t j = 0; j < BHD; ++j) ds[j] += dh_prev[j];
    }
    memcpy(dstates0, ds, (size_t)S * BHD * sizeof(double));
    if (cell == CELL_SLSTM) memset(dstates0 + 3 * BHD, 0, BHD * sizeof(double));
    free(ds); free(dg); free(dh_prev);
    return 0;
}

int oracle_bwd(int cell, int T, int B, int NH, int D, const double* Wx, const double* R, const double* bias,
               const double* states, const double* dH, const double* dstates_last, double* dWx, double* dR,
               double* db, double* dstates0) {
    return oracle_bwd_clipped(cell, T, B, NH, D, Wx, R, bias, states, dH, dstates_last, -1.0, dWx, dR, db, dstates0);
}
