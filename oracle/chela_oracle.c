/*
 * chela_oracle.c -- TEST INFRASTRUCTURE, not part of the product path.
 *
 * Plain, slow, fp64 CPU definition of causal (un-normalised) linear attention,
 *     O_t = sum_{s<=t} (q_t . k_s) v_s ,
 * i.e. the right-product linear attention of CHELA Sec. 2.1 Eq. 2 with the
 * lower-triangular (inclusive) mask that Sec. 4.1 applies inside a block, and
 * with Norm, scaling and feature maps left outside (the kernel's contract).
 * Sec. 4.1 describes a tiled evaluation of exactly this quantity ("lossless",
 * Sec. 4.4), so the oracle is the untiled definition written out twice:
 *
 *   quadratic form : the masked N x N score matrix applied to V, row by row;
 *   recurrent form : the token-by-token running sum of k v^T (the "cumsum"
 *                    formulation that Sec. 1 and Sec. 3 name as the baseline).
 *
 * No chunking, no blocking, no fusion: every loop below is the formula.
 * The backward pass is not described in the paper; it is the exact gradient of
 * the definition above (O is linear in each of Q, K and V separately).
 *
 * Layout: every tensor is [B, H, N, d] contiguous, d fastest; Q, K use d = dk,
 * V, O, dO, dV use d = dv.  All arithmetic is IEEE double.  The only
 * parallelism is OpenMP over the independent (b, h) pairs.
 *
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
 * call this library.  It shares no code with the HIP library.
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int chela_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- quadratic (masked parallel) form: Eq. 2 + causal mask of Sec. 4.1 ---- */
/* A[t,s] = q_t . k_s for s <= t, else 0 ;  O[t,:] = sum_s A[t,s] V[s,:].     */
void chela_oracle_fwd_quadratic(const double *Q, const double *K, const double *V,
                                double *O, int B, int H, int N, int dk, int dv)
{
    const long BH = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * (long)N * dk;
        const double *k = K + bh * (long)N * dk;
        const double *v = V + bh * (long)N * dv;
        double *o = O + bh * (long)N * dv;
        for (int t = 0; t < N; ++t) {
            for (int j = 0; j < dv; ++j) o[(long)t * dv + j] = 0.0;
            for (int s = 0; s <= t; ++s) {
                double a = 0.0;
                for (int i = 0; i < dk; ++i) a += q[(long)t * dk + i] * k[(long)s * dk + i];
                for (int j = 0; j < dv; ++j) o[(long)t * dv + j] += a * v[(long)s * dv + j];
            }
        }
    }
}

/* Gradient of the quadratic form.  With A as above and                        */
/* dA[t,s] = dO_t . v_s for s <= t, else 0:                                    */
/*   dQ = dA K,   dK = dA^T Q,   dV = A^T dO.                                  */
void chela_oracle_bwd_quadratic(const double *Q, const double *K, const double *V,
                                const double *dO, double *dQ, double *dK, double *dV,
                                int B, int H, int N, int dk, int dv)
{
    const long BH = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * (long)N * dk;
        const double *k = K + bh * (long)N * dk;
        const double *v = V + bh * (long)N * dv;
        const double *g = dO + bh * (long)N * dv;
        double *dq = dQ + bh * (long)N * dk;
        double *dkk = dK + bh * (long)N * dk;
        double *dvv = dV + bh * (long)N * dv;
        memset(dq, 0, sizeof(double) * (size_t)N * dk);
        memset(dkk, 0, sizeof(double) * (size_t)N * dk);
        memset(dvv, 0, sizeof(double) * (size_t)N * dv);
        for (int t = 0; t < N; ++t) {
            for (int s = 0; s <= t; ++s) {
                double a = 0.0, da = 0.0;
                for (int i = 0; i < dk; ++i) a += q[(long)t * dk + i] * k[(long)s * dk + i];
                for (int j = 0; j < dv; ++j) da += g[(long)t * dv + j] * v[(long)s * dv + j];
                for (int i = 0; i < dk; ++i) dq[(long)t * dk + i] += da * k[(long)s * dk + i];
                for (int i = 0; i < dk; ++i) dkk[(long)s * dk + i] += da * q[(long)t * dk + i];
                for (int j = 0; j < dv; ++j) dvv[(long)s * dv + j] += a * g[(long)t * dv + j];
            }
        }
    }
}

/* ---- recurrent (token-by-token) form: the running KV state of Sec. 4.1 ---- */
/* S <- 0 (dk x dv); for t = 0..N-1:  S += k_t v_t^T ;  o_t = S^T q_t.         */
void chela_oracle_fwd_recurrent(const double *Q, const double *K, const double *V,
                                double *O, int B, int H, int N, int dk, int dv)
{
    const long BH = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * (long)N * dk;
        const double *k = K + bh * (long)N * dk;
        const double *v = V + bh * (long)N * dv;
        double *o = O + bh * (long)N * dv;
        double *S = (double *)calloc((size_t)dk * dv, sizeof(double));
        for (int t = 0; t < N; ++t) {
            for (int i = 0; i < dk; ++i)
                for (int j = 0; j < dv; ++j)
                    S[(long)i * dv + j] += k[(long)t * dk + i] * v[(long)t * dv + j];
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < dk; ++i) acc += S[(long)i * dv + j] * q[(long)t * dk + i];
                o[(long)t * dv + j] = acc;
            }
        }
        free(S);
    }
}

/* Gradient in recurrent form.                                                 */
/* Forward sweep : S_t = S_{t-1} + k_t v_t^T ;  dq_t = S_t dO_t.               */
/* Reverse sweep : R_t = R_{t+1} + q_t dO_t^T ; dk_t = R_t v_t ; dv_t = R_t^T k_t. */
void chela_oracle_bwd_recurrent(const double *Q, const double *K, const double *V,
                                const double *dO, double *dQ, double *dK, double *dV,
                                int B, int H, int N, int dk, int dv)
{
    const long BH = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * (long)N * dk;
        const double *k = K + bh * (long)N * dk;
        const double *v = V + bh * (long)N * dv;
        const double *g = dO + bh * (long)N * dv;
        double *dq = dQ + bh * (long)N * dk;
        double *dkk = dK + bh * (long)N * dk;
        double *dvv = dV + bh * (long)N * dv;
        double *S = (double *)calloc((size_t)dk * dv, sizeof(double));
        for (int t = 0; t < N; ++t) {
            for (int i = 0; i < dk; ++i)
                for (int j = 0; j < dv; ++j)
                    S[(long)i * dv + j] += k[(long)t * dk + i] * v[(long)t * dv + j];
            for (int i = 0; i < dk; ++i) {
                double acc = 0.0;
                for (int j = 0; j < dv; ++j) acc += S[(long)i * dv + j] * g[(long)t * dv + j];
                dq[(long)t * dk + i] = acc;
            }
        }
        memset(S, 0, sizeof(double) * (size_t)dk * dv);   /* S now plays the role of R */
        for (int t = N - 1; t >= 0; --t) {
            for (int i = 0; i < dk; ++i)
                for (int j = 0; j < dv; ++j)
                    S[(long)i * dv + j] += q[(long)t * dk + i] * g[(long)t * dv + j];
            for (int i = 0; i < dk; ++i) {
                double acc = 0.0;
                for (int j = 0; j < dv; ++j) acc += S[(long)i * dv + j] * v[(long)t * dv + j];
                dkk[(long)t * dk + i] = acc;
            }
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < dk; ++i) acc += S[(long)i * dv + j] * k[(long)t * dk + i];
                dvv[(long)t * dv + j] = acc;
            }
        }
        free(S);
    }
}

/* ==========================================================================
 * State carry-in / carry-out (segment-wise processing, Sec. 5.3 and App. A:
 * training data is split into segments of consecutive chunks and test data
 * is processed segment by segment).  The running state of the recurrent form
 * is the only thing one segment hands to the next:
 *
 *     S_0 = S_in ;  S_t = S_{t-1} + k_t v_t^T ;  o_t = S_t^T q_t ;  S_out = S_N .
 *
 * S_in, S_out: [B, H, dk, dv].  A NULL S_in means zero; a NULL S_out is not
 * written.  With S_in = NULL and S_out = NULL this is chela_oracle_fwd_recurrent.
 * ========================================================================== */
void chela_oracle_fwd_state(const double *Q, const double *K, const double *V, const double *S_in,
                            double *O, double *S_out, int B, int H, int N, int dk, int dv)
{
    const long BH = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * (long)N * dk;
        const double *k = K + bh * (long)N * dk;
        const double *v = V + bh * (long)N * dv;
        double *o = O + bh * (long)N * dv;
        double *S = (double *)calloc((size_t)dk * dv, sizeof(double));
        if (S_in) memcpy(S, S_in + bh * (long)dk * dv, sizeof(double) * (size_t)dk * dv);
        for (int t = 0; t < N; ++t) {
            for (int i = 0; i < dk; ++i)
                for (int j = 0; j < dv; ++j)
                    S[(long)i * dv + j] += k[(long)t * dk + i] * v[(long)t * dv + j];
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < dk; ++i) acc += S[(long)i * dv + j] * q[(long)t * dk + i];
                o[(long)t * dv + j] = acc;
            }
        }
        if (S_out) memcpy(S_out + bh * (long)dk * dv, S, sizeof(double) * (size_t)dk * dv);
        free(S);
    }
}

/* Gradient of the map (Q, K, V, S_in) -> (O, S_out) for upstream gradients dO and dS_out (NULL = zero).
 * Forward sweep : S_t as above ;  dq_t = S_t dO_t.
 * Reverse sweep : R_{N+1} = dS_out ;  R_t = R_{t+1} + q_t dO_t^T ;  dk_t = R_t v_t ;  dv_t = R_t^T k_t.
 * dS_in = R_1 (every later state contains S_in once).  A NULL dS_in is not written. */
void chela_oracle_bwd_state(const double *Q, const double *K, const double *V, const double *S_in,
                            const double *dO, const double *dS_out, double *dQ, double *dK, double *dV,
                            double *dS_in, int B, int H, int N, int dk, int dv)
{
    const long BH = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < BH; ++bh) {
        const double *q = Q + bh * (long)N * dk;
        const double *k = K + bh * (long)N * dk;
        const double *v = V + bh * (long)N * dv;
        const double *g = dO + bh * (long)N * dv;
        double *dq = dQ + bh * (long)N * dk;
        double *dkk = dK + bh * (long)N * dk;
        double *dvv = dV + bh * (long)N * dv;
        double *S = (double *)calloc((size_t)dk * dv, sizeof(double));
        if (S_in) memcpy(S, S_in + bh * (long)dk * dv, sizeof(double) * (size_t)dk * dv);
        for (int t = 0; t < N; ++t) {
            for (int i = 0; i < dk; ++i)
                for (int j = 0; j < dv; ++j)
                    S[(long)i * dv + j] += k[(long)t * dk + i] * v[(long)t * dv + j];
            for (int i = 0; i < dk; ++i) {
                double acc = 0.0;
                for (int j = 0; j < dv; ++j) acc += S[(long)i * dv + j] * g[(long)t * dv + j];
                dq[(long)t * dk + i] = acc;
            }
        }
        memset(S, 0, sizeof(double) * (size_t)dk * dv);   /* S now plays the role of R */
        if (dS_out) memcpy(S, dS_out + bh * (long)dk * dv, sizeof(double) * (size_t)dk * dv);
        for (int t = N - 1; t >= 0; --t) {
            for (int i = 0; i < dk; ++i)
                for (int j = 0; j < dv; ++j)
                    S[(long)i * dv + j] += q[(long)t * dk + i] * g[(long)t * dv + j];
            for (int i = 0; i < dk; ++i) {
                double acc = 0.0;
                for (int j = 0; j < dv; ++j) acc += S[(long)i * dv + j] * v[(long)t * dv + j];
                dkk[(long)t * dk + i] = acc;
            }
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < dk; ++i) acc += S[(long)i * dv + j] * k[(long)t * dk + i];
                dvv[(long)t * dv + j] = acc;
            }
        }
        if (dS_in) memcpy(dS_in + bh * (long)dk * dv, S, sizeof(double) * (size_t)dk * dv);
        free(S);
    }
}

/* One decode step (autoregressive inference): S += k v^T ; o = S^T q, for every (b, h).
 * q, k: [B, H, dk]; v, o: [B, H, dv]; S: [B, H, dk, dv], updated in place. */
void chela_oracle_step(const double *q, const double *k, const double *v, double *S, double *o,
                       int B, int H, int dk, int dv)
{
    const long BH = (long)B * H;
    for (long bh = 0; bh < BH; ++bh) {
        double *s = S + bh * (long)dk * dv;
        for (int i = 0; i < dk; ++i)
            for (int j = 0; j < dv; ++j) s[(long)i * dv + j] += k[bh * dk + i] * v[bh * dv + j];
        for (int j = 0; j < dv; ++j) {
            double acc = 0.0;
            for (int i = 0; i < dk; ++i) acc += s[(long)i * dv + j] * q[bh * dk + i];
            o[bh * dv + j] = acc;
        }
    }
}

/* ======================================================================================================
 * Short-long convolutions, CHELA Sec. 4.2 Eq. 8:  Z = K_l( silu( K_s(X) ) ).
 * Depthwise (one kernel per channel), causal, zero history; tensors are [B][d][L] (time fastest).
 *   K_s : short kernel w[c][0..m-1]   (the paper's two parallel short kernels, of size 3 and 2 log10(L) + 1,
 *         summed tap by tap into one -- the structural re-parameterisation the section describes);
 *   silu: x / (1 + exp(-x));
 *   K_l : long kernel k[c][0..L-1], as long as the sequence (Sec. 2.3, "Long convolution").
 * Eq. 7 evaluates K_l by FFT; what it evaluates is the convolution sum, which is written out here:
 *   y[t] = sum_{s=0..t} k[s] * v[t-s].
 * O(L^2) per channel on purpose.
 * ====================================================================================================== */
#include <math.h>

/* V[b][c][t] = act( sum_{j=0..min(m-1,t)} w[c][j] * X[b][c][t-j] ),  act = silu if apply_silu else identity */
void chela_oracle_short_conv(const double *X, const double *w, double *V, int B, int d, int L, int m,
                             int apply_silu)
{
    const long BD = (long)B * d;
#pragma omp parallel for schedule(static)
    for (long bc = 0; bc < BD; ++bc) {
        const int c = (int)(bc % d);
        const double *x = X + bc * (long)L;
        double *v = V + bc * (long)L;
        for (int t = 0; t < L; ++t) {
            double a = 0.0;
            for (int j = 0; j < m && j <= t; ++j) a += w[(long)c * m + j] * x[t - j];
            v[t] = apply_silu ? a / (1.0 + exp(-a)) : a;
        }
    }
}

/* Y[b][c][t] = sum_{s=0..t} k[c][s] * V[b][c][t-s] */
void chela_oracle_long_conv(const double *V, const double *k, double *Y, int B, int d, int L)
{
    const long BD = (long)B * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (long bc = 0; bc < BD; ++bc) {
        const int c = (int)(bc % d);
        const double *v = V + bc * (long)L;
        const double *kc = k + (long)c * L;
        double *y = Y + bc * (long)L;
        for (int t = 0; t < L; ++t) {
            double a = 0.0;
            for (int s = 0; s <= t; ++s) a += kc[s] * v[t - s];
            y[t] = a;
        }
    }
}

/* Gradient of Z = K_l( silu( K_s(X) ) ) for an upstream gradient dZ (the paper gives no backward; this is the
 * exact gradient of the two sums above).  U = K_s(X) before the activation, V = silu(U).
 *   dV[b,c,t] = sum_{s>=t} k[c][s-t] dZ[b,c,s]
 *   dk[c][s]  = sum_b sum_{t>=s} dZ[b,c,t] V[b,c,t-s]
 *   dU        = dV * silu'(U),  silu'(u) = sig(u) (1 + u (1 - sig(u)))      (dU = dV if there is no short stage)
 *   dX[b,c,t] = sum_{j<m, t+j<L} w[c][j] dU[b,c,t+j]
 *   dw[c][j]  = sum_b sum_{t>=j} dU[b,c,t] X[b,c,t-j]
 * w == NULL: no short stage (V = X, dX = dV, dw untouched). */
void chela_oracle_short_long_conv_bwd(const double *X, const double *w, int m, const double *k, const double *dZ,
                                      double *dX, double *dw, double *dk, int B, int d, int L)
{
    for (long i = 0; i < (long)d * L; ++i) dk[i] = 0.0;
    if (w) for (long i = 0; i < (long)d * m; ++i) dw[i] = 0.0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int c = 0; c < d; ++c) {
        double *U = (double *)malloc(sizeof(double) * (size_t)L * 4);
        double *V = U + L, *dV = V + L, *dU = dV + L;
        for (int b = 0; b < B; ++b) {
            const double *x = X + ((long)b * d + c) * L;
            const double *dz = dZ + ((long)b * d + c) * L;
            double *dx = dX + ((long)b * d + c) * L;
            for (int t = 0; t < L; ++t) {
                if (w) {
                    double a = 0.0;
                    for (int j = 0; j < m && j <= t; ++j) a += w[(long)c * m + j] * x[t - j];
                    U[t] = a;
                    V[t] = a / (1.0 + exp(-a));
                } else {
                    U[t] = V[t] = x[t];
                }
            }
            for (int t = 0; t < L; ++t) {
                double a = 0.0;
                for (int s = t; s < L; ++s) a += k[(long)c * L + (s - t)] * dz[s];
                dV[t] = a;
            }
            for (int s = 0; s < L; ++s) {
                double a = 0.0;
                for (int t = s; t < L; ++t) a += dz[t] * V[t - s];
                dk[(long)c * L + s] += a;
            }
            if (!w) {
                for (int t = 0; t < L; ++t) dx[t] = dV[t];
                continue;
            }
            for (int t = 0; t < L; ++t) {
                const double sg = 1.0 / (1.0 + exp(-U[t]));
                dU[t] = dV[t] * sg * (1.0 + U[t] * (1.0 - sg));
            }
            for (int t = 0; t < L; ++t) {
                double a = 0.0;
                for (int j = 0; j < m && t + j < L; ++j) a += w[(long)c * m + j] * dU[t + j];
                dx[t] = a;
            }
            for (int j = 0; j < m; ++j) {
                double a = 0.0;
                for (int t = j; t < L; ++t) a += dU[t] * x[t - j];
                dw[(long)c * m + j] += a;
            }
        }
        free(U);
    }
}
