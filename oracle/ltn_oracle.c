/*
 * fp64 CPU oracle for Lightning Attention (arXiv 2307.14995).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * readable evaluation of what the GPU library must compute.  Only the test
 * suite, the smoke check and the benchmark's "cpu_baseline" leg may call it.
 * It shares no code, header, table or constant with the HIP library.
 *
 * What is computed (per batch b and head h, independent chains):
 *
 *   Definition (Sec. 3.2.1, "O = (Q K^T (.) M) V"; mask from Eq. 1 without
 *   the LRPE phase, as Sec. 3.3 drops it):
 *       O[t,:] = sum_{s=0..t} lambda_h^(t-s) * (q_t . k_s) * v_s
 *   No 1/sqrt(d) scale, no softmax, no normaliser (Sec. 3.1.3: the attention
 *   "eliminates the softmax and scaling operation").
 *
 *   Recurrent form (Sec. 3.3, Algorithm 2, the robust inference recurrence):
 *       kv_0 = kv_in (zero if absent);  kv_t = lambda*kv_{t-1} + k_t^T v_t;
 *       o_t = q_t kv_t
 *
 *   Gradients: derivative of the definition.  With A = (Q K^T) (.) M:
 *       dV = A^T dO,  dA = (dO V^T) (.) M,  dQ = dA K,  dK = dA^T Q
 *   (App. B, Algorithm 4, read with its evident misprints corrected: dK is
 *   the product of dA^T with Q, dQ accumulates into dQ).
 *
 * Tensor layout: contiguous row-major [Bt, H, N, D] doubles; decay[H]
 * doubles in [0,1]; states [Bt, H, D, D] with kv[i][j] = sum k[i]*v[j]
 * (row = key feature, column = value feature).
 *
 *   Gated, normalised output of the token mixer (Sec. 3.1.2, Eq. 3, with the
 *   SimpleRMSNorm of Sec. 3.1.3 taken per head over its D features):
 *       y = x / sqrt(|x|^2 / D + eps) (.) u      (eps = 0 is the printed formula)
 *   and its derivative with respect to x and u.
 *
 *   Input side (Sec. 3.1.2 Eq. 2: swish on the query/key projections; Sec. 3.1.1
 *   Eq. 1: LRPE-d, the phase exp(i theta (t-s)) on the score), near the end of
 *   this file together with the variants of Algorithm 2 and of the gradients
 *   for a query/key width different from the value width, which LRPE-d needs.
 *
 * Parity pins live in tests/test_oracle_pins.py (brute force, closed forms,
 * cumulative-sum special case, finite differences, Algorithm 1 == Algorithm 2
 * identity of App. C, block-form re-association).  Nothing is "parity unpinned".
 *
 * Parallelism: OpenMP over (b,h) only.  No blocking or reordering beyond what
 * each formula states.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef long long i64;

/* lambda^n for integer n >= 0 with the convention 0^0 = 1 (M[t,t] = 1 for every
 * lambda, Eq. 1 at s = t). */
static double decay_pow(double lam, i64 n) {
    if (n == 0) return 1.0;
    return pow(lam, (double)n);
}

int ltn_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void ltn_oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------ */
/* Forward, quadratic masked-matrix form: the definition written out.        */
/* Sec. 3.2.1: O = (Q K^T (.) M) V,  M[t,s] = lambda^(t-s) for t >= s.       */
/* ------------------------------------------------------------------------ */
void ltn_oracle_fwd_quadratic(const double* q, const double* k, const double* v,
                              const double* decay, int Bt, int H, i64 N, int D,
                              double* o) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        double* O = o + c * N * D;
        for (i64 t = 0; t < N; ++t) {
            for (int j = 0; j < D; ++j) O[t * D + j] = 0.0;
            for (i64 s = 0; s <= t; ++s) {
                double dot = 0.0;
                for (int i = 0; i < D; ++i) dot += Q[t * D + i] * K[s * D + i];
                const double a = dot * decay_pow(lam, t - s); /* A[t,s] */
                for (int j = 0; j < D; ++j) O[t * D + j] += a * V[s * D + j];
            }
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Forward, recurrent form: Algorithm 2 (Sec. 3.3), token by token.          */
/* kv_in / kv_out may be NULL (zero initial state / state not returned).     */
/* ------------------------------------------------------------------------ */
void ltn_oracle_fwd_recurrent(const double* q, const double* k, const double* v,
                              const double* decay, const double* kv_in,
                              int Bt, int H, i64 N, int D,
                              double* o, double* kv_out) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        double* O = o + c * N * D;
        double* kv = (double*)malloc(sizeof(double) * D * D);
        if (kv_in) memcpy(kv, kv_in + c * D * D, sizeof(double) * D * D);
        else memset(kv, 0, sizeof(double) * D * D);
        for (i64 t = 0; t < N; ++t) {
            /* kv_t = lambda kv_{t-1} + k_t^T v_t */
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j)
                    kv[i * D + j] = lam * kv[i * D + j] + K[t * D + i] * V[t * D + j];
            /* o_t = q_t kv_t */
            for (int j = 0; j < D; ++j) {
                double acc = 0.0;
                for (int i = 0; i < D; ++i) acc += Q[t * D + i] * kv[i * D + j];
                O[t * D + j] = acc;
            }
        }
        if (kv_out) memcpy(kv_out + c * D * D, kv, sizeof(double) * D * D);
        free(kv);
    }
}

/* ------------------------------------------------------------------------ */
/* Algorithm 1 (Sec. 3.3), the "origin" recurrence that factors the mask as   */
/* (q lambda^t)(k lambda^-t).  Kept only to test the identity of App. C,      */
/* kv_t = lambda^-t kvbar_t, and to show why no kernel may use this form.     */
/* Tokens are numbered t = 1..N as in the paper.  Returns the final state.    */
/* ------------------------------------------------------------------------ */
void ltn_oracle_fwd_origin(const double* q, const double* k, const double* v,
                           const double* decay, int Bt, int H, i64 N, int D,
                           double* o, double* kv_out) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        double* O = o + c * N * D;
        double* kv = (double*)calloc((size_t)D * D, sizeof(double));
        for (i64 t = 1; t <= N; ++t) {
            const double up = pow(lam, -(double)t);
            const double dn = pow(lam, (double)t);
            const i64 r = t - 1;
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j)
                    kv[i * D + j] += K[r * D + i] * up * V[r * D + j];
            for (int j = 0; j < D; ++j) {
                double acc = 0.0;
                for (int i = 0; i < D; ++i) acc += Q[r * D + i] * dn * kv[i * D + j];
                O[r * D + j] = acc;
            }
        }
        if (kv_out) memcpy(kv_out + c * D * D, kv, sizeof(double) * D * D);
        free(kv);
    }
}

/* ------------------------------------------------------------------------ */
/* Forward, paper's tiling (App. B, Algorithm 3): for each query block i,     */
/* loop over every key/value block j, A_ij = (Q_i K_j^T) (.) M_ij,            */
/* O_i += A_ij V_j.  Br and Bc may differ and need not divide N (the paper    */
/* assumes they do; a short last block is simply shorter).                    */
/* ------------------------------------------------------------------------ */
void ltn_oracle_fwd_tiled(const double* q, const double* k, const double* v,
                          const double* decay, int Bt, int H, i64 N, int D,
                          int Br, int Bc, double* o) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        double* O = o + c * N * D;
        double* A = (double*)malloc(sizeof(double) * Br * Bc);
        for (i64 i0 = 0; i0 < N; i0 += Br) {
            const i64 nr = (N - i0 < Br) ? (N - i0) : Br;
            for (i64 r = 0; r < nr; ++r)
                for (int j = 0; j < D; ++j) O[(i0 + r) * D + j] = 0.0;
            for (i64 j0 = 0; j0 < N; j0 += Bc) {
                const i64 nc = (N - j0 < Bc) ? (N - j0) : Bc;
                for (i64 r = 0; r < nr; ++r)
                    for (i64 cc = 0; cc < nc; ++cc) {
                        const i64 t = i0 + r, s = j0 + cc;
                        double m = (t >= s) ? decay_pow(lam, t - s) : 0.0; /* M_ij */
                        double dot = 0.0;
                        for (int i = 0; i < D; ++i) dot += Q[t * D + i] * K[s * D + i];
                        A[r * Bc + cc] = dot * m;
                    }
                for (i64 r = 0; r < nr; ++r)
                    for (i64 cc = 0; cc < nc; ++cc)
                        for (int j = 0; j < D; ++j)
                            O[(i0 + r) * D + j] += A[r * Bc + cc] * V[(j0 + cc) * D + j];
            }
        }
        free(A);
    }
}

/* ------------------------------------------------------------------------ */
/* Forward, block form: the intra-block masked tile plus the lambda-scaled    */
/* product with a running D x D state.  This is the re-association that a     */
/* blockwise kernel performs, evaluated literally in fp64:                     */
/*   S = Q_i K_i^T; A = S (.) M_B; O_i = A V_i + diag(lambda^(r+1)) Q_i KV_i   */
/*   KV_{i+1} = lambda^len KV_i + sum_c lambda^(len-1-c) k_c^T v_c             */
/* with len the number of tokens in block i.  Only non-negative exponents.    */
/* It validates the decay exponents before any kernel exists.                  */
/* ------------------------------------------------------------------------ */
void ltn_oracle_fwd_block(const double* q, const double* k, const double* v,
                          const double* decay, const double* kv_in,
                          int Bt, int H, i64 N, int D, int block,
                          double* o, double* kv_out) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        double* O = o + c * N * D;
        double* kv = (double*)malloc(sizeof(double) * D * D);
        double* nk = (double*)malloc(sizeof(double) * D * D);
        double* A = (double*)malloc(sizeof(double) * block * block);
        if (kv_in) memcpy(kv, kv_in + c * D * D, sizeof(double) * D * D);
        else memset(kv, 0, sizeof(double) * D * D);
        for (i64 b0 = 0; b0 < N; b0 += block) {
            const i64 len = (N - b0 < block) ? (N - b0) : block;
            /* intra scores and mask */
            for (i64 r = 0; r < len; ++r)
                for (i64 cc = 0; cc < len; ++cc) {
                    double dot = 0.0;
                    for (int i = 0; i < D; ++i) dot += Q[(b0 + r) * D + i] * K[(b0 + cc) * D + i];
                    A[r * block + cc] = (r >= cc) ? dot * decay_pow(lam, r - cc) : 0.0;
                }
            /* intra output + inter output */
            for (i64 r = 0; r < len; ++r) {
                const double lq = decay_pow(lam, r + 1);
                for (int j = 0; j < D; ++j) {
                    double intra = 0.0;
                    for (i64 cc = 0; cc < len; ++cc) intra += A[r * block + cc] * V[(b0 + cc) * D + j];
                    double inter = 0.0;
                    for (int i = 0; i < D; ++i) inter += Q[(b0 + r) * D + i] * kv[i * D + j];
                    O[(b0 + r) * D + j] = intra + lq * inter;
                }
            }
            /* state update */
            const double lb = decay_pow(lam, len);
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j) {
                    double acc = 0.0;
                    for (i64 cc = 0; cc < len; ++cc)
                        acc += decay_pow(lam, len - 1 - cc) * K[(b0 + cc) * D + i] * V[(b0 + cc) * D + j];
                    nk[i * D + j] = lb * kv[i * D + j] + acc;
                }
            memcpy(kv, nk, sizeof(double) * D * D);
        }
        if (kv_out) memcpy(kv_out + c * D * D, kv, sizeof(double) * D * D);
        free(A); free(nk); free(kv);
    }
}

/* ------------------------------------------------------------------------ */
/* Backward, quadratic form: materialise A and dA per chain.                  */
/*   dV = A^T dO;  dA = (dO V^T) (.) M;  dQ = dA K;  dK = dA^T Q              */
/* ------------------------------------------------------------------------ */
void ltn_oracle_bwd_quadratic(const double* q, const double* k, const double* v,
                              const double* d_o, const double* decay,
                              int Bt, int H, i64 N, int D,
                              double* dq, double* dk, double* dv) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        const double* G = d_o + c * N * D;
        double* DQ = dq + c * N * D;
        double* DK = dk + c * N * D;
        double* DV = dv + c * N * D;
        memset(DQ, 0, sizeof(double) * N * D);
        memset(DK, 0, sizeof(double) * N * D);
        memset(DV, 0, sizeof(double) * N * D);
        for (i64 t = 0; t < N; ++t)
            for (i64 s = 0; s <= t; ++s) {
                const double m = decay_pow(lam, t - s); /* M[t,s] */
                double qk = 0.0, gv = 0.0;
                for (int i = 0; i < D; ++i) {
                    qk += Q[t * D + i] * K[s * D + i];
                    gv += G[t * D + i] * V[s * D + i];
                }
                const double a = qk * m;  /* A[t,s]  */
                const double da = gv * m; /* dA[t,s] */
                for (int j = 0; j < D; ++j) {
                    DV[s * D + j] += a * G[t * D + j];
                    DQ[t * D + j] += da * K[s * D + j];
                    DK[s * D + j] += da * Q[t * D + j];
                }
            }
    }
}

/* ------------------------------------------------------------------------ */
/* Backward, recurrent form.                                                   */
/* Forward sweep re-runs Algorithm 2's state and emits dq_t = dO_t kv_t^T.    */
/* Reverse sweep carries dkv (same shape as kv): for t = N-1..0               */
/*   dkv = lambda dkv + q_t^T dO_t;  dk_t = v_t dkv^T;  dv_t = k_t dkv         */
/* (state updated before use, so the diagonal term s = t is included).         */
/* ------------------------------------------------------------------------ */
void ltn_oracle_bwd_recurrent(const double* q, const double* k, const double* v,
                              const double* d_o, const double* decay,
                              int Bt, int H, i64 N, int D,
                              double* dq, double* dk, double* dv) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        const double* G = d_o + c * N * D;
        double* DQ = dq + c * N * D;
        double* DK = dk + c * N * D;
        double* DV = dv + c * N * D;
        double* kv = (double*)calloc((size_t)D * D, sizeof(double));
        for (i64 t = 0; t < N; ++t) {
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j)
                    kv[i * D + j] = lam * kv[i * D + j] + K[t * D + i] * V[t * D + j];
            for (int i = 0; i < D; ++i) {
                double acc = 0.0;
                for (int j = 0; j < D; ++j) acc += G[t * D + j] * kv[i * D + j];
                DQ[t * D + i] = acc;
            }
        }
        memset(kv, 0, sizeof(double) * D * D); /* now the suffix state dkv */
        for (i64 t = N - 1; t >= 0; --t) {
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j)
                    kv[i * D + j] = lam * kv[i * D + j] + Q[t * D + i] * G[t * D + j];
            for (int i = 0; i < D; ++i) {
                double acc = 0.0;
                for (int j = 0; j < D; ++j) acc += V[t * D + j] * kv[i * D + j];
                DK[t * D + i] = acc;
            }
            for (int j = 0; j < D; ++j) {
                double acc = 0.0;
                for (int i = 0; i < D; ++i) acc += K[t * D + i] * kv[i * D + j];
                DV[t * D + j] = acc;
            }
        }
        free(kv);
    }
}

/* ------------------------------------------------------------------------ */
/* Backward, block form (forward-order sweep for dQ with the prefix state,    */
/* reverse-order sweep for dK, dV with the suffix state), evaluated literally */
/* in fp64 with non-negative decay exponents only:                             */
/*   forward sweep, block i with KV_i:                                         */
/*     dA = (dO_i V_i^T) (.) M_B;  dQ_i = dA K_i + diag(lambda^(r+1)) dO_i KV_i^T */
/*     KV_{i+1} as in the forward block form                                   */
/*   reverse sweep, block i with dKV_i (suffix state as seen from the block's  */
/*   end: sum over later tokens t of lambda^(t - end) q_t^T dO_t, end = first  */
/*   token after the block):                                                    */
/*     A = (Q_i K_i^T) (.) M_B                                                  */
/*     dV_i = A^T dO_i + diag(lambda^(len-c)) K_i dKV_i                         */
/*     dK_i = dA^T Q_i + diag(lambda^(len-c)) V_i dKV_i^T                       */
/*     dKV_{i-1} = lambda^len dKV_i + sum_r lambda^r q_r^T dO_r                 */
/* ------------------------------------------------------------------------ */
void ltn_oracle_bwd_block(const double* q, const double* k, const double* v,
                          const double* d_o, const double* decay,
                          int Bt, int H, i64 N, int D, int block,
                          double* dq, double* dk, double* dv) {
    const i64 chains = (i64)Bt * H;
    const i64 T = (N + block - 1) / block;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        const double* G = d_o + c * N * D;
        double* DQ = dq + c * N * D;
        double* DK = dk + c * N * D;
        double* DV = dv + c * N * D;
        double* st = (double*)calloc((size_t)D * D, sizeof(double));
        double* nx = (double*)malloc(sizeof(double) * D * D);
        double* A = (double*)malloc(sizeof(double) * block * block);
        double* dA = (double*)malloc(sizeof(double) * block * block);
        /* forward-order sweep: dQ */
        for (i64 ib = 0; ib < T; ++ib) {
            const i64 b0 = ib * block;
            const i64 len = (N - b0 < block) ? (N - b0) : block;
            for (i64 r = 0; r < len; ++r)
                for (i64 cc = 0; cc < len; ++cc) {
                    double gv = 0.0;
                    for (int j = 0; j < D; ++j) gv += G[(b0 + r) * D + j] * V[(b0 + cc) * D + j];
                    dA[r * block + cc] = (r >= cc) ? gv * decay_pow(lam, r - cc) : 0.0;
                }
            for (i64 r = 0; r < len; ++r) {
                const double lq = decay_pow(lam, r + 1);
                for (int i = 0; i < D; ++i) {
                    double intra = 0.0;
                    for (i64 cc = 0; cc < len; ++cc) intra += dA[r * block + cc] * K[(b0 + cc) * D + i];
                    double inter = 0.0;
                    for (int j = 0; j < D; ++j) inter += G[(b0 + r) * D + j] * st[i * D + j];
                    DQ[(b0 + r) * D + i] = intra + lq * inter;
                }
            }
            const double lb = decay_pow(lam, len);
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j) {
                    double acc = 0.0;
                    for (i64 cc = 0; cc < len; ++cc)
                        acc += decay_pow(lam, len - 1 - cc) * K[(b0 + cc) * D + i] * V[(b0 + cc) * D + j];
                    nx[i * D + j] = lb * st[i * D + j] + acc;
                }
            memcpy(st, nx, sizeof(double) * D * D);
        }
        /* reverse-order sweep: dK, dV */
        memset(st, 0, sizeof(double) * D * D);
        for (i64 ib = T - 1; ib >= 0; --ib) {
            const i64 b0 = ib * block;
            const i64 len = (N - b0 < block) ? (N - b0) : block;
            for (i64 r = 0; r < len; ++r)
                for (i64 cc = 0; cc < len; ++cc) {
                    double qk = 0.0, gv = 0.0;
                    for (int i = 0; i < D; ++i) {
                        qk += Q[(b0 + r) * D + i] * K[(b0 + cc) * D + i];
                        gv += G[(b0 + r) * D + i] * V[(b0 + cc) * D + i];
                    }
                    const double m = (r >= cc) ? decay_pow(lam, r - cc) : 0.0;
                    A[r * block + cc] = qk * m;
                    dA[r * block + cc] = gv * m;
                }
            for (i64 cc = 0; cc < len; ++cc) {
                const double lk = decay_pow(lam, len - cc);
                for (int j = 0; j < D; ++j) {
                    double intra = 0.0;
                    for (i64 r = 0; r < len; ++r) intra += A[r * block + cc] * G[(b0 + r) * D + j];
                    double inter = 0.0;
                    for (int i = 0; i < D; ++i) inter += K[(b0 + cc) * D + i] * st[i * D + j];
                    DV[(b0 + cc) * D + j] = intra + lk * inter;
                }
                for (int i = 0; i < D; ++i) {
                    double intra = 0.0;
                    for (i64 r = 0; r < len; ++r) intra += dA[r * block + cc] * Q[(b0 + r) * D + i];
                    double inter = 0.0;
                    for (int j = 0; j < D; ++j) inter += V[(b0 + cc) * D + j] * st[i * D + j];
                    DK[(b0 + cc) * D + i] = intra + lk * inter;
                }
            }
            const double lb = decay_pow(lam, len);
            for (int i = 0; i < D; ++i)
                for (int j = 0; j < D; ++j) {
                    double acc = 0.0;
                    for (i64 r = 0; r < len; ++r)
                        acc += decay_pow(lam, r) * Q[(b0 + r) * D + i] * G[(b0 + r) * D + j];
                    nx[i * D + j] = lb * st[i * D + j] + acc;
                }
            memcpy(st, nx, sizeof(double) * D * D);
        }
        free(dA); free(A); free(nx); free(st);
    }
}

/* ------------------------------------------------------------------------ */
/* One decode step: a single iteration of Algorithm 2 on a caller-held state. */
/* q,k,v,o: [Bt,H,D]; kv: [Bt,H,D,D], updated in place, then read:            */
/*   kv = lambda kv + k^T v;  o = q kv                                         */
/* ------------------------------------------------------------------------ */
void ltn_oracle_decode_step(const double* q, const double* k, const double* v,
                            const double* decay, int Bt, int H, int D,
                            double* kv, double* o) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(static)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        double* S = kv + c * D * D;
        for (int i = 0; i < D; ++i)
            for (int j = 0; j < D; ++j)
                S[i * D + j] = lam * S[i * D + j] + k[c * D + i] * v[c * D + j];
        for (int j = 0; j < D; ++j) {
            double acc = 0.0;
            for (int i = 0; i < D; ++i) acc += q[c * D + i] * S[i * D + j];
            o[c * D + j] = acc;
        }
    }
}

/* ------------------------------------------------------------------------
 * Gated SimpleRMSNorm (Sec. 3.1.2 Eq. 3: O = Norm(.) (.) U; Sec. 3.1.3:
 * SRMSNorm(x) = x / (|x|_2 / sqrt(d))), row by row over `rows` vectors of d
 * features.  eps is added to the mean square under the root; eps = 0 is the
 * printed formula (a zero row then gives 0/0 = NaN, as the formula does).
 * ---------------------------------------------------------------------- */
void ltn_oracle_gate_fwd(const double* x, const double* u, double eps, i64 rows, int d, double* y) {
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < rows; ++r) {
        const double* xr = x + r * d;
        const double* ur = u + r * d;
        double ss = 0.0;
        for (int i = 0; i < d; ++i) ss += xr[i] * xr[i];
        const double rms = sqrt(ss / (double)d + eps);
        for (int i = 0; i < d; ++i) y[r * d + i] = xr[i] / rms * ur[i];
    }
}

/* Derivative of the map above.  With n = x / rms (the normalised row):
 *   du = dy (.) n
 *   dx = (g - n * mean(g (.) n)) / rms,   g = dy (.) u
 * (quotient rule on x_i / sqrt(mean(x^2) + eps)). */
void ltn_oracle_gate_bwd(const double* x, const double* u, const double* dy, double eps, i64 rows, int d,
                         double* dx, double* du) {
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < rows; ++r) {
        const double* xr = x + r * d;
        const double* ur = u + r * d;
        const double* gr = dy + r * d;
        double ss = 0.0;
        for (int i = 0; i < d; ++i) ss += xr[i] * xr[i];
        const double rms = sqrt(ss / (double)d + eps);
        double dot = 0.0;
        for (int i = 0; i < d; ++i) dot += gr[i] * ur[i] * (xr[i] / rms);
        const double mean = dot / (double)d;
        for (int i = 0; i < d; ++i) {
            const double n = xr[i] / rms;
            du[r * d + i] = gr[i] * n;
            dx[r * d + i] = (gr[i] * ur[i] - n * mean) / rms;
        }
    }
}

/* ========================================================================
 * Query/key feature width Dk different from the value width Dv.
 * The definition (Sec. 3.2.1) and Algorithm 2 (Sec. 3.3) never use that the two
 * widths agree: q_t, k_s in R^Dk meet only in their dot product, the state
 * kv is [Dk x Dv].  LRPE-d (below) needs Dk = 2 Dv.  Layouts: q,k [Bt,H,N,Dk];
 * v,o [Bt,H,N,Dv]; states [Bt,H,Dk,Dv].
 * ====================================================================== */

/* Algorithm 2 (Sec. 3.3), token by token. */
void ltn_oracle_fwd_recurrent_dkdv(const double* q, const double* k, const double* v,
                                   const double* decay, const double* kv_in,
                                   int Bt, int H, i64 N, int Dk, int Dv,
                                   double* o, double* kv_out) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * Dk;
        const double* K = k + c * N * Dk;
        const double* V = v + c * N * Dv;
        double* O = o + c * N * Dv;
        const size_t sz = sizeof(double) * (size_t)Dk * Dv;
        double* kv = (double*)malloc(sz);
        if (kv_in) memcpy(kv, kv_in + c * Dk * Dv, sz);
        else memset(kv, 0, sz);
        for (i64 t = 0; t < N; ++t) {
            for (int i = 0; i < Dk; ++i)
                for (int j = 0; j < Dv; ++j)
                    kv[i * Dv + j] = lam * kv[i * Dv + j] + K[t * Dk + i] * V[t * Dv + j];
            for (int j = 0; j < Dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < Dk; ++i) acc += Q[t * Dk + i] * kv[i * Dv + j];
                O[t * Dv + j] = acc;
            }
        }
        if (kv_out) memcpy(kv_out + c * Dk * Dv, kv, sz);
        free(kv);
    }
}

/* Gradients in recurrent form (derivative of the definition):
 *   forward sweep:  kv_t as above,            dq_t = kv_t dO_t^T        (Dk)
 *   reverse sweep:  dkv = lambda dkv + q_t^T dO_t  ([Dk x Dv]),
 *                   dk_t = dkv v_t^T (Dk),    dv_t = k_t dkv (Dv)             */
void ltn_oracle_bwd_recurrent_dkdv(const double* q, const double* k, const double* v,
                                   const double* d_o, const double* decay,
                                   int Bt, int H, i64 N, int Dk, int Dv,
                                   double* dq, double* dk, double* dv) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* Q = q + c * N * Dk;
        const double* K = k + c * N * Dk;
        const double* V = v + c * N * Dv;
        const double* G = d_o + c * N * Dv;
        double* DQ = dq + c * N * Dk;
        double* DK = dk + c * N * Dk;
        double* DV = dv + c * N * Dv;
        double* kv = (double*)calloc((size_t)Dk * Dv, sizeof(double));
        for (i64 t = 0; t < N; ++t) {
            for (int i = 0; i < Dk; ++i)
                for (int j = 0; j < Dv; ++j)
                    kv[i * Dv + j] = lam * kv[i * Dv + j] + K[t * Dk + i] * V[t * Dv + j];
            for (int i = 0; i < Dk; ++i) {
                double acc = 0.0;
                for (int j = 0; j < Dv; ++j) acc += G[t * Dv + j] * kv[i * Dv + j];
                DQ[t * Dk + i] = acc;
            }
        }
        memset(kv, 0, sizeof(double) * (size_t)Dk * Dv); /* now the suffix state dkv */
        for (i64 t = N - 1; t >= 0; --t) {
            for (int i = 0; i < Dk; ++i)
                for (int j = 0; j < Dv; ++j)
                    kv[i * Dv + j] = lam * kv[i * Dv + j] + Q[t * Dk + i] * G[t * Dv + j];
            for (int i = 0; i < Dk; ++i) {
                double acc = 0.0;
                for (int j = 0; j < Dv; ++j) acc += V[t * Dv + j] * kv[i * Dv + j];
                DK[t * Dk + i] = acc;
            }
            for (int j = 0; j < Dv; ++j) {
                double acc = 0.0;
                for (int i = 0; i < Dk; ++i) acc += K[t * Dk + i] * kv[i * Dv + j];
                DV[t * Dv + j] = acc;
            }
        }
        free(kv);
    }
}

/* One iteration of Algorithm 2 on a caller-held [Dk x Dv] state. */
void ltn_oracle_decode_step_dkdv(const double* q, const double* k, const double* v,
                                 const double* decay, int Bt, int H, int Dk, int Dv,
                                 double* kv, double* o) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(static)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        double* S = kv + c * Dk * Dv;
        for (int i = 0; i < Dk; ++i)
            for (int j = 0; j < Dv; ++j)
                S[i * Dv + j] = lam * S[i * Dv + j] + k[c * Dk + i] * v[c * Dv + j];
        for (int j = 0; j < Dv; ++j) {
            double acc = 0.0;
            for (int i = 0; i < Dk; ++i) acc += q[c * Dk + i] * S[i * Dv + j];
            o[c * Dv + j] = acc;
        }
    }
}

/* ========================================================================
 * Input side of the token mixer: the activation of Eq. 2 (Q = phi(X W_q),
 * K = phi(X W_k) with phi = swish, Sec. 3.1.2) and the position encoding of
 * Eq. 1, LRPE-d (Sec. 3.1.1):
 *     a[t,s] = q_t^T k_s lambda^(t-s) exp(i theta (t-s))
 * The paper prints the complex form only.  Reading taken here: theta is a real
 * learnable vector per head, one angle per feature ([H, D]); the phase acts
 * feature by feature and the score is the real part,
 *     a[t,s] = lambda^(t-s) sum_d q_t[d] k_s[d] cos(theta_d (t - s)).
 * ====================================================================== */

/* The definition with the real part of Eq. 1 as the score, quadratic in N. */
void ltn_oracle_lrpe_fwd_quadratic(const double* q, const double* k, const double* v,
                                   const double* decay, const double* theta,
                                   int Bt, int H, i64 N, int D, double* o) {
    const i64 chains = (i64)Bt * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 c = 0; c < chains; ++c) {
        const double lam = decay[c % H];
        const double* th = theta + (c % H) * D;
        const double* Q = q + c * N * D;
        const double* K = k + c * N * D;
        const double* V = v + c * N * D;
        double* O = o + c * N * D;
        for (i64 t = 0; t < N; ++t) {
            for (int j = 0; j < D; ++j) O[t * D + j] = 0.0;
            for (i64 s = 0; s <= t; ++s) {
                double dot = 0.0;
                for (int i = 0; i < D; ++i)
                    dot += Q[t * D + i] * K[s * D + i] * cos(th[i] * (double)(t - s));
                const double a = dot * decay_pow(lam, t - s);
                for (int j = 0; j < D; ++j) O[t * D + j] += a * V[s * D + j];
            }
        }
    }
}

static double swish(double x) { return x / (1.0 + exp(-x)); }
/* d/dx [x sigma(x)] = sigma(x) (1 + x (1 - sigma(x))) */
static double swish_grad(double x) {
    const double s = 1.0 / (1.0 + exp(-x));
    return s * (1.0 + x * (1.0 - s));
}

/* What the linear-cost evaluation feeds to the attention: Eq. 1 "can be decomposed
 * with respect to s and t separately" (Sec. 3.1.1) because
 * cos(theta (t-s)) = cos(theta t) cos(theta s) + sin(theta t) sin(theta s).  For a
 * token at absolute position p = pos0 + (row index) and z = phi(x) (act != 0) or x:
 *     y = [ z (.) cos(theta p) | z (.) sin(theta p) ]      (width 2D)
 * applied to queries and keys alike; their dot product is then the real-part
 * score above.  theta == NULL: no position encoding, y = z (width D). */
void ltn_oracle_prologue_fwd(const double* x, const double* theta, int act,
                             int Bt, int H, i64 N, int D, i64 pos0, double* y) {
    const i64 chains = (i64)Bt * H;
    const int W = theta ? 2 * D : D;
#pragma omp parallel for schedule(static)
    for (i64 c = 0; c < chains; ++c) {
        const double* th = theta ? theta + (c % H) * D : NULL;
        for (i64 t = 0; t < N; ++t) {
            const double* xr = x + (c * N + t) * D;
            double* yr = y + (c * N + t) * W;
            const double p = (double)(pos0 + t);
            for (int i = 0; i < D; ++i) {
                const double z = act ? swish(xr[i]) : xr[i];
                if (th) {
                    yr[i] = z * cos(th[i] * p);
                    yr[D + i] = z * sin(th[i] * p);
                } else {
                    yr[i] = z;
                }
            }
        }
    }
}

/* Derivative of the map above, given dy (width 2D, or D without theta):
 *     dz = dy_c cos(theta p) + dy_s sin(theta p),      dx = dz phi'(x)
 *     dtheta[h,d] = sum over batch and tokens of  p z (dy_s cos(theta p) - dy_c sin(theta p))
 * dtheta ([H, D]) may be NULL.  Parallel over heads so that the sum has a fixed order. */
void ltn_oracle_prologue_bwd(const double* x, const double* theta, const double* dy, int act,
                             int Bt, int H, i64 N, int D, i64 pos0,
                             double* dx, double* dtheta) {
    const int W = theta ? 2 * D : D;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h) {
        const double* th = theta ? theta + (i64)h * D : NULL;
        if (dtheta) for (int i = 0; i < D; ++i) dtheta[(i64)h * D + i] = 0.0;
        for (int b = 0; b < Bt; ++b) {
            const i64 c = (i64)b * H + h;
            for (i64 t = 0; t < N; ++t) {
                const double* xr = x + (c * N + t) * D;
                const double* gr = dy + (c * N + t) * W;
                double* dxr = dx + (c * N + t) * D;
                const double p = (double)(pos0 + t);
                for (int i = 0; i < D; ++i) {
                    const double z = act ? swish(xr[i]) : xr[i];
                    const double dphi = act ? swish_grad(xr[i]) : 1.0;
                    if (th) {
                        const double cs = cos(th[i] * p), sn = sin(th[i] * p);
                        dxr[i] = (gr[i] * cs + gr[D + i] * sn) * dphi;
                        if (dtheta) dtheta[(i64)h * D + i] += p * z * (gr[D + i] * cs - gr[i] * sn);
                    } else {
                        dxr[i] = gr[i] * dphi;
                    }
                }
            }
        }
    }
}
