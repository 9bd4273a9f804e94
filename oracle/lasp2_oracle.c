/*
 * CPU oracle for causal (unnormalised, identity-kernel) linear attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path, is
 * never called by it, and only tests, the smoke check and the bench's
 * cpu_baseline leg may load it.
 *
 * Everything is fp64.  Tensors are [G][N][d] row-major, where G = B*H
 * independent (batch, head) groups; d is the fastest axis.
 *
 * Packed variable-length input (LASP-2 paper, "Variable Length" paragraph of
 * the Compatibility appendix; block-diagonal reading: no state crosses a
 * document boundary): the N tokens of every group are cut into documents by
 * `cu` (n_docs+1 monotone offsets, cu[0]=0, cu[n_docs]=N).  n_docs==1 with
 * cu={0,N} is the ordinary single-sequence case.
 *
 * Three independent families are provided so they can be pinned against each
 * other and against closed forms by the CPU tests:
 *   *_def     : the token-level definition, LASP-2 paper Eq. (3)
 *               o_s = sum_{i<=s} (q_s . k_i) v_i     (diagonal inclusive)
 *               and its analytic gradient written as the same kind of
 *               double sum (Algorithm "LASP-2 w/ Masking (Backward Pass)"
 *               with a single chunk).
 *   *_rec     : the recurrent form, Eq. (4):  M_s = M_{s-1} + k_s^T v_s,
 *               o_s = q_s M_s, and the matching two-scan backward.
 *   chunk_states / state_prefix / attn_*_chunked :
 *               the steps of Algorithm "LASP-2 w/ Masking" and its backward,
 *               in the paper's order, over an arbitrary partition of the
 *               tokens into chunks.
 *   *_decay      : the same three families for scalar decay (one factor lam in (0,1] per
 *               group, mask entries lam^(i-j) instead of 1), the form the Retention and
 *               Lightning Attention layers of the paper's Table 2 use; the paper prints no
 *               formulas for them, so the definition below is the reference and the
 *               recurrence and chunked steps are derived from it.
 *   softmax_*    : standard softmax attention, O = Softmax(Q K^T / sqrt(d)) V, the local
 *               computation of Algorithm "AllGather-based Context Parallelism" (the
 *               standard-attention layers of the hybrid model), with its gradient.
 *   nomask_*_def / state_total / rows_times_state :
 *               linear attention without the mask (every token of a document
 *               attends to every token of it): the double-sum definition and
 *               the steps of Algorithm "LASP-2 w/o Masking" and its backward.
 *
 * Readings of the paper used here:
 *   - the mask Psi multiplies elementwise, so the entries the paper prints as
 *     "-infinity" act as 0 (Eq. (3) sums over i <= s only);
 *   - empty prefix M_{1:0} and empty suffix dM_{T+1:T} are zero matrices;
 *   - no 1/sqrt(d) factor, no normaliser, no feature map (basic linear
 *     attention).
 */
#include <stdlib.h>
#include <math.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int lasp2_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double dot(const double* a, const double* b, long d)
{
    double s = 0.0;
    for (long c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

/* document index of every token: doc[i] = k  <=>  cu[k] <= i < cu[k+1] */
static long* doc_ids(long N, const long* cu, long n_docs)
{
    long* doc = (long*)malloc(sizeof(long) * (size_t)(N > 0 ? N : 1));
    for (long k = 0; k < n_docs; ++k)
        for (long i = cu[k]; i < cu[k + 1]; ++i) doc[i] = k;
    return doc;
}

/* ------------------------------------------------------------------ */
/* Definition, Eq. (3): O[i,:] = sum_{j<=i, doc(j)=doc(i)} (q_i.k_j) v_j */
/* ------------------------------------------------------------------ */
void lasp2_oracle_fwd_def(const double* Q, const double* K, const double* V,
                          double* O, long G, long N, long d,
                          const long* cu, long n_docs)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long i = 0; i < N; ++i) {
            const double* q = Q + (g * N + i) * d;
            double* o = O + (g * N + i) * d;
            for (long c = 0; c < d; ++c) o[c] = 0.0;
            for (long j = cu[doc[i]]; j <= i; ++j) {
                double s = dot(q, K + (g * N + j) * d, d);
                const double* v = V + (g * N + j) * d;
                for (long c = 0; c < d; ++c) o[c] += s * v[c];
            }
        }
    }
    free(doc);
}

/*
 * Gradient of <dO, O> under the definition.  With S_ij = q_i.k_j and
 * G_ij = dO_i.v_j on the allowed pairs (j <= i, same document):
 *   dQ[i,:] = sum_{j<=i} G_ij k_j
 *   dK[j,:] = sum_{i>=j} G_ij q_i
 *   dV[j,:] = sum_{i>=j} S_ij dO_i
 * (backward algorithm with masking, taken with one chunk per document).
 */
void lasp2_oracle_bwd_def(const double* Q, const double* K, const double* V,
                          const double* dO, double* dQ, double* dK, double* dV,
                          long G, long N, long d, const long* cu, long n_docs)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long i = 0; i < N; ++i) {
            const double* go = dO + (g * N + i) * d;
            double* dq = dQ + (g * N + i) * d;
            for (long c = 0; c < d; ++c) dq[c] = 0.0;
            for (long j = cu[doc[i]]; j <= i; ++j) {
                double gij = dot(go, V + (g * N + j) * d, d);
                const double* k = K + (g * N + j) * d;
                for (long c = 0; c < d; ++c) dq[c] += gij * k[c];
            }
        }
    }
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long j = 0; j < N; ++j) {
            const double* k = K + (g * N + j) * d;
            const double* v = V + (g * N + j) * d;
            double* dk = dK + (g * N + j) * d;
            double* dv = dV + (g * N + j) * d;
            for (long c = 0; c < d; ++c) { dk[c] = 0.0; dv[c] = 0.0; }
            for (long i = j; i < cu[doc[j] + 1]; ++i) {
                const double* q = Q + (g * N + i) * d;
                const double* go = dO + (g * N + i) * d;
                double gij = dot(go, v, d);
                double sij = dot(q, k, d);
                for (long c = 0; c < d; ++c) {
                    dk[c] += gij * q[c];
                    dv[c] += sij * go[c];
                }
            }
        }
    }
    free(doc);
}

/*
 * Selected rows of the definition, for sizes where the full double sum is
 * out of reach.  One group (Q,K,V,dO are [N][d]); rows[r] is a token index.
 * which: 0 -> O rows, 1 -> dQ rows, 2 -> dK rows, 3 -> dV rows.
 * For which==0 the dO argument is unused and may be NULL.
 */
void lasp2_oracle_def_rows(const double* Q, const double* K, const double* V,
                           const double* dO, long N, long d,
                           const long* cu, long n_docs,
                           const long* rows, long n_rows, int which,
                           double* out /* [n_rows][d] */)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < n_rows; ++r) {
        long t = rows[r];
        double* o = out + r * d;
        for (long c = 0; c < d; ++c) o[c] = 0.0;
        if (which == 0) {
            for (long j = cu[doc[t]]; j <= t; ++j) {
                double s = dot(Q + t * d, K + j * d, d);
                for (long c = 0; c < d; ++c) o[c] += s * V[j * d + c];
            }
        } else if (which == 1) {
            for (long j = cu[doc[t]]; j <= t; ++j) {
                double gij = dot(dO + t * d, V + j * d, d);
                for (long c = 0; c < d; ++c) o[c] += gij * K[j * d + c];
            }
        } else if (which == 2) {
            for (long i = t; i < cu[doc[t] + 1]; ++i) {
                double gij = dot(dO + i * d, V + t * d, d);
                for (long c = 0; c < d; ++c) o[c] += gij * Q[i * d + c];
            }
        } else {
            for (long i = t; i < cu[doc[t] + 1]; ++i) {
                double sij = dot(Q + i * d, K + t * d, d);
                for (long c = 0; c < d; ++c) o[c] += sij * dO[i * d + c];
            }
        }
    }
    free(doc);
}

/* ------------------------------------------------------------------ */
/* Recurrent form, Eq. (4).  State update first, then read-out, so the */
/* diagonal is included; the state is cleared at each document start.  */
/* ------------------------------------------------------------------ */
void lasp2_oracle_fwd_rec(const double* Q, const double* K, const double* V,
                          double* O, long G, long N, long d,
                          const long* cu, long n_docs)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        double* M = (double*)malloc(sizeof(double) * (size_t)(d * d));
        for (long k = 0; k < n_docs; ++k) {
            memset(M, 0, sizeof(double) * (size_t)(d * d));
            for (long s = cu[k]; s < cu[k + 1]; ++s) {
                const double* q = Q + (g * N + s) * d;
                const double* kk = K + (g * N + s) * d;
                const double* v = V + (g * N + s) * d;
                double* o = O + (g * N + s) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) M[a * d + b] += kk[a] * v[b];
                for (long b = 0; b < d; ++b) o[b] = 0.0;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) o[b] += q[a] * M[a * d + b];
            }
        }
        free(M);
    }
}

/*
 * Backward of the recurrence.  dq_s = dO_s M_s^T uses the same forward scan;
 * the adjoint state D_s = sum_{i>=s} q_i^T dO_i runs backwards (update before
 * use, cleared at each document end):  dk_s = v_s D_s^T,  dv_s = k_s D_s.
 */
void lasp2_oracle_bwd_rec(const double* Q, const double* K, const double* V,
                          const double* dO, double* dQ, double* dK, double* dV,
                          long G, long N, long d, const long* cu, long n_docs)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        double* M = (double*)malloc(sizeof(double) * (size_t)(d * d));
        for (long k = 0; k < n_docs; ++k) {
            memset(M, 0, sizeof(double) * (size_t)(d * d));
            for (long s = cu[k]; s < cu[k + 1]; ++s) {
                const double* kk = K + (g * N + s) * d;
                const double* v = V + (g * N + s) * d;
                const double* go = dO + (g * N + s) * d;
                double* dq = dQ + (g * N + s) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) M[a * d + b] += kk[a] * v[b];
                for (long a = 0; a < d; ++a) {
                    double acc = 0.0;
                    for (long b = 0; b < d; ++b) acc += go[b] * M[a * d + b];
                    dq[a] = acc;
                }
            }
            memset(M, 0, sizeof(double) * (size_t)(d * d));
            for (long s = cu[k + 1] - 1; s >= cu[k]; --s) {
                const double* q = Q + (g * N + s) * d;
                const double* kk = K + (g * N + s) * d;
                const double* v = V + (g * N + s) * d;
                const double* go = dO + (g * N + s) * d;
                double* dk = dK + (g * N + s) * d;
                double* dv = dV + (g * N + s) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) M[a * d + b] += q[a] * go[b];
                for (long a = 0; a < d; ++a) {
                    double acc = 0.0;
                    for (long b = 0; b < d; ++b) acc += v[b] * M[a * d + b];
                    dk[a] = acc;
                }
                for (long b = 0; b < d; ++b) dv[b] = 0.0;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) dv[b] += kk[a] * M[a * d + b];
            }
        }
        free(M);
    }
}

/* ------------------------------------------------------------------ */
/* The steps of Algorithm "LASP-2 w/ Masking" over a chunk partition.   */
/* bounds: n_chunks+1 monotone token offsets (bounds[0]=0, last = N);   */
/* chunk t holds tokens bounds[t] .. bounds[t+1]-1.                     */
/* ------------------------------------------------------------------ */

/* line "Compute M_t = K_t^T V_t":  M is [G][n_chunks][d][d] */
void lasp2_oracle_chunk_states(const double* K, const double* V, double* M,
                               long G, long N, long d,
                               const long* bounds, long n_chunks)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        for (long t = 0; t < n_chunks; ++t) {
            double* m = M + (g * n_chunks + t) * d * d;
            for (long e = 0; e < d * d; ++e) m[e] = 0.0;
            for (long s = bounds[t]; s < bounds[t + 1]; ++s) {
                const double* kk = K + (g * N + s) * d;
                const double* v = V + (g * N + s) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) m[a * d + b] += kk[a] * v[b];
            }
        }
    }
}

/*
 * PrefixSum / SuffixSum over the gathered states, exclusive, by the
 * recursion M_{1:t-1} = M_{1:t-2} + M_{t-1}.
 *   reverse == 0:  P_t = sum_{s<t} M_s, restarted from zero at every chunk t
 *                  with first[t] != 0 (chunk t opens a document);
 *   reverse != 0:  P_t = sum_{s>t} M_s, restarted from zero at every chunk t
 *                  that closes a document (t == n_chunks-1 or first[t+1]).
 * first may be NULL (only chunk 0 opens a document).
 */
void lasp2_oracle_state_prefix(const double* M, double* P, long G,
                               long n_chunks, long d, const int* first,
                               int reverse)
{
    long dd = d * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        double* run = (double*)malloc(sizeof(double) * (size_t)dd);
        memset(run, 0, sizeof(double) * (size_t)dd);
        if (!reverse) {
            for (long t = 0; t < n_chunks; ++t) {
                if (t == 0 || (first && first[t])) memset(run, 0, sizeof(double) * (size_t)dd);
                const double* m = M + (g * n_chunks + t) * dd;
                double* p = P + (g * n_chunks + t) * dd;
                for (long e = 0; e < dd; ++e) { double add = m[e]; p[e] = run[e]; run[e] += add; }
            }
        } else {
            for (long t = n_chunks - 1; t >= 0; --t) {
                if (t == n_chunks - 1 || (first && first[t + 1])) memset(run, 0, sizeof(double) * (size_t)dd);
                const double* m = M + (g * n_chunks + t) * dd;
                double* p = P + (g * n_chunks + t) * dd;
                for (long e = 0; e < dd; ++e) { double add = m[e]; p[e] = run[e]; run[e] += add; }
            }
        }
        free(run);
    }
}

/*
 * O_t = [(Q_t K_t^T) (.) Psi] V_t + Q_t M_{1:t-1}: the intra-chunk masked left
 * product plus the inter-chunk product with the exclusive prefix state P_t.
 */
void lasp2_oracle_attn_fwd_chunked(const double* Q, const double* K, const double* V,
                                   const double* P, double* O,
                                   long G, long N, long d,
                                   const long* bounds, long n_chunks)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        for (long t = 0; t < n_chunks; ++t) {
            long lo = bounds[t], hi = bounds[t + 1], C = hi - lo;
            if (C <= 0) continue;
            const double* p = P + (g * n_chunks + t) * d * d;
            double* S = (double*)malloc(sizeof(double) * (size_t)(C * C));
            /* S = (Q_t K_t^T) (.) Psi, Psi_ij = 1 if i >= j else 0 */
            for (long i = 0; i < C; ++i)
                for (long j = 0; j < C; ++j)
                    S[i * C + j] = (i >= j)
                        ? dot(Q + (g * N + lo + i) * d, K + (g * N + lo + j) * d, d) : 0.0;
            for (long i = 0; i < C; ++i) {
                double* o = O + (g * N + lo + i) * d;
                const double* q = Q + (g * N + lo + i) * d;
                for (long b = 0; b < d; ++b) {
                    double intra = 0.0, inter = 0.0;
                    for (long j = 0; j < C; ++j) intra += S[i * C + j] * V[(g * N + lo + j) * d + b];
                    for (long a = 0; a < d; ++a) inter += q[a] * p[a * d + b];
                    o[b] = intra + inter;
                }
            }
            free(S);
        }
    }
}

/*
 * Backward with masking, per chunk t, given the cached prefix P_t = M_{1:t-1}
 * and the suffix dP_t = dM_{t+1:T}:
 *   dQ_t = [(dO_t V_t^T)(.)Psi] K_t   + dO_t P_t^T
 *   dK_t = [(dO_t V_t^T)(.)Psi]^T Q_t + V_t dP_t^T
 *   dV_t = [(Q_t K_t^T)(.)Psi]^T dO_t + K_t dP_t
 */
void lasp2_oracle_attn_bwd_chunked(const double* Q, const double* K, const double* V,
                                   const double* dO, const double* P, const double* dP,
                                   double* dQ, double* dK, double* dV,
                                   long G, long N, long d,
                                   const long* bounds, long n_chunks)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        for (long t = 0; t < n_chunks; ++t) {
            long lo = bounds[t], hi = bounds[t + 1], C = hi - lo;
            if (C <= 0) continue;
            const double* p = P + (g * n_chunks + t) * d * d;
            const double* dp = dP + (g * n_chunks + t) * d * d;
            double* S = (double*)malloc(sizeof(double) * (size_t)(C * C));
            double* Gm = (double*)malloc(sizeof(double) * (size_t)(C * C));
            for (long i = 0; i < C; ++i)
                for (long j = 0; j < C; ++j) {
                    int keep = (i >= j);
                    S[i * C + j] = keep ? dot(Q + (g * N + lo + i) * d, K + (g * N + lo + j) * d, d) : 0.0;
                    Gm[i * C + j] = keep ? dot(dO + (g * N + lo + i) * d, V + (g * N + lo + j) * d, d) : 0.0;
                }
            for (long i = 0; i < C; ++i) {
                const double* go = dO + (g * N + lo + i) * d;
                double* dq = dQ + (g * N + lo + i) * d;
                for (long a = 0; a < d; ++a) {
                    double intra = 0.0, inter = 0.0;
                    for (long j = 0; j < C; ++j) intra += Gm[i * C + j] * K[(g * N + lo + j) * d + a];
                    for (long b = 0; b < d; ++b) inter += go[b] * p[a * d + b];
                    dq[a] = intra + inter;
                }
            }
            for (long j = 0; j < C; ++j) {
                const double* kk = K + (g * N + lo + j) * d;
                const double* v = V + (g * N + lo + j) * d;
                double* dk = dK + (g * N + lo + j) * d;
                double* dv = dV + (g * N + lo + j) * d;
                for (long a = 0; a < d; ++a) {
                    double intra = 0.0, inter = 0.0;
                    for (long i = 0; i < C; ++i) intra += Gm[i * C + j] * Q[(g * N + lo + i) * d + a];
                    for (long b = 0; b < d; ++b) inter += v[b] * dp[a * d + b];
                    dk[a] = intra + inter;
                }
                for (long b = 0; b < d; ++b) {
                    double intra = 0.0, inter = 0.0;
                    for (long i = 0; i < C; ++i) intra += S[i * C + j] * dO[(g * N + lo + i) * d + b];
                    for (long a = 0; a < d; ++a) inter += kk[a] * dp[a * d + b];
                    dv[b] = intra + inter;
                }
            }
            free(S);
            free(Gm);
        }
    }
}

/* ------------------------------------------------------------------ */
/* Without masking.  Definition: O[i,:] = sum_{j: doc(j)=doc(i)} (q_i.k_j) v_j */
/* (Section "LASP-2 without Masking": O = (Q K^T) V with no mask).      */
/* ------------------------------------------------------------------ */
void lasp2_oracle_nomask_fwd_def(const double* Q, const double* K, const double* V,
                                 double* O, long G, long N, long d,
                                 const long* cu, long n_docs)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long i = 0; i < N; ++i) {
            double* o = O + (g * N + i) * d;
            for (long b = 0; b < d; ++b) o[b] = 0.0;
            for (long j = cu[doc[i]]; j < cu[doc[i] + 1]; ++j) {
                double s = dot(Q + (g * N + i) * d, K + (g * N + j) * d, d);
                const double* v = V + (g * N + j) * d;
                for (long b = 0; b < d; ++b) o[b] += s * v[b];
            }
        }
    }
    free(doc);
}

/*
 * Gradient of <dO, O> for the unmasked definition.  With S_ij = q_i.k_j and
 * G_ij = dO_i.v_j over all pairs of one document:
 *   dQ[i,:] = sum_j G_ij k_j,   dK[j,:] = sum_i G_ij q_i,   dV[j,:] = sum_i S_ij dO_i.
 */
void lasp2_oracle_nomask_bwd_def(const double* Q, const double* K, const double* V,
                                 const double* dO, double* dQ, double* dK, double* dV,
                                 long G, long N, long d, const long* cu, long n_docs)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long i = 0; i < N; ++i) {
            long lo = cu[doc[i]], hi = cu[doc[i] + 1];
            double* dq = dQ + (g * N + i) * d;
            double* dk = dK + (g * N + i) * d;
            double* dv = dV + (g * N + i) * d;
            for (long a = 0; a < d; ++a) { dq[a] = 0.0; dk[a] = 0.0; dv[a] = 0.0; }
            for (long j = lo; j < hi; ++j) {
                /* row i as a query against key/value j */
                double gij = dot(dO + (g * N + i) * d, V + (g * N + j) * d, d);
                const double* kj = K + (g * N + j) * d;
                for (long a = 0; a < d; ++a) dq[a] += gij * kj[a];
                /* row i as a key/value against query j */
                double gji = dot(dO + (g * N + j) * d, V + (g * N + i) * d, d);
                double sji = dot(Q + (g * N + j) * d, K + (g * N + i) * d, d);
                const double* qj = Q + (g * N + j) * d;
                const double* doj = dO + (g * N + j) * d;
                for (long a = 0; a < d; ++a) { dk[a] += gji * qj[a]; dv[a] += sji * doj[a]; }
            }
        }
    }
    free(doc);
}

/*
 * Line "Compute M_{1:T} = Sum([M_t]_1^T)" of Algorithm "LASP-2 w/o Masking",
 * by the recursive accumulation the text describes (M_{1:t-1} + M_t), once per
 * document; every chunk t receives the total of its own document, as every
 * rank holds M_{1:T} after the gather.  first as in state_prefix.
 */
void lasp2_oracle_state_total(const double* M, double* S, long G, long n_chunks,
                              long d, const int* first)
{
    long dd = d * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        double* run = (double*)malloc(sizeof(double) * (size_t)dd);
        long t0 = 0;
        while (t0 < n_chunks) {
            long t1 = t0 + 1;
            while (t1 < n_chunks && !(first && first[t1])) ++t1;
            memset(run, 0, sizeof(double) * (size_t)dd);
            for (long t = t0; t < t1; ++t) {
                const double* m = M + (g * n_chunks + t) * dd;
                for (long e = 0; e < dd; ++e) run[e] += m[e];
            }
            for (long t = t0; t < t1; ++t) memcpy(S + (g * n_chunks + t) * dd, run, sizeof(double) * (size_t)dd);
            t0 = t1;
        }
        free(run);
    }
}

/*
 * out_t = A_t S_t (transpose == 0) or A_t S_t^T (transpose != 0) for every
 * chunk t: the lines O_t = Q_t M_{1:T}, dQ_t = dO_t M_{1:T}^T,
 * dK_t = V_t dM_{1:T}^T and dV_t = K_t dM_{1:T} of the two algorithms
 * without masking.  S is [G][n_chunks][d][d].
 */
void lasp2_oracle_rows_times_state(const double* A, const double* S, double* out,
                                   long G, long N, long d, const long* bounds,
                                   long n_chunks, int transpose)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        for (long t = 0; t < n_chunks; ++t) {
            const double* s = S + (g * n_chunks + t) * d * d;
            for (long i = bounds[t]; i < bounds[t + 1]; ++i) {
                const double* a = A + (g * N + i) * d;
                double* o = out + (g * N + i) * d;
                for (long c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (long r = 0; r < d; ++r) acc += a[r] * (transpose ? s[c * d + r] : s[r * d + c]);
                    o[c] = acc;
                }
            }
        }
    }
}

/*
 * Selected rows of the unmasked definition (one group; Q,K,V,dO are [N][d]).
 * which: 0 -> O rows, 1 -> dQ rows, 2 -> dK rows, 3 -> dV rows; dO may be NULL
 * for which == 0.
 */
void lasp2_oracle_nomask_def_rows(const double* Q, const double* K, const double* V,
                                  const double* dO, long N, long d, const long* cu,
                                  long n_docs, const long* rows, long n_rows, int which,
                                  double* out)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < n_rows; ++r) {
        long i = rows[r];
        long lo = cu[doc[i]], hi = cu[doc[i] + 1];
        double* o = out + r * d;
        for (long a = 0; a < d; ++a) o[a] = 0.0;
        for (long j = lo; j < hi; ++j) {
            if (which == 0) {            /* O_i   = sum_j (q_i.k_j) v_j   */
                double s = dot(Q + i * d, K + j * d, d);
                for (long a = 0; a < d; ++a) o[a] += s * V[j * d + a];
            } else if (which == 1) {     /* dQ_i  = sum_j (dO_i.v_j) k_j  */
                double gij = dot(dO + i * d, V + j * d, d);
                for (long a = 0; a < d; ++a) o[a] += gij * K[j * d + a];
            } else if (which == 2) {     /* dK_i  = sum_j (dO_j.v_i) q_j  */
                double gji = dot(dO + j * d, V + i * d, d);
                for (long a = 0; a < d; ++a) o[a] += gji * Q[j * d + a];
            } else {                     /* dV_i  = sum_j (q_j.k_i) dO_j  */
                double sji = dot(Q + j * d, K + i * d, d);
                for (long a = 0; a < d; ++a) o[a] += sji * dO[j * d + a];
            }
        }
    }
    free(doc);
}

/* ================================================================== */
/* Scalar decay.  lam[g] in (0,1] per group; lam == 1 is the plain case. */
/* Definition: O[i,:] = sum_{j<=i, same doc} lam^(i-j) (q_i.k_j) v_j     */
/* ================================================================== */
void lasp2_oracle_fwd_def_decay(const double* Q, const double* K, const double* V,
                                double* O, long G, long N, long d,
                                const long* cu, long n_docs, const double* lam)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long i = 0; i < N; ++i) {
            double* o = O + (g * N + i) * d;
            for (long b = 0; b < d; ++b) o[b] = 0.0;
            for (long j = cu[doc[i]]; j <= i; ++j) {
                double s = pow(lam[g], (double)(i - j)) * dot(Q + (g * N + i) * d, K + (g * N + j) * d, d);
                const double* v = V + (g * N + j) * d;
                for (long b = 0; b < d; ++b) o[b] += s * v[b];
            }
        }
    }
    free(doc);
}

/*
 * Gradient of <dO, O> under the decayed definition, as double sums:
 *   dQ[i,:] = sum_{j<=i} lam^(i-j) (dO_i.v_j) k_j
 *   dK[j,:] = sum_{i>=j} lam^(i-j) (dO_i.v_j) q_i
 *   dV[j,:] = sum_{i>=j} lam^(i-j) (q_i.k_j) dO_i
 */
void lasp2_oracle_bwd_def_decay(const double* Q, const double* K, const double* V,
                                const double* dO, double* dQ, double* dK, double* dV,
                                long G, long N, long d, const long* cu, long n_docs,
                                const double* lam)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long i = 0; i < N; ++i) {
            long lo = cu[doc[i]], hi = cu[doc[i] + 1];
            double* dq = dQ + (g * N + i) * d;
            double* dk = dK + (g * N + i) * d;
            double* dv = dV + (g * N + i) * d;
            for (long a = 0; a < d; ++a) { dq[a] = 0.0; dk[a] = 0.0; dv[a] = 0.0; }
            for (long j = lo; j <= i; ++j) {         /* i as a query */
                double w = pow(lam[g], (double)(i - j));
                double gij = w * dot(dO + (g * N + i) * d, V + (g * N + j) * d, d);
                const double* kj = K + (g * N + j) * d;
                for (long a = 0; a < d; ++a) dq[a] += gij * kj[a];
            }
            for (long r = i; r < hi; ++r) {          /* i as a key/value of the later query r */
                double w = pow(lam[g], (double)(r - i));
                double gri = w * dot(dO + (g * N + r) * d, V + (g * N + i) * d, d);
                double sri = w * dot(Q + (g * N + r) * d, K + (g * N + i) * d, d);
                const double* qr = Q + (g * N + r) * d;
                const double* dor = dO + (g * N + r) * d;
                for (long a = 0; a < d; ++a) { dk[a] += gri * qr[a]; dv[a] += sri * dor[a]; }
            }
        }
    }
    free(doc);
}

/*
 * Recurrent form with decay: M_s = lam M_{s-1} + k_s^T v_s, o_s = q_s M_s (state cleared at
 * each document start); backward: dq_s = dO_s M_s^T, adjoint D_s = lam D_{s+1} + q_s^T dO_s
 * (cleared at each document end), dk_s = v_s D_s^T, dv_s = k_s D_s.
 */
void lasp2_oracle_fwd_rec_decay(const double* Q, const double* K, const double* V, double* O,
                                long G, long N, long d, const long* cu, long n_docs,
                                const double* lam)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        double* M = (double*)malloc(sizeof(double) * (size_t)(d * d));
        for (long k = 0; k < n_docs; ++k) {
            memset(M, 0, sizeof(double) * (size_t)(d * d));
            for (long s = cu[k]; s < cu[k + 1]; ++s) {
                const double* q = Q + (g * N + s) * d;
                const double* kk = K + (g * N + s) * d;
                const double* v = V + (g * N + s) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) M[a * d + b] = lam[g] * M[a * d + b] + kk[a] * v[b];
                double* o = O + (g * N + s) * d;
                for (long b = 0; b < d; ++b) {
                    double acc = 0.0;
                    for (long a = 0; a < d; ++a) acc += q[a] * M[a * d + b];
                    o[b] = acc;
                }
            }
        }
        free(M);
    }
}

void lasp2_oracle_bwd_rec_decay(const double* Q, const double* K, const double* V,
                                const double* dO, double* dQ, double* dK, double* dV,
                                long G, long N, long d, const long* cu, long n_docs,
                                const double* lam)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        double* M = (double*)malloc(sizeof(double) * (size_t)(d * d));
        for (long k = 0; k < n_docs; ++k) {
            memset(M, 0, sizeof(double) * (size_t)(d * d));
            for (long s = cu[k]; s < cu[k + 1]; ++s) {
                const double* kk = K + (g * N + s) * d;
                const double* v = V + (g * N + s) * d;
                const double* go = dO + (g * N + s) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) M[a * d + b] = lam[g] * M[a * d + b] + kk[a] * v[b];
                double* dq = dQ + (g * N + s) * d;
                for (long a = 0; a < d; ++a) {
                    double acc = 0.0;
                    for (long b = 0; b < d; ++b) acc += go[b] * M[a * d + b];
                    dq[a] = acc;
                }
            }
            memset(M, 0, sizeof(double) * (size_t)(d * d));   /* now the adjoint state D */
            for (long s = cu[k + 1] - 1; s >= cu[k]; --s) {
                const double* q = Q + (g * N + s) * d;
                const double* kk = K + (g * N + s) * d;
                const double* v = V + (g * N + s) * d;
                const double* go = dO + (g * N + s) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) M[a * d + b] = lam[g] * M[a * d + b] + q[a] * go[b];
                double* dk = dK + (g * N + s) * d;
                double* dv = dV + (g * N + s) * d;
                for (long a = 0; a < d; ++a) {
                    double acc = 0.0;
                    for (long b = 0; b < d; ++b) acc += v[b] * M[a * d + b];
                    dk[a] = acc;
                }
                for (long b = 0; b < d; ++b) {
                    double acc = 0.0;
                    for (long a = 0; a < d; ++a) acc += kk[a] * M[a * d + b];
                    dv[b] = acc;
                }
            }
        }
        free(M);
    }
}

/*
 * Chunked steps with decay, derived from the recurrence over a chunk partition `bounds`
 * (chunk t = tokens lo_t .. hi_t - 1, n_t = hi_t - lo_t):
 *   states, anchor_start == 0:  M_t = sum_j lam^(hi_t - 1 - j) k_j^T v_j   (the state as the chunk's
 *                               last token sees it; the forward's K^T V states)
 *           anchor_start != 0:  M_t = sum_j lam^(j - lo_t) x_j^T y_j       (the adjoint as the chunk's
 *                               first token sees it; the backward's Q^T dO states)
 */
void lasp2_oracle_chunk_states_decay(const double* X, const double* Y, double* M,
                                     long G, long N, long d, const long* bounds, long n_chunks,
                                     const double* lam, int anchor_start)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        for (long t = 0; t < n_chunks; ++t) {
            double* m = M + (g * n_chunks + t) * d * d;
            memset(m, 0, sizeof(double) * (size_t)(d * d));
            for (long j = bounds[t]; j < bounds[t + 1]; ++j) {
                double w = pow(lam[g], (double)(anchor_start ? j - bounds[t] : bounds[t + 1] - 1 - j));
                const double* x = X + (g * N + j) * d;
                const double* y = Y + (g * N + j) * d;
                for (long a = 0; a < d; ++a)
                    for (long b = 0; b < d; ++b) m[a * d + b] += w * x[a] * y[b];
            }
        }
    }
}

/*
 * Decayed combine of the gathered states (exclusive, restarted at document edges):
 *   reverse == 0:  P_t = lam^(n_{t-1}) P_{t-1} + M_{t-1}   (M anchored at chunk ends)
 *   reverse != 0:  P_t = lam^(n_{t+1}) P_{t+1} + M_{t+1}   (M anchored at chunk starts)
 * so that P_t is the state the last token before chunk t holds (resp. the adjoint the first
 * token after it holds).
 */
void lasp2_oracle_state_prefix_decay(const double* M, double* P, long G, long n_chunks, long d,
                                     const int* first, int reverse, const long* bounds,
                                     const double* lam)
{
    long dd = d * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        double* run = (double*)malloc(sizeof(double) * (size_t)dd);
        memset(run, 0, sizeof(double) * (size_t)dd);
        for (long u = 0; u < n_chunks; ++u) {
            long t = reverse ? n_chunks - 1 - u : u;
            int edge = reverse ? (t == n_chunks - 1 || (first && first[t + 1]))
                               : (t == 0 || (first && first[t]));
            if (edge) memset(run, 0, sizeof(double) * (size_t)dd);
            const double* m = M + (g * n_chunks + t) * dd;
            double* p = P + (g * n_chunks + t) * dd;
            double w = pow(lam[g], (double)(bounds[t + 1] - bounds[t]));
            for (long e = 0; e < dd; ++e) { double add = m[e]; p[e] = run[e]; run[e] = w * run[e] + add; }
        }
        free(run);
    }
}

/*
 * Forward per chunk with decay: for the token at local index a of chunk t,
 *   o = sum_{b<=a} lam^(a-b) (q_a.k_b) v_b  +  lam^(a+1) q_a P_t .
 */
void lasp2_oracle_attn_fwd_chunked_decay(const double* Q, const double* K, const double* V,
                                         const double* P, double* O, long G, long N, long d,
                                         const long* bounds, long n_chunks, const double* lam)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        for (long t = 0; t < n_chunks; ++t) {
            long lo = bounds[t], hi = bounds[t + 1];
            const double* p = P + (g * n_chunks + t) * d * d;
            for (long i = lo; i < hi; ++i) {
                const double* q = Q + (g * N + i) * d;
                double* o = O + (g * N + i) * d;
                double wi = pow(lam[g], (double)(i - lo + 1));
                for (long b = 0; b < d; ++b) {
                    double inter = 0.0;
                    for (long a = 0; a < d; ++a) inter += q[a] * p[a * d + b];
                    o[b] = wi * inter;
                }
                for (long j = lo; j <= i; ++j) {
                    double s = pow(lam[g], (double)(i - j)) * dot(q, K + (g * N + j) * d, d);
                    for (long b = 0; b < d; ++b) o[b] += s * V[(g * N + j) * d + b];
                }
            }
        }
    }
}

/*
 * Backward per chunk with decay, from the cached prefix P_t and the decayed suffix dP_t:
 *   dq_a = sum_{b<=a} lam^(a-b) (dO_a.v_b) k_b + lam^(a+1) dO_a P_t^T
 *   dk_b = sum_{a>=b} lam^(a-b) (dO_a.v_b) q_a + lam^(n-b) v_b dP_t^T
 *   dv_b = sum_{a>=b} lam^(a-b) (q_a.k_b) dO_a + lam^(n-b) k_b dP_t
 * (n = chunk length; lam^(n-b) carries the adjoint from the first token after the chunk).
 */
void lasp2_oracle_attn_bwd_chunked_decay(const double* Q, const double* K, const double* V,
                                         const double* dO, const double* P, const double* dP,
                                         double* dQ, double* dK, double* dV, long G, long N, long d,
                                         const long* bounds, long n_chunks, const double* lam)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        for (long t = 0; t < n_chunks; ++t) {
            long lo = bounds[t], hi = bounds[t + 1];
            const double* p = P + (g * n_chunks + t) * d * d;
            const double* dp = dP + (g * n_chunks + t) * d * d;
            for (long i = lo; i < hi; ++i) {
                const double* go = dO + (g * N + i) * d;
                double* dq = dQ + (g * N + i) * d;
                double wi = pow(lam[g], (double)(i - lo + 1));
                for (long a = 0; a < d; ++a) {
                    double inter = 0.0;
                    for (long b = 0; b < d; ++b) inter += go[b] * p[a * d + b];
                    dq[a] = wi * inter;
                }
                for (long j = lo; j <= i; ++j) {
                    double gij = pow(lam[g], (double)(i - j)) * dot(go, V + (g * N + j) * d, d);
                    for (long a = 0; a < d; ++a) dq[a] += gij * K[(g * N + j) * d + a];
                }
            }
            for (long j = lo; j < hi; ++j) {
                const double* kk = K + (g * N + j) * d;
                const double* v = V + (g * N + j) * d;
                double* dk = dK + (g * N + j) * d;
                double* dv = dV + (g * N + j) * d;
                double wj = pow(lam[g], (double)(hi - j));
                for (long a = 0; a < d; ++a) {
                    double inter = 0.0;
                    for (long b = 0; b < d; ++b) inter += v[b] * dp[a * d + b];
                    dk[a] = wj * inter;
                }
                for (long b = 0; b < d; ++b) {
                    double inter = 0.0;
                    for (long a = 0; a < d; ++a) inter += kk[a] * dp[a * d + b];
                    dv[b] = wj * inter;
                }
                for (long i = j; i < hi; ++i) {
                    double w = pow(lam[g], (double)(i - j));
                    double gij = w * dot(dO + (g * N + i) * d, v, d);
                    double sij = w * dot(Q + (g * N + i) * d, kk, d);
                    for (long a = 0; a < d; ++a) {
                        dk[a] += gij * Q[(g * N + i) * d + a];
                        dv[a] += sij * dO[(g * N + i) * d + a];
                    }
                }
            }
        }
    }
}

/*
 * Selected rows of the decayed definition (one group; Q,K,V,dO are [N][d]; lam is that group's
 * factor).  which: 0 -> O rows, 1 -> dQ rows, 2 -> dK rows, 3 -> dV rows.
 */
void lasp2_oracle_def_rows_decay(const double* Q, const double* K, const double* V,
                                 const double* dO, long N, long d, const long* cu, long n_docs,
                                 const long* rows, long n_rows, int which, double lam, double* out)
{
    long* doc = doc_ids(N, cu, n_docs);
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < n_rows; ++r) {
        long i = rows[r];
        long lo = cu[doc[i]], hi = cu[doc[i] + 1];
        double* o = out + r * d;
        for (long a = 0; a < d; ++a) o[a] = 0.0;
        if (which <= 1) {
            for (long j = lo; j <= i; ++j) {
                double w = pow(lam, (double)(i - j));
                double s = w * (which == 0 ? dot(Q + i * d, K + j * d, d) : dot(dO + i * d, V + j * d, d));
                const double* x = (which == 0 ? V : K) + j * d;
                for (long a = 0; a < d; ++a) o[a] += s * x[a];
            }
        } else {
            for (long q = i; q < hi; ++q) {
                double w = pow(lam, (double)(q - i));
                double s = w * (which == 2 ? dot(dO + q * d, V + i * d, d) : dot(Q + q * d, K + i * d, d));
                const double* x = (which == 2 ? Q : dO) + q * d;
                for (long a = 0; a < d; ++a) o[a] += s * x[a];
            }
        }
    }
    free(doc);
}

/* ================================================================== */
/* Softmax attention, the compute line of Algorithm "AllGather-based   */
/* Context Parallelism": O = Softmax(Q K^T / sqrt(d)) V, row-wise, over */
/* the keys of the query's document; causal != 0 keeps keys j <= i only */
/* (the algorithm prints no mask; the text names causal and document    */
/* masks as what the gathered form makes easy).                         */
/* lse (may be NULL) receives log(sum_j exp(s_ij)) per row.             */
/* ================================================================== */
void lasp2_oracle_softmax_fwd(const double* Q, const double* K, const double* V,
                              double* O, double* lse, long G, long N, long d,
                              const long* cu, long n_docs, int causal)
{
    long* doc = doc_ids(N, cu, n_docs);
    double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (long g = 0; g < G; ++g) {
        for (long i = 0; i < N; ++i) {
            long lo = cu[doc[i]], hi = causal ? i + 1 : cu[doc[i] + 1];
            double* sc = (double*)malloc(sizeof(double) * (size_t)(hi - lo));
            double mx = -INFINITY;
            for (long j = lo; j < hi; ++j) {
                sc[j - lo] = scale * dot(Q + (g * N + i) * d, K + (g * N + j) * d, d);
                if (sc[j - lo] > mx) mx = sc[j - lo];
            }
            double sum = 0.0;
            for (long j = lo; j < hi; ++j) { sc[j - lo] = exp(sc[j - lo] - mx); sum += sc[j - lo]; }
            double* o = O + (g * N + i) * d;
            for (long b = 0; b < d; ++b) o[b] = 0.0;
            for (long j = lo; j < hi; ++j) {
                double p = sc[j - lo] / sum;
                const double* v = V + (g * N + j) * d;
                for (long b = 0; b < d; ++b) o[b] += p * v[b];
            }
            if (lse) lse[g * N + i] = mx + log(sum);
            free(sc);
        }
    }
    free(doc);
}

/*
 * Gradient of <dO, O> for softmax attention.  With P the row-softmax of the scaled scores,
 * dP_ij = dO_i . v_j and delta_i = sum_j P_ij dP_ij (= dO_i . O_i):
 *   dS_ij = P_ij (dP_ij - delta_i),
 *   dQ_i = scale sum_j dS_ij k_j,  dK_j = scale sum_i dS_ij q_i,  dV_j = sum_i P_ij dO_i.
 */
void lasp2_oracle_softmax_bwd(const double* Q, const double* K, const double* V,
                              const double* dO, double* dQ, double* dK, double* dV,
                              long G, long N, long d, const long* cu, long n_docs, int causal)
{
    long* doc = doc_ids(N, cu, n_docs);
    double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
    for (long g = 0; g < G; ++g) {
        memset(dQ + g * N * d, 0, sizeof(double) * (size_t)(N * d));
        memset(dK + g * N * d, 0, sizeof(double) * (size_t)(N * d));
        memset(dV + g * N * d, 0, sizeof(double) * (size_t)(N * d));
        for (long i = 0; i < N; ++i) {
            long lo = cu[doc[i]], hi = causal ? i + 1 : cu[doc[i] + 1];
            long n = hi - lo;
            double* p = (double*)malloc(sizeof(double) * (size_t)n);
            double* dp = (double*)malloc(sizeof(double) * (size_t)n);
            double mx = -INFINITY, sum = 0.0, delta = 0.0;
            for (long j = lo; j < hi; ++j) {
                p[j - lo] = scale * dot(Q + (g * N + i) * d, K + (g * N + j) * d, d);
                if (p[j - lo] > mx) mx = p[j - lo];
            }
            for (long j = lo; j < hi; ++j) { p[j - lo] = exp(p[j - lo] - mx); sum += p[j - lo]; }
            for (long j = lo; j < hi; ++j) {
                p[j - lo] /= sum;
                dp[j - lo] = dot(dO + (g * N + i) * d, V + (g * N + j) * d, d);
                delta += p[j - lo] * dp[j - lo];
            }
            for (long j = lo; j < hi; ++j) {
                double ds = p[j - lo] * (dp[j - lo] - delta);
                for (long a = 0; a < d; ++a) {
                    dQ[(g * N + i) * d + a] += scale * ds * K[(g * N + j) * d + a];
                    dK[(g * N + j) * d + a] += scale * ds * Q[(g * N + i) * d + a];
                    dV[(g * N + j) * d + a] += p[j - lo] * dO[(g * N + i) * d + a];
                }
            }
            free(p);
            free(dp);
        }
    }
    free(doc);
}

/* Selected rows of the softmax output (one group; Q,K,V are [N][d]). */
void lasp2_oracle_softmax_rows(const double* Q, const double* K, const double* V, long N, long d,
                               const long* cu, long n_docs, const long* rows, long n_rows,
                               int causal, double* out, double* lse)
{
    long* doc = doc_ids(N, cu, n_docs);
    double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < n_rows; ++r) {
        long i = rows[r];
        long lo = cu[doc[i]], hi = causal ? i + 1 : cu[doc[i] + 1];
        double* sc = (double*)malloc(sizeof(double) * (size_t)(hi - lo));
        double mx = -INFINITY, sum = 0.0;
        for (long j = lo; j < hi; ++j) {
            sc[j - lo] = scale * dot(Q + i * d, K + j * d, d);
            if (sc[j - lo] > mx) mx = sc[j - lo];
        }
        for (long j = lo; j < hi; ++j) { sc[j - lo] = exp(sc[j - lo] - mx); sum += sc[j - lo]; }
        double* o = out + r * d;
        for (long b = 0; b < d; ++b) o[b] = 0.0;
        for (long j = lo; j < hi; ++j)
            for (long b = 0; b < d; ++b) o[b] += sc[j - lo] / sum * V[j * d + b];
        if (lse) lse[r] = mx + log(sum);
        free(sc);
    }
    free(doc);
}

/*
 * Selected rows of dQ (which = 0), dK (1) or dV (2) of the softmax gradient above, one group;
 * Q, K, V, dO are [N][d].  lse[i] and delta[i] = dO_i . O_i come from this oracle's own forward
 * over the whole group; with them P_ij = exp(scale q_i . k_j - lse_i) needs no further row sums,
 * which is what makes single rows of dK and dV (sums over all queries) affordable at sizes
 * where the full gradient is not.
 */
void lasp2_oracle_softmax_bwd_rows(const double* Q, const double* K, const double* V,
                                   const double* dO, const double* lse, const double* delta,
                                   long N, long d, const long* cu, long n_docs, const long* rows,
                                   long n_rows, int which, int causal, double* out)
{
    long* doc = doc_ids(N, cu, n_docs);
    double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < n_rows; ++r) {
        long t = rows[r];
        long dlo = cu[doc[t]], dhi = cu[doc[t] + 1];
        double* o = out + r * d;
        for (long a = 0; a < d; ++a) o[a] = 0.0;
        if (which == 0) {
            long hi = causal ? t + 1 : dhi;
            for (long j = dlo; j < hi; ++j) {
                double p = exp(scale * dot(Q + t * d, K + j * d, d) - lse[t]);
                double ds = p * (dot(dO + t * d, V + j * d, d) - delta[t]);
                for (long a = 0; a < d; ++a) o[a] += scale * ds * K[j * d + a];
            }
        } else {
            long lo = causal ? t : dlo;
            for (long i = lo; i < dhi; ++i) {
                double p = exp(scale * dot(Q + i * d, K + t * d, d) - lse[i]);
                if (which == 1) {
                    double ds = p * (dot(dO + i * d, V + t * d, d) - delta[i]);
                    for (long a = 0; a < d; ++a) o[a] += scale * ds * Q[i * d + a];
                } else {
                    for (long a = 0; a < d; ++a) o[a] += p * dO[i * d + a];
                }
            }
        }
    }
    free(doc);
}
