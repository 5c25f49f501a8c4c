/*
 * CPU oracle for Scrambled Distributed Attention (FedRAG, Section 4).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the hot path computes.  It shares no code with the HIP library, is
 * never called by it, and may be used only by the tests, by the smoke check
 * and by the benchmark's cpu_baseline leg.
 *
 * Conventions (Section 2.1 footnote): vectors are rows, d is the head
 * dimension.  All tensors are dense row-major fp64:
 *     Q        [B, Hq,  Lq, d]
 *     K, V     [B, Hkv, Lk, d]
 *     Phi      [Hkv, d, d]          one scrambling matrix per KV head
 *     perm     [n_perm, L] int32    gather indices, out row j <- in row perm[j]
 * Query head h reads KV head h / (Hq / Hkv).
 *
 * One exception to fp64: the transport codec (oracle_quantize_rows /
 * oracle_dequantize_rows) decides integer codes by floating point, and takes
 * those decisions in IEEE single precision, operation by operation, as its
 * header states - the precision is part of that definition.
 *
 * Every loop below follows the order of the equation it cites; there is no
 * blocking, fusion or reordering.  OpenMP is used only across independent
 * (batch, head) units so that the benchmark can time it on all host cores.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 0; /* 0 = OpenMP default */

void oracle_set_threads(int n) { g_threads = n; }

int oracle_get_threads(void)
{
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}

#ifdef _OPENMP
#define NTHREADS() (g_threads > 0 ? g_threads : omp_get_max_threads())
#else
#define NTHREADS() 1
#endif

/* ------------------------------------------------------------------------ */
/* Eq. (1): Attention(Q,K,V) = softmax(Q K^T / sqrt(d)) V, written out.      */
/* Also returns lse[b,h,i] = ln sum_t exp(Q K^T / sqrt(d))_{i,t}, which is   */
/* the logarithm of the normalisation factor of Section 4.1.                 */
/* The row of logits is materialised, soft-maxed with the row maximum        */
/* subtracted (the textbook stable form of the same function), then          */
/* multiplied into V.                                                        */
/* ------------------------------------------------------------------------ */
void oracle_plain_attention(const double *Q, const double *K, const double *V,
                            int B, int Hq, int Hkv, int64_t Lq, int64_t Lk, int d,
                            double *O, double *lse)
{
    const int G = Hq / Hkv;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(NTHREADS())
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const double *Qh = Q + ((int64_t)b * Hq + h) * Lq * d;
            const double *Kg = K + ((int64_t)b * Hkv + g) * Lk * d;
            const double *Vg = V + ((int64_t)b * Hkv + g) * Lk * d;
            double *Oh = O + ((int64_t)b * Hq + h) * Lq * d;
            double *lh = lse + ((int64_t)b * Hq + h) * Lq;
            double *row = (double *)malloc(sizeof(double) * (size_t)(Lk > 0 ? Lk : 1));
            for (int64_t i = 0; i < Lq; ++i) {
                /* logits of row i */
                double mx = -INFINITY;
                for (int64_t t = 0; t < Lk; ++t) {
                    double s = 0.0;
                    for (int c = 0; c < d; ++c) s += Qh[i * d + c] * Kg[t * d + c];
                    s *= inv_sqrt_d;
                    row[t] = s;
                    if (s > mx) mx = s;
                }
                /* softmax of the row */
                double sum = 0.0;
                for (int64_t t = 0; t < Lk; ++t) {
                    row[t] = exp(row[t] - mx);
                    sum += row[t];
                }
                for (int c = 0; c < d; ++c) Oh[i * d + c] = 0.0;
                if (Lk == 0) { /* no keys: empty sum */
                    lh[i] = -INFINITY;
                    continue;
                }
                for (int64_t t = 0; t < Lk; ++t) row[t] /= sum;
                /* times V */
                for (int64_t t = 0; t < Lk; ++t)
                    for (int c = 0; c < d; ++c) Oh[i * d + c] += row[t] * Vg[t * d + c];
                lh[i] = mx + log(sum);
            }
            free(row);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Section 4.1, literally: node-local output O_i = softmax(Q K_i^T/sqrt d)V_i*/
/* and the RAW normalisation factor [w_i]_l = sum_t exp(Q K_i^T/sqrt d)_{l,t}*/
/* with no maximum subtracted anywhere.  Only usable while every logit stays */
/* below ~700 (fp64 exp range); the tests use it on benign data to pin the   */
/* log-domain functions below.                                               */
/* ------------------------------------------------------------------------ */
void oracle_local_attention_raw(const double *Q, const double *K, const double *V,
                                int B, int Hq, int Hkv, int64_t Lq, int64_t Lk, int d,
                                double *O, double *w)
{
    const int G = Hq / Hkv;
    const double sqrt_d = sqrt((double)d);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const double *Qh = Q + ((int64_t)b * Hq + h) * Lq * d;
            const double *Kg = K + ((int64_t)b * Hkv + g) * Lk * d;
            const double *Vg = V + ((int64_t)b * Hkv + g) * Lk * d;
            double *Oh = O + ((int64_t)b * Hq + h) * Lq * d;
            double *wh = w + ((int64_t)b * Hq + h) * Lq;
            for (int64_t l = 0; l < Lq; ++l) {
                double wl = 0.0;
                for (int c = 0; c < d; ++c) Oh[l * d + c] = 0.0;
                for (int64_t t = 0; t < Lk; ++t) {
                    double s = 0.0;
                    for (int c = 0; c < d; ++c) s += Qh[l * d + c] * Kg[t * d + c];
                    const double e = exp(s / sqrt_d);
                    wl += e;
                    for (int c = 0; c < d; ++c) Oh[l * d + c] += e * Vg[t * d + c];
                }
                for (int c = 0; c < d; ++c) Oh[l * d + c] = (Lk > 0) ? Oh[l * d + c] / wl : 0.0;
                wh[l] = wl;
            }
        }
}

/* Section 4.1, global aggregation, literally:                               */
/*   Attention = (sum_i w_i (.) O_i) / (sum_i w_i), row-wise.                */
/* O_parts [M, rows, d], w [M, rows] -> O [rows, d], w_total [rows].         */
void oracle_aggregate_raw(const double *O_parts, const double *w, int M, int64_t rows, int d,
                          double *O, double *w_total)
{
    for (int64_t r = 0; r < rows; ++r) {
        double den = 0.0;
        for (int i = 0; i < M; ++i) den += w[(int64_t)i * rows + r];
        for (int c = 0; c < d; ++c) {
            double num = 0.0;
            for (int i = 0; i < M; ++i)
                num += w[(int64_t)i * rows + r] * O_parts[((int64_t)i * rows + r) * d + c];
            O[r * d + c] = (den > 0.0) ? num / den : 0.0;
        }
        w_total[r] = den;
    }
}

/* ------------------------------------------------------------------------ */
/* Enc of the scrambled attention protocol (Section 4.2): one operand.       */
/*   out[b,h,j,:] = X[b,h,perm[j],:] . Phi[h / G]                            */
/* i.e. the token permutation P X (gather reading) followed by the feature   */
/* scramble (row vector times matrix).  Called with                          */
/*   X=Q, Phi=Phi_KQ,      G=Hq/Hkv                                          */
/*   X=K, Phi=Phi_KQ^{-T}, G=1                                               */
/*   X=V, Phi=Phi_V,       G=1                                               */
/* perm may be NULL (identity).  n_perm is 1 (shared by every sequence) or B.*/
/* ------------------------------------------------------------------------ */
void oracle_scramble(const double *X, const double *Phi, const int32_t *perm, int n_perm,
                     int B, int H, int G, int64_t L, int d, double *out)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(NTHREADS())
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const double *Xh = X + ((int64_t)b * H + h) * L * d;
            double *Yh = out + ((int64_t)b * H + h) * L * d;
            const double *P = Phi + (int64_t)(h / G) * d * d;
            const int32_t *pi = perm ? perm + (n_perm > 1 ? (int64_t)b * L : 0) : NULL;
            for (int64_t j = 0; j < L; ++j) {
                const int64_t src = pi ? (int64_t)pi[j] : j;
                for (int c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int k = 0; k < d; ++k) acc += Xh[src * d + k] * P[(int64_t)k * d + c];
                    Yh[j * d + c] = acc;
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------ */
/* What one Compute Node returns for one KV shard (Section 4.1), carried in  */
/* the log domain: O_i as defined there, and lse_i = ln [w_i].               */
/* Per query row: logits s_t, running over the shard's keys once to find     */
/* m = max_t s_t, then p_t = exp(s_t - m), l = sum p_t,                      */
/* O = sum p_t v_t / l,  lse = m + ln l.  An empty shard gives O=0, -inf.    */
/* ------------------------------------------------------------------------ */
void oracle_partial_attn(const double *Q, const double *K, const double *V,
                         int B, int Hq, int Hkv, int64_t Lq, int64_t Lk, int d,
                         double scale, double *O, double *lse)
{
    const int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(NTHREADS())
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const double *Qh = Q + ((int64_t)b * Hq + h) * Lq * d;
            const double *Kg = K + ((int64_t)b * Hkv + g) * Lk * d;
            const double *Vg = V + ((int64_t)b * Hkv + g) * Lk * d;
            double *Oh = O + ((int64_t)b * Hq + h) * Lq * d;
            double *lh = lse + ((int64_t)b * Hq + h) * Lq;
            double *s = (double *)malloc(sizeof(double) * (size_t)(Lk > 0 ? Lk : 1));
            for (int64_t i = 0; i < Lq; ++i) {
                double m = -INFINITY;
                for (int64_t t = 0; t < Lk; ++t) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += Qh[i * d + c] * Kg[t * d + c];
                    s[t] = dot * scale;
                    if (s[t] > m) m = s[t];
                }
                for (int c = 0; c < d; ++c) Oh[i * d + c] = 0.0;
                if (Lk == 0) {
                    lh[i] = -INFINITY;
                    continue;
                }
                double l = 0.0;
                for (int64_t t = 0; t < Lk; ++t) {
                    const double p = exp(s[t] - m);
                    l += p;
                    for (int c = 0; c < d; ++c) Oh[i * d + c] += p * Vg[t * d + c];
                }
                for (int c = 0; c < d; ++c) Oh[i * d + c] /= l;
                lh[i] = m + log(l);
            }
            free(s);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* A batch of sequences of unequal length (Section 5.2: the re-ranker scores */
/* ten query-document pairs, each its own sequence), stored padded to Lk     */
/* rows: sequence b attends to its first kv_lens[b] keys only, as            */
/* oracle_partial_attn does over a shard of that length (0 keys: O = 0,      */
/* lse = -inf).                                                              */
/* ------------------------------------------------------------------------ */
void oracle_partial_attn_varlen(const double *Q, const double *K, const double *V, const int32_t *kv_lens,
                                int B, int Hq, int Hkv, int64_t Lq, int64_t Lk, int d,
                                double scale, double *O, double *lse)
{
    const int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(NTHREADS())
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const int64_t n = kv_lens[b];
            const double *Qh = Q + ((int64_t)b * Hq + h) * Lq * d;
            const double *Kg = K + ((int64_t)b * Hkv + g) * Lk * d;
            const double *Vg = V + ((int64_t)b * Hkv + g) * Lk * d;
            double *Oh = O + ((int64_t)b * Hq + h) * Lq * d;
            double *lh = lse + ((int64_t)b * Hq + h) * Lq;
            double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
            for (int64_t i = 0; i < Lq; ++i) {
                for (int c = 0; c < d; ++c) Oh[i * d + c] = 0.0;
                if (n == 0) {
                    lh[i] = -INFINITY;
                    continue;
                }
                double m = -INFINITY;
                for (int64_t t = 0; t < n; ++t) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += Qh[i * d + c] * Kg[t * d + c];
                    s[t] = dot * scale;
                    if (s[t] > m) m = s[t];
                }
                double l = 0.0;
                for (int64_t t = 0; t < n; ++t) {
                    const double p = exp(s[t] - m);
                    l += p;
                    for (int c = 0; c < d; ++c) Oh[i * d + c] += p * Vg[t * d + c];
                }
                for (int c = 0; c < d; ++c) Oh[i * d + c] /= l;
                lh[i] = m + log(l);
            }
            free(s);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* The Inquirer's own part of a decoder layer's attention (Section 5.3,      */
/* prefill and decoding phases): the queries of the current input segment    */
/* against the K, V the Inquirer holds itself, where a token attends only to */
/* itself and the tokens before it.  The Lq queries are the LAST Lq of the   */
/* Lk local tokens, so query i sees keys t <= i + (Lk - Lq).  Same outputs   */
/* as oracle_partial_attn: O as in Section 4.1 and lse = ln w, to be         */
/* aggregated with the descrambled remote result.  Needs Lk >= Lq.           */
/* ------------------------------------------------------------------------ */
void oracle_local_causal_attn(const double *Q, const double *K, const double *V,
                              int B, int Hq, int Hkv, int64_t Lq, int64_t Lk, int d,
                              double scale, double *O, double *lse)
{
    const int G = Hq / Hkv;
    const int64_t off = Lk - Lq;
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(NTHREADS())
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const double *Qh = Q + ((int64_t)b * Hq + h) * Lq * d;
            const double *Kg = K + ((int64_t)b * Hkv + g) * Lk * d;
            const double *Vg = V + ((int64_t)b * Hkv + g) * Lk * d;
            double *Oh = O + ((int64_t)b * Hq + h) * Lq * d;
            double *lh = lse + ((int64_t)b * Hq + h) * Lq;
            double *s = (double *)malloc(sizeof(double) * (size_t)(Lk > 0 ? Lk : 1));
            for (int64_t i = 0; i < Lq; ++i) {
                const int64_t n_vis = i + off + 1;  /* keys 0 .. i + off */
                double m = -INFINITY;
                for (int64_t t = 0; t < n_vis; ++t) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += Qh[i * d + c] * Kg[t * d + c];
                    s[t] = dot * scale;
                    if (s[t] > m) m = s[t];
                }
                double l = 0.0;
                for (int c = 0; c < d; ++c) Oh[i * d + c] = 0.0;
                for (int64_t t = 0; t < n_vis; ++t) {
                    const double p = exp(s[t] - m);
                    l += p;
                    for (int c = 0; c < d; ++c) Oh[i * d + c] += p * Vg[t * d + c];
                }
                for (int c = 0; c < d; ++c) Oh[i * d + c] /= l;
                lh[i] = m + log(l);
            }
            free(s);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Global aggregation of Section 4.1 with w_i = exp(lse_i), evaluated in the */
/* log domain: M = max_i lse_i, a_i = exp(lse_i - M),                        */
/* O = sum a_i O_i / sum a_i, lse = M + ln sum a_i.                          */
/* A shard with lse = -inf has weight zero; if all are -inf, O = 0, -inf.    */
/* O_parts [S, rows, d], lses [S, rows] -> O [rows, d], lse [rows].          */
/* ------------------------------------------------------------------------ */
void oracle_lse_merge(const double *O_parts, const double *lses, int S, int64_t rows, int d,
                      double *O, double *lse)
{
    for (int64_t r = 0; r < rows; ++r) {
        double M = -INFINITY;
        for (int i = 0; i < S; ++i)
            if (lses[(int64_t)i * rows + r] > M) M = lses[(int64_t)i * rows + r];
        if (M == -INFINITY) {
            for (int c = 0; c < d; ++c) O[r * d + c] = 0.0;
            lse[r] = -INFINITY;
            continue;
        }
        double den = 0.0;
        for (int i = 0; i < S; ++i) den += exp(lses[(int64_t)i * rows + r] - M);
        for (int c = 0; c < d; ++c) {
            double num = 0.0;
            for (int i = 0; i < S; ++i) {
                const double a = exp(lses[(int64_t)i * rows + r] - M);
                if (a > 0.0) num += a * O_parts[((int64_t)i * rows + r) * d + c];
            }
            O[r * d + c] = num / den;
        }
        lse[r] = M + log(den);
    }
}

/* ------------------------------------------------------------------------ */
/* Dec of the protocol (Section 4.2): P_Q^{-1} (.) Phi_V^{-1}.               */
/*   out[b,h,perm[i],:] = O[b,h,i,:] . PhiInv[h / G]                         */
/* perm is the SAME gather array that scrambled Q (NULL = identity), so the  */
/* inverse permutation is a scatter.                                         */
/* ------------------------------------------------------------------------ */
void oracle_unscramble(const double *O, const double *PhiInv, const int32_t *perm,
                       int B, int H, int G, int64_t L, int d, double *out)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(NTHREADS())
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const double *Xh = O + ((int64_t)b * H + h) * L * d;
            double *Yh = out + ((int64_t)b * H + h) * L * d;
            const double *P = PhiInv + (int64_t)(h / G) * d * d;
            for (int64_t i = 0; i < L; ++i) {
                const int64_t dst = perm ? (int64_t)perm[i] : i;
                for (int c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int k = 0; k < d; ++k) acc += Xh[i * d + k] * P[(int64_t)k * d + c];
                    Yh[dst * d + c] = acc;
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------ */
/* The structured scrambling matrix of Section 4.2 ("Our construction"),      */
/* Phi = S1 P1 H P2 S2, applied to row vectors factor by factor in the order */
/* the factors are written: scale, channel permutation, normalised Hadamard, */
/* channel permutation, scale.  Key of one KV head, permutations as gathers: */
/*   u[i] = x[i] * a[i]                       (x S1)                         */
/*   v[j] = u[g1[j]]                          (. P1)                         */
/*   w[m] = sum_i v[i] Hs[i][m] / sqrt(d)     (. H),  Hs[i][m] = +1 or -1    */
/*          according to the parity of popcount(i AND m): Sylvester's        */
/*          construction, d a power of two                                   */
/*   y[j] = w[g2[j]] * b[j]                   (. P2 S2)                      */
/* Rows are gathered (scatter = 0: out row j <- in row perm[j], Enc) or      */
/* scattered (scatter = 1: out row perm[i] <- in row i, Dec).                */
/* ------------------------------------------------------------------------ */
static int parity_of(unsigned x)
{
    int p = 0;
    while (x) { p ^= (int)(x & 1u); x >>= 1; }
    return p;
}

void oracle_structured(const double *X, const double *a, const int32_t *g1, const int32_t *g2,
                       const double *b, const int32_t *perm, int n_perm, int scatter,
                       int B, int H, int G, int64_t L, int d, double *out)
{
    const double norm = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(NTHREADS())
    for (int bb = 0; bb < B; ++bb) {
        for (int h = 0; h < H; ++h) {
            const double *Xh = X + ((int64_t)bb * H + h) * L * d;
            double *Yh = out + ((int64_t)bb * H + h) * L * d;
            const int64_t ko = (int64_t)(h / G) * d;
            const int32_t *pi = perm ? perm + (n_perm > 1 ? (int64_t)bb * L : 0) : NULL;
            double *v = (double *)malloc(sizeof(double) * (size_t)d * 2);
            double *w = v + d;
            for (int64_t r = 0; r < L; ++r) {
                const int64_t src = (pi && !scatter) ? (int64_t)pi[r] : r;
                const int64_t dst = (pi && scatter) ? (int64_t)pi[r] : r;
                for (int j = 0; j < d; ++j) {
                    const int i = g1[ko + j];
                    v[j] = Xh[src * d + i] * a[ko + i];
                }
                for (int m = 0; m < d; ++m) {
                    double acc = 0.0;
                    for (int i = 0; i < d; ++i)
                        acc += parity_of((unsigned)i & (unsigned)m) ? -v[i] : v[i];
                    w[m] = acc * norm;
                }
                for (int j = 0; j < d; ++j) Yh[dst * d + j] = w[g2[ko + j]] * b[ko + j];
            }
            free(v);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Transport codec (Section 7.5: "standard affine min-max quantization" of   */
/* the intermediate states before they are sent).  One row = one token's d   */
/* channels, quantised on its own range to `bits` bits (8 or 4):             */
/*   lo = min_c x_c, hi = max_c x_c, levels = 2^bits - 1,                    */
/*   scale = (hi - lo) / levels,  steps = levels / (hi - lo),                */
/*   code_c = clamp(floor((x_c - lo) * steps + 1/2), 0, levels)   (0 when    */
/*            hi = lo: a constant row),                                      */
/*   dequantised value = code_c * scale + lo.                                */
/* A code is an integer decided by floating point, so the precision of that  */
/* decision is part of the definition: every operation above is an IEEE      */
/* single-precision operation, rounded once; "(x - lo) * steps + 1/2" and    */
/* "code * scale + lo" are one fused multiply-add each.  This is the one     */
/* place where the oracle computes in fp32 instead of fp64, on purpose.      */
/* params[r] = (scale, lo).  4-bit codes are packed two per byte, channel    */
/* 2k in the low half and channel 2k+1 in the high half.                     */
/* ------------------------------------------------------------------------ */
void oracle_quantize_rows(const float *X, int64_t n_rows, int d, int bits, uint8_t *codes, float *params)
{
    const int levels = (1 << bits) - 1;
    const int row_bytes = d * bits / 8;
#pragma omp parallel for schedule(static) num_threads(NTHREADS())
    for (int64_t r = 0; r < n_rows; ++r) {
        const float *x = X + r * d;
        float lo = x[0], hi = x[0];
        for (int c = 1; c < d; ++c) {
            if (x[c] < lo) lo = x[c];
            if (x[c] > hi) hi = x[c];
        }
        const float range = hi - lo;
        const float scale = range / (float)levels;
        const float steps = (float)levels / range;   /* unused (inf) for a constant row */
        params[2 * r] = scale;
        params[2 * r + 1] = lo;
        uint8_t *out = codes + r * row_bytes;
        for (int c = 0; c < row_bytes; ++c) out[c] = 0;
        for (int c = 0; c < d; ++c) {
            int q = 0;
            if (range > 0.0f) {
                const float t = x[c] - lo;
                const float v = floorf(fmaf(t, steps, 0.5f));
                q = (int)fminf(fmaxf(v, 0.0f), (float)levels);   /* clamped as a float: steps may be huge */
            }
            if (bits == 8) out[c] = (uint8_t)q;
            else out[c / 2] |= (uint8_t)(q << (4 * (c % 2)));
        }
    }
}

void oracle_dequantize_rows(const uint8_t *codes, const float *params, int64_t n_rows, int d, int bits, float *X)
{
    const int row_bytes = d * bits / 8;
#pragma omp parallel for schedule(static) num_threads(NTHREADS())
    for (int64_t r = 0; r < n_rows; ++r) {
        const uint8_t *in = codes + r * row_bytes;
        const float scale = params[2 * r], lo = params[2 * r + 1];
        for (int c = 0; c < d; ++c) {
            const int q = bits == 8 ? in[c] : (in[c / 2] >> (4 * (c % 2))) & 15;
            X[r * d + c] = fmaf((float)q, scale, lo);
        }
    }
}

/* inv[perm[j]] = j : the permutation that undoes the gather `perm`. */
void oracle_invert_perm(const int32_t *perm, int64_t L, int32_t *inv)
{
    for (int64_t j = 0; j < L; ++j) inv[perm[j]] = (int32_t)j;
}
