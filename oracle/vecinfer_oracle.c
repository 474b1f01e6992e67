/*
 * VecInfer CPU oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, float64 implementation of what the fused VQ decode-attention
 * path computes, written from the paper's definitions.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the GPU
 * library shares no code, header, table or constant with this file.
 *
 * Every function works on doubles.  The caller widens fp16/fp32 inputs to
 * double (an exact conversion) before calling, so the oracle sees exactly the
 * values the GPU kernels see.
 *
 * What follows which passage of the paper:
 *   vo_hadamard            Sec. 3.2, Eq. 5 (recursive Walsh-Hadamard matrix)
 *   vo_smoothing_factors   Sec. 3.2, Eq. 4
 *   vo_transform_keys      Sec. 3.2, Eq. 3 (key side) then Eq. 6; Alg. 1 "Preprocessing"
 *   vo_transform_query     Sec. 3.2, Eq. 3 (query side) then Eq. 6; Eq. 7
 *   vo_vq_encode           Sec. 2.2, Eq. 2; Sec. 3.2, Eq. 8
 *   vo_vq_dequantize       Sec. 2.2 (last paragraph): VQ^{-1} = centroid lookup
 *   vo_vq_attention        Sec. 3.2, Eq. 10 (explicit dequantize-then-attend)
 *   vo_vq_attention_alg1   App. A, Alg. 1 as a self-check of Eq. 10: lookup-table scores, tiles, LSE merge
 *   vo_vq_attention_residual  Eq. 10 plus the full-precision residual window of Sec. 4.1
 *                          (the 128 most recent tokens kept unquantized)
 *   vo_kmeans_update       centroid update of one Lloyd iteration of the K-Means codebook training
 *                          (Sec. 2.2: the codebook is built by K-Means; Sec. 4.1: at most 30 iterations)
 *   vo_vq_encode_g, vo_vq_dequantize_g, vo_vq_attention_g, vo_encode_batch_g, vo_decode_batch_g
 *                          the same definitions (Eq. 2, VQ^{-1}, Eq. 10) for codes of up to 16 bits and
 *                          for a codebook shared by all sub-spaces, as Alg. 1 states it (one C_k, one
 *                          C_v of 2^b centroids; Sec. 5.3 sizes the codebook at 2^b * d * 2 bytes), which the
 *                          configurations with 10- and 12-bit codes (d8b12, d4b12, d4b10; Sec. 4.1,
 *                          Tables 1-3) call for
 *   vo_kmeans_update_g     the same update for a codebook shared by the sub-spaces (pooled sub-vectors)
 *   vo_merge_splits        log-sum-exp merge of per-split (o, L) pairs; the paper
 *                          returns L (Alg. 1 step 22) but does not print the merge
 *
 * The OpenMP pragmas only hand independent output rows to different threads;
 * no arithmetic is blocked, fused or reordered by them.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int vo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void vo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Eq. 5: H_1 = [1];  H_{2n} = (1/sqrt 2) [[H_n, H_n], [H_n, -H_n]].
 * H is D x D row-major, D a power of two.  Returns 0, or -1 if D is not. */
int vo_hadamard(int D, double *H)
{
    if (D < 1 || (D & (D - 1)) != 0) return -1;
    const double r = 1.0 / sqrt(2.0);
    H[0] = 1.0;
    /* grow the top-left n x n block into the top-left 2n x 2n block */
    for (int n = 1; n < D; n *= 2) {
        /* scale the existing block first, then copy it into the other three */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) H[i * D + j] *= r;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                const double h = H[i * D + j];
                H[i * D + (j + n)] = h;
                H[(i + n) * D + j] = h;
                H[(i + n) * D + (j + n)] = -h;
            }
    }
    return 0;
}

/* Eq. 4: lambda_i = sqrt(max_n |K[n,i]|), K is [N, D]. */
void vo_smoothing_factors(const double *K, int64_t N, int D, double *lam)
{
    for (int i = 0; i < D; ++i) {
        double mx = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            const double a = fabs(K[n * D + i]);
            if (a > mx) mx = a;
        }
        lam[i] = sqrt(mx);
    }
}

/* Key side of the dual transform: Kt[n,:] = (K[n,:] diag(lam)^-1) H_D.
 * H is the dense D x D matrix from vo_hadamard. */
void vo_transform_keys(const double *K, int64_t N, int D, const double *lam,
                       const double *H, double *Kt)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *y = (double *)malloc(sizeof(double) * (size_t)D);
        for (int i = 0; i < D; ++i) y[i] = K[n * D + i] / lam[i];
        for (int j = 0; j < D; ++j) {
            double acc = 0.0;
            for (int i = 0; i < D; ++i) acc += y[i] * H[i * D + j];
            Kt[n * D + j] = acc;
        }
        free(y);
    }
}

/* Query side: qt = (q diag(lam)) H_D. */
void vo_transform_query(const double *q, int D, const double *lam,
                        const double *H, double *qt)
{
    for (int j = 0; j < D; ++j) {
        double acc = 0.0;
        for (int i = 0; i < D; ++i) acc += (q[i] * lam[i]) * H[i * D + j];
        qt[j] = acc;
    }
}

/* Eq. 2 applied to every sub-vector of every row.
 *   X   [N, D]      rows to quantize
 *   cb  [M, C, d]   one codebook of C centroids per sub-space, M = D / d
 *   idx [N, M]      argmin_c sum_j (x[m*d+j] - cb[m][c][j])^2, lowest c on ties
 *   relgap [N, M] or NULL: (second-smallest - smallest) / max(smallest, 1e-300),
 *                          so a caller can tell a near-tie from a real mismatch. */
void vo_vq_encode(const double *X, int64_t N, int D, int d, int C,
                  const double *cb, uint8_t *idx, double *relgap)
{
    const int M = D / d;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            const double *x = X + n * D + (int64_t)m * d;
            double best = INFINITY, second = INFINITY;
            int arg = 0;
            for (int c = 0; c < C; ++c) {
                const double *cen = cb + ((int64_t)m * C + c) * d;
                double dist = 0.0;
                for (int j = 0; j < d; ++j) {
                    const double t = x[j] - cen[j];
                    dist += t * t;
                }
                if (dist < best) {
                    second = best;
                    best = dist;
                    arg = c;
                } else if (dist < second) {
                    second = dist;
                }
            }
            idx[n * M + m] = (uint8_t)arg;
            if (relgap) relgap[n * M + m] = (second - best) / (best > 1e-300 ? best : 1e-300);
        }
    }
}

/* VQ^{-1}: Xhat[n, m*d + j] = cb[m][idx[n,m]][j]. */
void vo_vq_dequantize(const uint8_t *idx, int64_t N, int D, int d, int C,
                      const double *cb, double *Xhat)
{
    const int M = D / d;
    for (int64_t n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            const double *cen = cb + ((int64_t)m * C + idx[n * M + m]) * d;
            for (int j = 0; j < d; ++j) Xhat[n * D + (int64_t)m * d + j] = cen[j];
        }
}

/* Eq. 10 for one query row against one KV head:
 *   s_n = qt . Khat[n,:] / sqrt(D),  p = softmax(s),  o = p Vhat,
 *   L = log sum_n exp(s_n)   (Alg. 1 step 22 computes the same L = m + log l).
 * Khat and Vhat are dequantized explicitly; nothing is tiled or fused.
 * Returns 0, or -1 if N < 1 (softmax of nothing is undefined). */
int vo_vq_attention(const double *qt, const uint8_t *kidx, const uint8_t *vidx,
                    const double *cb_k, const double *cb_v, int64_t N, int D,
                    int d_k, int d_v, int C, double *out, double *lse)
{
    if (N < 1) return -1;
    double *Khat = (double *)malloc(sizeof(double) * (size_t)N * D);
    double *Vhat = (double *)malloc(sizeof(double) * (size_t)N * D);
    double *s = (double *)malloc(sizeof(double) * (size_t)N);
    vo_vq_dequantize(kidx, N, D, d_k, C, cb_k, Khat);
    vo_vq_dequantize(vidx, N, D, d_v, C, cb_v, Vhat);
    const double scale = 1.0 / sqrt((double)D);
    double mx = -INFINITY;
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int i = 0; i < D; ++i) acc += qt[i] * Khat[n * D + i];
        s[n] = acc * scale;
        if (s[n] > mx) mx = s[n];
    }
    double denom = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        s[n] = exp(s[n] - mx);
        denom += s[n];
    }
    for (int i = 0; i < D; ++i) out[i] = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        const double p = s[n] / denom;
        for (int i = 0; i < D; ++i) out[i] += p * Vhat[n * D + i];
    }
    if (lse) *lse = mx + log(denom);
    free(Khat);
    free(Vhat);
    free(s);
    return 0;
}

/* Eq. 10 with a residual window (Sec. 4.1 keeps the most recent tokens, 128 of them in the
 * paper's runs, in full precision).  The N quantized tokens are scored as in vo_vq_attention
 * (transformed query against dequantized transformed keys); the R window tokens are scored
 * with the raw query against their raw keys, which is the same quantity by Eq. 7; one softmax
 * runs over all N + R scores and the window contributes its raw values.
 * Returns 0, or -1 if N + R < 1. */
int vo_vq_attention_residual(const double *qt, const double *q_raw, const uint8_t *kidx,
                             const uint8_t *vidx, const double *cb_k, const double *cb_v,
                             int64_t N, const double *kres, const double *vres, int64_t R, int D,
                             int d_k, int d_v, int C, double *out, double *lse)
{
    if (N < 0 || R < 0 || N + R < 1) return -1;
    const int64_t T = N + R;
    double *Kall = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1) * D);
    double *Vall = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *s = (double *)malloc(sizeof(double) * (size_t)T);
    if (N > 0) {
        vo_vq_dequantize(kidx, N, D, d_k, C, cb_k, Kall);
        vo_vq_dequantize(vidx, N, D, d_v, C, cb_v, Vall);
    }
    for (int64_t r = 0; r < R; ++r)
        for (int i = 0; i < D; ++i) Vall[(N + r) * D + i] = vres[r * D + i];
    const double scale = 1.0 / sqrt((double)D);
    double mx = -INFINITY;
    for (int64_t n = 0; n < T; ++n) {
        double acc = 0.0;
        if (n < N)
            for (int i = 0; i < D; ++i) acc += qt[i] * Kall[n * D + i];
        else
            for (int i = 0; i < D; ++i) acc += q_raw[i] * kres[(n - N) * D + i];
        s[n] = acc * scale;
        if (s[n] > mx) mx = s[n];
    }
    double denom = 0.0;
    for (int64_t n = 0; n < T; ++n) {
        s[n] = exp(s[n] - mx);
        denom += s[n];
    }
    for (int i = 0; i < D; ++i) out[i] = 0.0;
    for (int64_t n = 0; n < T; ++n) {
        const double p = s[n] / denom;
        for (int i = 0; i < D; ++i) out[i] += p * Vall[n * D + i];
    }
    if (lse) *lse = mx + log(denom);
    free(Kall);
    free(Vall);
    free(s);
    return 0;
}

void vo_merge_splits(const double *o_parts, const double *L_parts, int S, int D, double *out, double *lse);

/* What App. A, Alg. 1 computes for one query row against one KV head, put together from two facts
 * rather than from the listing's running updates:
 *   (1) the score of a token is a sum of table entries: with lut[m][c] = qt_m . C_k[m][c], the dot
 *       product of qt with the dequantized key is sum_m lut[m][K_q[n][m]]  (the lookup of Sec. 3.3);
 *   (2) attention over a token range can be computed tile by tile: every tile of `Bt` tokens gets
 *       its own plain softmax result (o_t, L_t), and the tiles are joined by the log-sum-exp merge
 *       (vo_merge_splits), which is what the online rescaling of Alg. 1 amounts to.
 * The tests check that this equals the Eq. 10 definition (vo_vq_attention) for any tile size. */
int vo_vq_attention_alg1(const double *qt, const uint8_t *kidx, const uint8_t *vidx,
                         const double *cb_k, const double *cb_v, int64_t N, int D,
                         int d_k, int d_v, int C, int64_t Bt, double *out, double *lse)
{
    if (N < 1 || Bt < 1) return -1;
    const int Mk = D / d_k, Mv = D / d_v;
    const int64_t T = (N + Bt - 1) / Bt;
    if (T > 0x7fffffff) return -1;
    double *lut = (double *)malloc(sizeof(double) * (size_t)Mk * C);
    double *s = (double *)malloc(sizeof(double) * (size_t)Bt);
    double *o_t = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *L_t = (double *)malloc(sizeof(double) * (size_t)T);
    for (int m = 0; m < Mk; ++m)
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int j = 0; j < d_k; ++j)
                acc += qt[m * d_k + j] * cb_k[((int64_t)m * C + c) * d_k + j];
            lut[m * C + c] = acc;
        }
    const double scale = 1.0 / sqrt((double)D);
    for (int64_t t = 0; t < T; ++t) {
        const int64_t n0 = t * Bt;
        const int64_t nb = (N - n0 < Bt) ? (N - n0) : Bt;
        double mx = -INFINITY;
        for (int64_t r = 0; r < nb; ++r) {
            double acc = 0.0;
            for (int m = 0; m < Mk; ++m) acc += lut[m * C + kidx[(n0 + r) * Mk + m]];
            s[r] = acc * scale;
            if (s[r] > mx) mx = s[r];
        }
        double denom = 0.0;
        for (int64_t r = 0; r < nb; ++r) {
            s[r] = exp(s[r] - mx);
            denom += s[r];
        }
        double *o = o_t + t * D;
        for (int i = 0; i < D; ++i) o[i] = 0.0;
        for (int64_t r = 0; r < nb; ++r) {
            const double p = s[r] / denom;
            for (int m = 0; m < Mv; ++m) {
                const double *cen = cb_v + ((int64_t)m * C + vidx[(n0 + r) * Mv + m]) * d_v;
                for (int j = 0; j < d_v; ++j) o[m * d_v + j] += p * cen[j];
            }
        }
        L_t[t] = mx + log(denom);
    }
    vo_merge_splits(o_t, L_t, (int)T, D, out, lse);
    free(lut);
    free(s);
    free(o_t);
    free(L_t);
    return 0;
}

/* Merge S partial results of one query row, each (o_s [D], L_s) computed over a
 * disjoint token range:  L = log sum_s exp(L_s),  o = sum_s exp(L_s - L) o_s. */
void vo_merge_splits(const double *o_parts, const double *L_parts, int S, int D,
                     double *out, double *lse)
{
    double mx = -INFINITY;
    for (int s = 0; s < S; ++s)
        if (L_parts[s] > mx) mx = L_parts[s];
    double denom = 0.0;
    for (int s = 0; s < S; ++s) denom += exp(L_parts[s] - mx);
    const double L = mx + log(denom);
    for (int i = 0; i < D; ++i) out[i] = 0.0;
    for (int s = 0; s < S; ++s) {
        const double w = exp(L_parts[s] - L);
        for (int i = 0; i < D; ++i) out[i] += w * o_parts[(int64_t)s * D + i];
    }
    if (lse) *lse = L;
}

/* ---- batch drivers: loop the single-row functions over (batch, head) ---- */

/* Keys: K [B, Hkv, T, D], lam [Hkv, D], cb [Hkv, M, C, d] -> idx [B, Hkv, T, M].
 * transform != 0: smooth + Hadamard first (keys); transform == 0: raw rows (values). */
int vo_encode_batch(const double *X, const double *lam, const double *cb, int B, int Hkv,
                    int64_t T, int D, int d, int C, int transform, uint8_t *idx,
                    double *relgap)
{
    if (D % d != 0) return -1;
    const int M = D / d;
    double *H = NULL;
    if (transform) {
        H = (double *)malloc(sizeof(double) * (size_t)D * D);
        if (vo_hadamard(D, H) != 0) {
            free(H);
            return -1;
        }
    }
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g) {
            const int64_t row0 = ((int64_t)b * Hkv + g) * T;
            const double *Xbg = X + row0 * D;
            const double *cbg = cb + (int64_t)g * M * C * d;
            double *gap = relgap ? relgap + row0 * M : NULL;
            if (transform) {
                double *Kt = (double *)malloc(sizeof(double) * (size_t)T * D);
                vo_transform_keys(Xbg, T, D, lam + (int64_t)g * D, H, Kt);
                vo_vq_encode(Kt, T, D, d, C, cbg, idx + row0 * M, gap);
                free(Kt);
            } else {
                vo_vq_encode(Xbg, T, D, d, C, cbg, idx + row0 * M, gap);
            }
        }
    free(H);
    return 0;
}

/* Decode step for a batch with grouped-query heads.
 *   q     [B, Hq, D]          lam [Hkv, D]
 *   cb_k  [Hkv, Mk, C, d_k]   cb_v [Hkv, Mv, C, d_v]
 *   kidx  [B, Hkv, n_cap, Mk] vidx [B, Hkv, n_cap, Mv]
 *   seq_lens [B]  (tokens 0 .. seq_lens[b]-1 of each cache are attended)
 *   out   [B, Hq, D]          lse [B, Hq]
 * Query head h reads KV head h / (Hq / Hkv).
 * path 0: Eq. 10 explicit;  path 1: Alg. 1 with tile size Bt. */
int vo_decode_batch(const double *q, const double *lam, const double *cb_k,
                    const double *cb_v, const uint8_t *kidx, const uint8_t *vidx,
                    const int64_t *seq_lens, int B, int Hq, int Hkv, int64_t n_cap, int D,
                    int d_k, int d_v, int C, int path, int64_t Bt, double *out, double *lse)
{
    if (Hq % Hkv != 0 || D % d_k != 0 || D % d_v != 0) return -1;
    const int G = Hq / Hkv, Mk = D / d_k, Mv = D / d_v;
    double *H = (double *)malloc(sizeof(double) * (size_t)D * D);
    if (vo_hadamard(D, H) != 0) {
        free(H);
        return -1;
    }
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            double *qt = (double *)malloc(sizeof(double) * (size_t)D);
            vo_transform_query(q + ((int64_t)b * Hq + h) * D, D, lam + (int64_t)g * D, H, qt);
            const uint8_t *ki = kidx + ((int64_t)b * Hkv + g) * n_cap * Mk;
            const uint8_t *vi = vidx + ((int64_t)b * Hkv + g) * n_cap * Mv;
            const double *ck = cb_k + (int64_t)g * Mk * C * d_k;
            const double *cv = cb_v + (int64_t)g * Mv * C * d_v;
            double *o = out + ((int64_t)b * Hq + h) * D;
            double *L = lse + ((int64_t)b * Hq + h);
            int rc;
            if (path == 0)
                rc = vo_vq_attention(qt, ki, vi, ck, cv, seq_lens[b], D, d_k, d_v, C, o, L);
            else
                rc = vo_vq_attention_alg1(qt, ki, vi, ck, cv, seq_lens[b], D, d_k, d_v, C, Bt, o, L);
            if (rc != 0) {
#pragma omp atomic write
                err = -1;
            }
            free(qt);
        }
    free(H);
    return err;
}

/* Decode step with a residual window: as vo_decode_batch (path 0) plus
 *   kres, vres [B, Hkv, r_cap, D]  raw keys / values of the window
 *   res_lens   [B]                 window tokens in use per sequence (0 .. r_cap)
 * seq_lens[b] may be 0 when res_lens[b] >= 1. */
int vo_decode_residual_batch(const double *q, const double *lam, const double *cb_k,
                             const double *cb_v, const uint8_t *kidx, const uint8_t *vidx,
                             const int64_t *seq_lens, const double *kres, const double *vres,
                             const int64_t *res_lens, int B, int Hq, int Hkv, int64_t n_cap,
                             int64_t r_cap, int D, int d_k, int d_v, int C, double *out, double *lse)
{
    if (Hq % Hkv != 0 || D % d_k != 0 || D % d_v != 0) return -1;
    const int G = Hq / Hkv, Mk = D / d_k, Mv = D / d_v;
    double *H = (double *)malloc(sizeof(double) * (size_t)D * D);
    if (vo_hadamard(D, H) != 0) {
        free(H);
        return -1;
    }
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const double *qr = q + ((int64_t)b * Hq + h) * D;
            double *qt = (double *)malloc(sizeof(double) * (size_t)D);
            vo_transform_query(qr, D, lam + (int64_t)g * D, H, qt);
            const int64_t bg = (int64_t)b * Hkv + g;
            const int rc = vo_vq_attention_residual(
                qt, qr, kidx + bg * n_cap * Mk, vidx + bg * n_cap * Mv, cb_k + (int64_t)g * Mk * C * d_k,
                cb_v + (int64_t)g * Mv * C * d_v, seq_lens[b], kres + bg * r_cap * D, vres + bg * r_cap * D,
                res_lens[b], D, d_k, d_v, C, out + ((int64_t)b * Hq + h) * D, lse + ((int64_t)b * Hq + h));
            if (rc != 0) {
#pragma omp atomic write
                err = -1;
            }
            free(qt);
        }
    free(H);
    return err;
}

/* Centroid update of one Lloyd iteration (K-Means builds the codebook, Sec. 2.2; it is trained on
 * the transformed keys and on the raw values, Sec. 3.2, for at most 30 iterations, Sec. 4.1).
 * X [N, D] rows already assigned: idx [N, M] holds the code of every sub-vector (Eq. 2, from
 * vo_vq_encode).  New centroid of (m, c) = mean of the sub-vectors assigned to it; a centroid
 * nobody was assigned to keeps its old value.  cb_in, cb_out [M, C, d]; counts [M, C]. */
void vo_kmeans_update(const double *X, const uint8_t *idx, int64_t N, int D, int d, int C,
                      const double *cb_in, double *cb_out, int64_t *counts)
{
    const int M = D / d;
    for (int m = 0; m < M; ++m) {
        double *sum = (double *)calloc((size_t)C * d, sizeof(double));
        int64_t *cnt = counts + (int64_t)m * C;
        for (int c = 0; c < C; ++c) cnt[c] = 0;
        for (int64_t n = 0; n < N; ++n) {
            const int c = idx[n * M + m];
            cnt[c] += 1;
            for (int j = 0; j < d; ++j) sum[c * d + j] += X[n * D + m * d + j];
        }
        for (int c = 0; c < C; ++c)
            for (int j = 0; j < d; ++j) {
                const int64_t e = ((int64_t)m * C + c) * d + j;
                cb_out[e] = cnt[c] > 0 ? sum[c * d + j] / (double)cnt[c] : cb_in[e];
            }
        free(sum);
    }
}


/* ---- general forms: codes of up to 16 bits; per-sub-space or shared codebooks ----
 *
 * cb is [Mcb, C, d] with Mcb = M (sub-space m uses table m, as in the functions above) or
 * Mcb = 1 (every sub-space uses the one table: Alg. 1's C in R^{2^b x D/M}).  Indices are
 * uint16, one per sub-vector, unpacked; the packed b-bit stream the GPU library stores is
 * formed from them by the caller. */

static const double *table_of(const double *cb, int Mcb, int m, int C, int d)
{
    return cb + (Mcb == 1 ? (int64_t)0 : (int64_t)m * C * d);
}

/* Eq. 2, lowest index on ties; relgap as in vo_vq_encode. */
void vo_vq_encode_g(const double *X, int64_t N, int D, int d, int C, int Mcb, const double *cb,
                    uint16_t *idx, double *relgap)
{
    const int M = D / d;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            const double *x = X + n * D + (int64_t)m * d;
            const double *tab = table_of(cb, Mcb, m, C, d);
            double best = INFINITY, second = INFINITY;
            int arg = 0;
            for (int c = 0; c < C; ++c) {
                double dist = 0.0;
                for (int j = 0; j < d; ++j) {
                    const double t = x[j] - tab[(int64_t)c * d + j];
                    dist += t * t;
                }
                if (dist < best) {
                    second = best;
                    best = dist;
                    arg = c;
                } else if (dist < second) {
                    second = dist;
                }
            }
            idx[n * M + m] = (uint16_t)arg;
            if (relgap) relgap[n * M + m] = (second - best) / (best > 1e-300 ? best : 1e-300);
        }
    }
}

/* VQ^{-1}: Xhat[n, m*d + j] = table(m)[idx[n,m]][j]. */
void vo_vq_dequantize_g(const uint16_t *idx, int64_t N, int D, int d, int C, int Mcb,
                        const double *cb, double *Xhat)
{
    const int M = D / d;
    for (int64_t n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            const double *cen = table_of(cb, Mcb, m, C, d) + (int64_t)idx[n * M + m] * d;
            for (int j = 0; j < d; ++j) Xhat[n * D + (int64_t)m * d + j] = cen[j];
        }
}

/* Eq. 10 for one query row against one KV head; keys and values may differ in sub-vector
 * dim, number of centroids and codebook sharing (Sec. 3.2: K and V are quantized separately). */
int vo_vq_attention_g(const double *qt, const uint16_t *kidx, const uint16_t *vidx,
                      const double *cb_k, const double *cb_v, int64_t N, int D, int d_k, int C_k,
                      int Mcb_k, int d_v, int C_v, int Mcb_v, double *out, double *lse)
{
    if (N < 1) return -1;
    double *Khat = (double *)malloc(sizeof(double) * (size_t)N * D);
    double *Vhat = (double *)malloc(sizeof(double) * (size_t)N * D);
    double *s = (double *)malloc(sizeof(double) * (size_t)N);
    vo_vq_dequantize_g(kidx, N, D, d_k, C_k, Mcb_k, cb_k, Khat);
    vo_vq_dequantize_g(vidx, N, D, d_v, C_v, Mcb_v, cb_v, Vhat);
    const double scale = 1.0 / sqrt((double)D);
    double mx = -INFINITY;
    for (int64_t n = 0; n < N; ++n) {
        double acc = 0.0;
        for (int i = 0; i < D; ++i) acc += qt[i] * Khat[n * D + i];
        s[n] = acc * scale;
        if (s[n] > mx) mx = s[n];
    }
    double denom = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        s[n] = exp(s[n] - mx);
        denom += s[n];
    }
    for (int i = 0; i < D; ++i) out[i] = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        const double p = s[n] / denom;
        for (int i = 0; i < D; ++i) out[i] += p * Vhat[n * D + i];
    }
    if (lse) *lse = mx + log(denom);
    free(Khat);
    free(Vhat);
    free(s);
    return 0;
}

/* X [B, Hkv, T, D], lam [Hkv, D], cb [Hkv, Mcb, C, d] -> idx [B, Hkv, T, M] (uint16). */
int vo_encode_batch_g(const double *X, const double *lam, const double *cb, int B, int Hkv,
                      int64_t T, int D, int d, int C, int Mcb, int transform, uint16_t *idx,
                      double *relgap)
{
    if (D % d != 0 || (Mcb != 1 && Mcb != D / d) || C < 1 || C > 65536) return -1;
    const int M = D / d;
    double *H = NULL;
    if (transform) {
        H = (double *)malloc(sizeof(double) * (size_t)D * D);
        if (vo_hadamard(D, H) != 0) {
            free(H);
            return -1;
        }
    }
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g) {
            const int64_t row0 = ((int64_t)b * Hkv + g) * T;
            const double *Xbg = X + row0 * D;
            const double *cbg = cb + (int64_t)g * Mcb * C * d;
            double *gap = relgap ? relgap + row0 * M : NULL;
            if (transform) {
                double *Kt = (double *)malloc(sizeof(double) * (size_t)T * D);
                vo_transform_keys(Xbg, T, D, lam + (int64_t)g * D, H, Kt);
                vo_vq_encode_g(Kt, T, D, d, C, Mcb, cbg, idx + row0 * M, gap);
                free(Kt);
            } else {
                vo_vq_encode_g(Xbg, T, D, d, C, Mcb, cbg, idx + row0 * M, gap);
            }
        }
    free(H);
    return 0;
}

/* As vo_decode_batch (path 0), with cb_k [Hkv, Mcb_k, C_k, d_k], cb_v [Hkv, Mcb_v, C_v, d_v]
 * and uint16 indices kidx [B, Hkv, n_cap, Mk], vidx [B, Hkv, n_cap, Mv]. */
int vo_decode_batch_g(const double *q, const double *lam, const double *cb_k, const double *cb_v,
                      const uint16_t *kidx, const uint16_t *vidx, const int64_t *seq_lens, int B,
                      int Hq, int Hkv, int64_t n_cap, int D, int d_k, int C_k, int Mcb_k, int d_v,
                      int C_v, int Mcb_v, double *out, double *lse)
{
    if (Hq % Hkv != 0 || D % d_k != 0 || D % d_v != 0) return -1;
    const int G = Hq / Hkv, Mk = D / d_k, Mv = D / d_v;
    if ((Mcb_k != 1 && Mcb_k != Mk) || (Mcb_v != 1 && Mcb_v != Mv)) return -1;
    double *H = (double *)malloc(sizeof(double) * (size_t)D * D);
    if (vo_hadamard(D, H) != 0) {
        free(H);
        return -1;
    }
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            double *qt = (double *)malloc(sizeof(double) * (size_t)D);
            vo_transform_query(q + ((int64_t)b * Hq + h) * D, D, lam + (int64_t)g * D, H, qt);
            const int64_t bg = (int64_t)b * Hkv + g;
            const int rc = vo_vq_attention_g(qt, kidx + bg * n_cap * Mk, vidx + bg * n_cap * Mv,
                                             cb_k + (int64_t)g * Mcb_k * C_k * d_k,
                                             cb_v + (int64_t)g * Mcb_v * C_v * d_v, seq_lens[b], D, d_k,
                                             C_k, Mcb_k, d_v, C_v, Mcb_v, out + ((int64_t)b * Hq + h) * D,
                                             lse + ((int64_t)b * Hq + h));
            if (rc != 0) {
#pragma omp atomic write
                err = -1;
            }
            free(qt);
        }
    free(H);
    return err;
}

/* Eq. 10 with the full-precision residual window (as vo_vq_attention_residual) in the general
 * form: the N quantized tokens through (transformed query, looked-up transformed keys), the R
 * window tokens through (raw query, raw keys), one softmax over all N + R scores. */
int vo_vq_attention_residual_g(const double *qt, const double *q_raw, const uint16_t *kidx,
                               const uint16_t *vidx, const double *cb_k, const double *cb_v, int64_t N,
                               const double *kres, const double *vres, int64_t R, int D, int d_k,
                               int C_k, int Mcb_k, int d_v, int C_v, int Mcb_v, double *out, double *lse)
{
    if (N < 0 || R < 0 || N + R < 1) return -1;
    const int64_t T = N + R;
    double *Kall = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1) * D);
    double *Vall = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *s = (double *)malloc(sizeof(double) * (size_t)T);
    if (N > 0) {
        vo_vq_dequantize_g(kidx, N, D, d_k, C_k, Mcb_k, cb_k, Kall);
        vo_vq_dequantize_g(vidx, N, D, d_v, C_v, Mcb_v, cb_v, Vall);
    }
    for (int64_t r = 0; r < R; ++r)
        for (int i = 0; i < D; ++i) Vall[(N + r) * D + i] = vres[r * D + i];
    const double scale = 1.0 / sqrt((double)D);
    double mx = -INFINITY;
    for (int64_t n = 0; n < T; ++n) {
        double acc = 0.0;
        if (n < N)
            for (int i = 0; i < D; ++i) acc += qt[i] * Kall[n * D + i];
        else
            for (int i = 0; i < D; ++i) acc += q_raw[i] * kres[(n - N) * D + i];
        s[n] = acc * scale;
        if (s[n] > mx) mx = s[n];
    }
    double denom = 0.0;
    for (int64_t n = 0; n < T; ++n) {
        s[n] = exp(s[n] - mx);
        denom += s[n];
    }
    for (int i = 0; i < D; ++i) out[i] = 0.0;
    for (int64_t n = 0; n < T; ++n) {
        const double p = s[n] / denom;
        for (int i = 0; i < D; ++i) out[i] += p * Vall[n * D + i];
    }
    if (lse) *lse = mx + log(denom);
    free(Kall);
    free(Vall);
    free(s);
    return 0;
}

/* As vo_decode_residual_batch, general form. */
int vo_decode_residual_batch_g(const double *q, const double *lam, const double *cb_k, const double *cb_v,
                               const uint16_t *kidx, const uint16_t *vidx, const int64_t *seq_lens,
                               const double *kres, const double *vres, const int64_t *res_lens, int B,
                               int Hq, int Hkv, int64_t n_cap, int64_t r_cap, int D, int d_k, int C_k,
                               int Mcb_k, int d_v, int C_v, int Mcb_v, double *out, double *lse)
{
    if (Hq % Hkv != 0 || D % d_k != 0 || D % d_v != 0) return -1;
    const int G = Hq / Hkv, Mk = D / d_k, Mv = D / d_v;
    if ((Mcb_k != 1 && Mcb_k != Mk) || (Mcb_v != 1 && Mcb_v != Mv)) return -1;
    double *H = (double *)malloc(sizeof(double) * (size_t)D * D);
    if (vo_hadamard(D, H) != 0) {
        free(H);
        return -1;
    }
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const double *qr = q + ((int64_t)b * Hq + h) * D;
            double *qt = (double *)malloc(sizeof(double) * (size_t)D);
            vo_transform_query(qr, D, lam + (int64_t)g * D, H, qt);
            const int64_t bg = (int64_t)b * Hkv + g;
            const int rc = vo_vq_attention_residual_g(
                qt, qr, kidx + bg * n_cap * Mk, vidx + bg * n_cap * Mv, cb_k + (int64_t)g * Mcb_k * C_k * d_k,
                cb_v + (int64_t)g * Mcb_v * C_v * d_v, seq_lens[b], kres + bg * r_cap * D, vres + bg * r_cap * D,
                res_lens[b], D, d_k, C_k, Mcb_k, d_v, C_v, Mcb_v, out + ((int64_t)b * Hq + h) * D,
                lse + ((int64_t)b * Hq + h));
            if (rc != 0) {
#pragma omp atomic write
                err = -1;
            }
            free(qt);
        }
    free(H);
    return err;
}

/* Centroid update of one Lloyd iteration in the general form.  Mcb = M: as vo_kmeans_update, one
 * table per sub-space.  Mcb = 1: the one table shared by all sub-spaces is trained on the
 * sub-vectors of all of them pooled (Sec. 2.2: K-Means constructs the codebook C of 2^b
 * centroids of dimension d from the sub-vectors).  idx is uint16; cb_in, cb_out [Mcb, C, d];
 * counts [Mcb, C]; a centroid nobody was assigned to keeps its old value. */
void vo_kmeans_update_g(const double *X, const uint16_t *idx, int64_t N, int D, int d, int C, int Mcb,
                        const double *cb_in, double *cb_out, int64_t *counts)
{
    const int M = D / d;
    double *sum = (double *)calloc((size_t)Mcb * C * d, sizeof(double));
    for (int64_t e = 0; e < (int64_t)Mcb * C; ++e) counts[e] = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            const int64_t t = (Mcb == 1 ? 0 : (int64_t)m * C) + idx[n * M + m];
            counts[t] += 1;
            for (int j = 0; j < d; ++j) sum[t * d + j] += X[n * D + m * d + j];
        }
    for (int64_t t = 0; t < (int64_t)Mcb * C; ++t)
        for (int j = 0; j < d; ++j)
            cb_out[t * d + j] = counts[t] > 0 ? sum[t * d + j] / (double)counts[t] : cb_in[t * d + j];
    free(sum);
}
