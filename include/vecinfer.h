/*
 * vecinfer.h -- C ABI of the MI355X (gfx950) fused vector-quantized decode attention.
 *
 * The library implements the hot path of VecInfer: a KV cache stored as uint8
 * codebook indices (Sec. 2.2, Eq. 2) after the key-side smooth + Hadamard
 * transform (Sec. 3.2, Eq. 3-8), and a decode step that attends to that cache
 * without ever materialising it in full precision (Sec. 3.2 Eq. 10; Sec. 3.3;
 * App. A Alg. 1).
 *
 * Conventions shared by every call
 *   - Every data pointer is a DEVICE pointer on the current HIP device, owned by
 *     the caller, valid until the work enqueued on `stream` has finished.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work; they never synchronise, allocate or free device memory.
 *   - Inputs are read-only.  Outputs are fully overwritten for the rows named.
 *   - Return value: VECINFER_OK (0) or a negative VECINFER_E* code.  Arguments are
 *     validated on the host before anything is launched; on error nothing was
 *     enqueued.  No exception crosses the boundary.
 *   - Thread-safe and stateless; decode needs a caller-provided scratch workspace.
 *
 * Notation (paper): D head dim, d sub-vector dim, M = D / d sub-spaces, b code bits
 * (2^b centroids; the "dnbm" names of Sec. 4.1 are d = n, b = m), H_q query heads,
 * H_kv KV heads, G = H_q / H_kv, query head h reads KV head h / G (consecutive grouping).
 *
 * Layouts (row-major, innermost last)
 *   keys / values      fp16  [B, H_kv, T, D]
 *   lambda             fp32  [H_kv, D]          smoothing factors, all > 0
 *   queries / output   fp16  [B, H_q, D]
 *   lse                fp32  [B, H_q]           natural-log sum of exp of the scores
 *  8-bit codes (b = 8)
 *   codebooks          fp16  [H_kv, M, 256, d]  one codebook per (KV head, sub-space)
 *   code cache         uint8 [B, H_kv, n_cap, M] one byte per (token, sub-space): the
 *                                               paper's N x M code matrix per head
 *  10- and 12-bit codes (d8b12, d4b12, d4b10, ... of Sec. 4.1; d = 4 or 8; a row must be a whole
 *  number of 32-bit words, which rules out only d = 8 with 10-bit codes at D = 64)
 *   codebooks          fp16  [H_kv, 2^b, d]     one codebook per KV head, shared by its M
 *                                               sub-spaces: the single codebook of Sec. 2.2
 *                                               and Alg. 1 (2^b x d x 2 bytes; 64 KB at d8b12,
 *                                               Sec. 4.4)
 *   code cache         uint8 [B, H_kv, n_cap, M b / 8]  a token's M codes end to end as one
 *                                               little-endian bit string: code m fills bits
 *                                               m b .. m b + b - 1 of the row, bit i of the row
 *                                               being bit i % 8 of byte i / 8 (the
 *                                               (D / d) x (b / 8) bytes per vector of Sec. 2.2)
 *  Keys and values choose d and b independently (k_*, v_* of vecinfer_cfg); the layouts above
 *  apply per side.  vecinfer_index_row_bytes / vecinfer_codebook_elems return the sizes.
 */
#ifndef VECINFER_H
#define VECINFER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VECINFER_VERSION 300          /* major*10000 + minor*100 + patch */
#define VECINFER_MAX_SPLITS 256       /* upper bound of num_splits */
#define VECINFER_MAX_APPEND 16        /* most tokens vecinfer_append_kv takes per call */
#define VECINFER_MAX_RESIDUAL 128     /* most rows of the full-precision residual window */
#define VECINFER_STATIC_SCRATCH_BYTES (4u << 20) /* workspace limit of vecinfer_decode_attention_static */
#define VECINFER_KMEANS_MAX_ITERS 30   /* most iterations of vecinfer_kmeans_train (Sec. 4.1) */
#define VECINFER_LAMBDA_FLOOR 1e-5f    /* smallest smoothing factor vecinfer_calibrate_lambda returns */

enum {
    VECINFER_OK = 0,
    VECINFER_EINVAL = -1,       /* null pointer, non-positive size, inconsistent shapes      */
    VECINFER_EUNSUPPORTED = -2, /* a shape the kernels do not cover (see vecinfer_cfg)       */
    VECINFER_EWORKSPACE = -3,   /* workspace NULL, misaligned or smaller than required       */
    VECINFER_ELAUNCH = -4       /* the HIP runtime rejected a launch or a device query       */
};

/* Decode kernel families (argument `variant` of vecinfer_decode_attention). */
enum {
    VECINFER_VARIANT_AUTO = 0,   /* fastest kernel that covers the configuration             */
    VECINFER_VARIANT_LUT = 1,    /* query-centroid lookup table in LDS, vector ALU (Alg. 1
                                    steps 4 and 11 taken literally); covers every supported
                                    configuration                                            */
    VECINFER_VARIANT_MFMA = 2    /* codebooks in LDS, dequantized tiles fed to the matrix
                                    cores for both q.K and P.V; D in {64,128}, d_k and d_v
                                    in {2,4,8}, any G the cfg allows; the only variant for 10- / 12-bit codes, which
                                    need d = 4 or 8 on BOTH sides.  Code rows are addressed
                                    with 32-bit byte offsets: N * D / 2 < 2^31 (N < 33 554 432
                                    tokens at D = 128); longer caches fall to the lookup-table
                                    variant under AUTO                                       */
    ,
    VECINFER_VARIANT_ROLES = 3   /* the matrix-core kernel with the work of a tile split between
                                    score wavefronts (q.K, online softmax) and value wavefronts
                                    (P.V), 16 wavefronts per workgroup, probabilities handed over
                                    through LDS; same arithmetic, results equal to MFMA's up to
                                    fp32 summation order.  8-bit codes, D = 128, G <= 4, d_k and
                                    d_v in {2, 4}, value codes in rows or tiles.  Never chosen by AUTO: it
                                    measures 1 - 2 us slower per call than MFMA at 196608 tokens
                                    (the tile loop is bound by LDS and issue throughput, not by
                                    latency, so more wavefronts per SIMD buy nothing); kept as
                                    the measured alternative                                 */
};

typedef struct vecinfer_cfg {
    int32_t head_dim;      /* D: 64 or 128 (Walsh-Hadamard needs a power of two, Eq. 5)      */
    int32_t num_q_heads;   /* H_q                                                            */
    int32_t num_kv_heads;  /* H_kv, divides H_q; G = H_q / H_kv in 1 .. 8                    */
    int32_t k_sub_dim;     /* d for keys: 2, 4 or 8                                          */
    int32_t v_sub_dim;     /* d for values: 2, 4 or 8 (keys and values may differ, Sec. 3.2)  */
    int32_t k_bits;        /* code width b for keys: 8 (one byte per code, 256 centroids per
                              sub-space), or 10 / 12 (packed rows, one shared codebook of 2^b
                              centroids per KV head; needs d_k = 4 or 8 and (D / d_k) b a
                              multiple of 32)                                                  */
    int32_t v_bits;        /* code width for values: 8, 10 or 12, same rules with d_v        */
    int32_t v_tiled;       /* physical layout of the value code cache (8-bit value codes only):
                              0 = rows, [B, H_kv, n_cap, M_v] as above;
                              1 = tiles of 64 tokens, see "Tiled value codes" below           */
} vecinfer_cfg;

/*
 * Tiled value codes (cfg.v_tiled = 1; v_bits = 8; M_v >= 16, i.e. not d_v = 8 at D = 64;
 * n_cap a multiple of 64).
 * The cache holds the same N x M_v code matrix of a (sequence, KV head), stored in blocks of
 * 64 tokens (64 M_v bytes each, block t / 64 of token t) in the order in which the lanes of the
 * matrix-core attention kernel consume them, so that a lane fetches its share of a block with
 * 16-byte loads instead of one narrow load per token (about 1 us per call at 196608 tokens).
 * With R = M_v / 16, i = t % 64, sub-space m and j = ((i / 16) * 4 + (i % 16) / 4) * R + m % R,
 * the byte of (t, m) sits at offset
 *     (t / 64) * 64 M_v  +  (j / 16) * 1024  +  ((i % 4) * 16 + m / R) * 16  +  j % 16
 * of the (sequence, KV head)'s cache.  vecinfer_encode_values, vecinfer_append_kv and
 * vecinfer_decode_step write this layout and the matrix-core attention reads it when the flag is
 * set; vecinfer_export_value_codes returns the rows form.  The lookup-table variant and
 * vecinfer_kmeans_step (whose `codes` output is always rows) do not take it.
 */

/*
 * Cache fill for keys: Alg. 1 "Preprocessing" + "Quantization" (Eq. 3, 6, 8):
 * for each of the T new tokens, k~ = (k / lambda) H_D, then for every sub-space m
 *   k_idx[b, g, pos0 + t, m] = argmin_c || k~[m*d .. m*d+d) - cb_k[g, m, c, :] ||^2   (Eq. 2)
 * with the squared distance summed directly in fp32 in channel order and the lowest
 * index winning ties.  k~ is not rounded to fp16 before the search.
 * T = 1 with pos0 = current length is the decode-time append of Eq. 9.
 *   k_f16   [B, H_kv, T, D] fp16      lambda [H_kv, D] fp32
 *   cb_k    [H_kv, M_k, 256, d_k]     k_idx  [B, H_kv, n_cap, M_k], rows pos0 .. pos0+T-1 written
 * With k_bits = 10 or 12 the search runs over the one shared codebook cb_k [H_kv, 2^b, d_k] and
 * the row written is the packed one, [B, H_kv, n_cap, M_k b / 8] (layouts at the top).
 * Errors: EINVAL for null pointers, B < 1, T < 1, pos0 < 0, pos0 + T > n_cap;
 * EUNSUPPORTED for a cfg outside the ranges above.
 */
int vecinfer_encode_keys(const vecinfer_cfg *cfg, const void *k_f16, const float *lambda,
                         const void *cb_k_f16, uint8_t *k_idx, int32_t B, int64_t T,
                         int64_t pos0, int64_t n_cap, void *stream);

/*
 * Cache fill for values: Eq. 8 on the untransformed values (no smoothing, no Hadamard).
 * Same argmin rule, layouts and errors as vecinfer_encode_keys, with d_v / M_v.  With
 * cfg.v_tiled = 1 each code goes to its place in the tiled layout ("Tiled value codes"; EINVAL
 * unless n_cap is a multiple of 64); bytes of other tokens of a block are left as they are.
 */
int vecinfer_encode_values(const vecinfer_cfg *cfg, const void *v_f16, const void *cb_v_f16,
                           uint8_t *v_idx, int32_t B, int64_t T, int64_t pos0,
                           int64_t n_cap, void *stream);

/*
 * Decode-time append of Eq. 9 in one launch: the same result as vecinfer_encode_keys followed
 * by vecinfer_encode_values on the T new tokens (identical codes, value codes tiled when
 * cfg.v_tiled is set), for 1 <= T <= VECINFER_MAX_APPEND.
 * Arguments and errors as for those two calls; EINVAL if T > VECINFER_MAX_APPEND.
 */
int vecinfer_append_kv(const vecinfer_cfg *cfg, const void *k_f16, const void *v_f16,
                       const float *lambda, const void *cb_k_f16, const void *cb_v_f16,
                       uint8_t *k_idx, uint8_t *v_idx, int32_t B, int64_t T, int64_t pos0,
                       int64_t n_cap, void *stream);

/*
 * Calibration of the smoothing factors, Eq. 4: per KV head g and channel i
 *   lambda[g, i] = max( sqrt( max over b, t of |k[b, g, t, i]| ), VECINFER_LAMBDA_FLOOR )
 * over the T calibration tokens of all B sequences (the paper calibrates offline on 256 samples
 * of 512 tokens, Sec. 4.1).  The floor keeps a channel that is zero in every calibration token
 * usable (every other call needs lambda > 0); Eq. 4 itself has none.
 *   k_f16  [B, H_kv, T, D] fp16 raw keys     lambda [H_kv, D] fp32 (fully overwritten)
 * Errors: EINVAL for null pointers, B < 1, T < 1; EUNSUPPORTED for a cfg outside the ranges above.
 */
int vecinfer_calibrate_lambda(const vecinfer_cfg *cfg, const void *k_f16, float *lambda, int32_t B,
                              int64_t T, void *stream);

/*
 * One Lloyd iteration of the K-Means codebook training.  The paper builds the codebooks by
 * K-Means (Sec. 2.2), on the transformed keys and on the original values (Sec. 3.2), with at most
 * 30 iterations (Sec. 4.1); initialisation, the number of iterations and the stopping rule are the
 * caller's.  Per (KV head, sub-space), over the T tokens of all B sequences:
 *   assignment  codes[b, g, t, m] = the code vecinfer_encode_keys (lambda != NULL: the vectors
 *               are smoothed and Hadamard-transformed first) or vecinfer_encode_values
 *               (lambda == NULL) would write with cb_in
 *   update      cb_out[g, m, c, :] = fp16(mean of the sub-vectors assigned to c), summed in fp32;
 *               a centroid nobody was assigned to keeps its cb_in value
 * The sums are formed with fp32 atomics, so their last bits (and rarely the fp16
 * rounding of a centroid) may differ between runs.
 *   x_f16  [B, H_kv, T, D] fp16       cb_in_f16, cb_out_f16 [H_kv, M, 256, d] (may not alias)
 *   codes  [B, H_kv, T, M] uint8 (written)    counts int32 [H_kv, M, 256] or NULL: cluster sizes
 *   workspace  vecinfer_kmeans_workspace_bytes(cfg, lambda != NULL) bytes, 256-byte aligned
 * d and M are the key values of cfg when lambda is given, else the value ones.
 * With 10- or 12-bit codes on that side the one codebook of a KV head, [H_kv, 2^b, d], is trained on
 * the sub-vectors of all its sub-spaces pooled (Sec. 2.2); codes are the packed rows
 * [B, H_kv, T, M b / 8] and counts is [H_kv, 2^b].
 * Errors: as vecinfer_encode_keys / _values, plus EWORKSPACE.
 */
size_t vecinfer_kmeans_workspace_bytes(const vecinfer_cfg *cfg, int32_t keys);
int vecinfer_kmeans_step(const vecinfer_cfg *cfg, const void *x_f16, const float *lambda,
                         const void *cb_in_f16, void *cb_out_f16, uint8_t *codes, int32_t *counts,
                         int32_t B, int64_t T, void *workspace, size_t workspace_bytes, void *stream);

/*
 * K-Means codebook training: Lloyd's algorithm, at most max_iters <= VECINFER_KMEANS_MAX_ITERS = 30
 * iterations (Sec. 2.2: the codebook is built by K-Means; Sec. 3.2: on the transformed keys and the
 * original values; Sec. 4.1: maximum number of iterations 30), with the quantization error
 * computed on the device and a stopping rule there.  Any supported code width: with 10- or 12-bit
 * codes the KV head's one shared codebook is trained on the sub-vectors of all its sub-spaces, as
 * for vecinfer_kmeans_step.
 * Iteration t = 0, 1, ..:
 *   assignment  as vecinfer_kmeans_step, with the centroids cb_t (cb_0 = what cb_f16 holds on entry)
 *   error       E_t = sum over all KV heads, sub-spaces and tokens of |x - cb_t[code]|^2 (fp32 per
 *               sub-vector, summed in fp64): the quantization error of that assignment
 *   update      cb_{t+1} = fp16(cluster means), in place in cb_f16; empty clusters keep their centroid
 *   stop        after the update of iteration t when t = max_iters - 1, or when t >= 1 and
 *               E_{t-1} - E_t <= tol * E_{t-1}  (tol < 0: never before max_iters)
 * All max_iters iterations are enqueued; those after the stop return at once (a flag in the
 * workspace), so the call never synchronises.  Initial centroids are the caller's (e.g. a sample
 * of the training vectors).
 *   cb_f16     [H_kv, M, 256, d] fp16 (10- / 12-bit codes: [H_kv, 2^b, d]), read and overwritten
 *   codes      [B, H_kv, T, row bytes] uint8 (rows as vecinfer_encode_* writes them): the assignment
 *              of the last iteration run
 *   counts     int32, one per centroid ([H_kv, M, 256] or [H_kv, 2^b]), or NULL: its cluster sizes
 *   iters_run  int32 on the device or NULL: iterations run
 *   errors     fp64 [max_iters] on the device or NULL: E_0 .. E_{iters_run - 1}; the rest untouched
 *   workspace  vecinfer_kmeans_workspace_bytes(cfg, lambda != NULL) bytes, 256-byte aligned
 * The cluster sums are formed with fp32 atomics (in LDS, then one per workgroup and centroid in
 * memory), so their last bits, and rarely the fp16 rounding of a centroid, may differ between runs.
 * Errors: as vecinfer_kmeans_step; EINVAL for max_iters outside 1 .. 30 or tol = NaN.
 */
int vecinfer_kmeans_train(const vecinfer_cfg *cfg, const void *x_f16, const float *lambda, void *cb_f16,
                          uint8_t *codes, int32_t *counts, int32_t B, int64_t T, int32_t max_iters,
                          float tol, int32_t *iters_run, double *errors, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Number of sequence splits the library would pick for (B, N) when num_splits = 0
 * (grid axis "num_splits" of Sec. 3.3).  Host-only; returns >= 1, or a negative code.
 */
int32_t vecinfer_decode_auto_splits(const vecinfer_cfg *cfg, int32_t B, int64_t N);

/*
 * Bytes of workspace vecinfer_decode_attention needs for batch B, up to N tokens and
 * `num_splits` splits (0 = whatever vecinfer_decode_auto_splits returns for (B, N)).
 * N = 0 (only meaningful for vecinfer_decode_attention_residual) gives the one-split size.
 * Host-only.  Returns 0 for an invalid cfg or negative sizes.
 */
size_t vecinfer_decode_workspace_bytes(const vecinfer_cfg *cfg, int32_t B, int64_t N,
                                       int32_t num_splits);

/*
 * One decode step of VQ attention (Eq. 10 via Alg. 1 steps 4-23) for a batch:
 *   q~ = (q * lambda[g]) H_D                                   (Eq. 3, 6, 7)
 *   s_n = q~ . concat_m cb_k[g, m, k_idx[b, g, n, m], :] / sqrt(D)
 *   p = softmax(s) over n < len_b;  o = sum_n p_n concat_m cb_v[g, m, v_idx[b, g, n, m], :]
 *   L = log sum_n exp(s_n)                                      (Alg. 1 step 22)
 * computed per (b, q head h), g = h / G, fp32 accumulation, fp16 output.  The sequence
 * is cut into `num_splits` chunks handled by different workgroups; their (o, m, l)
 * partials go through `workspace` and are merged by log-sum-exp by a second small kernel
 * enqueued right behind (with one split the attention kernel finalises by itself).
 * The result does not depend on num_splits beyond fp32 rounding, and not at all on the layout
 * of the value codes (cfg.v_tiled: v_idx is then read as tiles; n_cap a multiple of 64, else EINVAL).
 *   seq_lens  int32 [B] on the device, or NULL: every sequence has N tokens.  Values are
 *             clamped to [0, N]; a sequence of length 0 yields o = 0 and L = -inf.
 *   N         tokens attended (upper bound when seq_lens is given), 1 <= N <= n_cap
 *   num_splits 0 = auto, else 1 .. VECINFER_MAX_SPLITS
 *   variant   VECINFER_VARIANT_*
 *   workspace at least vecinfer_decode_workspace_bytes(cfg, B, N, num_splits) bytes,
 *             256-byte aligned; contents need no initialisation and are overwritten;
 *             calls that share a workspace must be ordered on one stream
 *   out_f16   [B, H_q, D] fp16          lse  [B, H_q] fp32 or NULL
 * Errors: EINVAL (null pointers, B < 1, N < 1, N > n_cap, num_splits out of range),
 * EUNSUPPORTED (cfg, variant that does not cover cfg, B or H_kv above 65535), EWORKSPACE, ELAUNCH.
 */
int vecinfer_decode_attention(const vecinfer_cfg *cfg, const void *q_f16, const float *lambda,
                              const void *cb_k_f16, const void *cb_v_f16,
                              const uint8_t *k_idx, const uint8_t *v_idx,
                              const int32_t *seq_lens, int32_t B, int64_t N, int64_t n_cap,
                              int32_t num_splits, int32_t variant, void *workspace,
                              size_t workspace_bytes, void *out_f16, float *lse, void *stream);

/*
 * vecinfer_decode_attention for callers that cannot allocate device memory or hand over a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (minus the workspace), same kernels, same results bit for bit.
 * The split partials go to a fixed array of VECINFER_STATIC_SCRATCH_BYTES (4 MiB) inside the
 * library's device code; every GPU the library runs on holds its own copy until the process ends.
 * The call allocates and frees nothing, on the device or through any library; the first call
 * on a device looks the array's address up once (make that first call outside a capture).
 *   - A request whose workspace (vecinfer_decode_workspace_bytes for the same cfg, B, N,
 *     num_splits) exceeds VECINFER_STATIC_SCRATCH_BYTES returns EWORKSPACE; nothing is enqueued.
 *     (Llama-3.1-8B shapes: B = 1 with 32 splits needs 0.55 MiB; B x H_q x splits x (D + 2)
 *     floats in general.)
 *   - All calls on one GPU share that GPU's array.  It needs no clearing (every partial a merge
 *     reads was written by the attention kernel of the same call), but calls that overlap on one
 *     GPU - different streams without ordering, or different host threads - race on it: order them.
 * Errors: as vecinfer_decode_attention, EWORKSPACE as above, ELAUNCH if the device query or the
 * address lookup fails.
 */
int vecinfer_decode_attention_static(const vecinfer_cfg *cfg, const void *q_f16, const float *lambda,
                                     const void *cb_k_f16, const void *cb_v_f16,
                                     const uint8_t *k_idx, const uint8_t *v_idx,
                                     const int32_t *seq_lens, int32_t B, int64_t N, int64_t n_cap,
                                     int32_t num_splits, int32_t variant, void *out_f16, float *lse,
                                     void *stream);

/*
 * Decode step with a full-precision residual window.  The paper's runs keep the most recent
 * tokens (residual length 128, Sec. 4.1) unquantized; this call attends to the N quantized
 * tokens exactly as vecinfer_decode_attention does and, in the same softmax, to the window:
 *   s_r = q . k_res[b, g, r, :] / sqrt(D)     raw query against raw key, which equals the
 *                                             transformed product q~ . k~ by Eq. 7
 *   p = softmax over the len_b + res_len_b scores;   o += sum_r p_r v_res[b, g, r, :]
 * The window is scored by the merge kernel and joins the log-sum-exp merge as one more partial.
 * Filling the window and flushing it into the code cache (vecinfer_encode_keys / _values with
 * T = window length, pos0 = N, reading the window as [B, H_kv, T, D] when r_cap = T) is the caller's.
 *   k_res_f16, v_res_f16  fp16 [B, H_kv, r_cap, D], rows 0 .. res_len_b - 1 are attended
 *   res_lens  int32 [B] on the device, or NULL: every window holds R rows; clamped to [0, R]
 *   R         window rows attended, 0 <= R <= min(r_cap, VECINFER_MAX_RESIDUAL)
 *   N         may be 0 when R >= 1 (nothing quantized yet); k_idx / v_idx may then be NULL
 * A sequence with no token in either part yields o = 0 and L = -inf.  Everything else, and the
 * workspace size, as for vecinfer_decode_attention.
 * Errors: as vecinfer_decode_attention, plus EINVAL for a NULL window, R < 0, R > r_cap,
 * N + R < 1, and EUNSUPPORTED for R > VECINFER_MAX_RESIDUAL.
 */
int vecinfer_decode_attention_residual(const vecinfer_cfg *cfg, const void *q_f16, const float *lambda,
                                       const void *cb_k_f16, const void *cb_v_f16,
                                       const uint8_t *k_idx, const uint8_t *v_idx,
                                       const int32_t *seq_lens, int32_t B, int64_t N, int64_t n_cap,
                                       const void *k_res_f16, const void *v_res_f16,
                                       const int32_t *res_lens, int32_t R, int64_t r_cap,
                                       int32_t num_splits, int32_t variant, void *workspace,
                                       size_t workspace_bytes, void *out_f16, float *lse, void *stream);

/*
 * One whole decode step of a layer: the append of Eq. 9 and the attention of Eq. 10 in one call.
 * The new token of sequence b (key k_new[b, g, 0, :], value v_new[b, g, 0, :]) becomes its last
 * token, position len_b - 1 (len_b = seq_lens[b] clamped to [0, N], or N without seq_lens, so
 * len_b counts the new token); rows len_b - 1 of k_idx and v_idx receive exactly the codes
 * vecinfer_append_kv would write there, and the output is what vecinfer_decode_attention
 * returns afterwards for the same N and seq_lens.  A sequence with len_b = 0 appends nothing
 * and yields o = 0, L = -inf.
 * With VECINFER_VARIANT_MFMA (or AUTO when it covers cfg) nothing is launched in front of the
 * attention: its workgroups share out the sub-spaces of the new token while the code cache of
 * the older tokens streams, and the merge kernel joins the new token as one more partial.
 * The lookup-table variant runs the append kernel first.
 *   k_new_f16, v_new_f16  fp16 [B, H_kv, 1, D]
 *   k_idx, v_idx          as in vecinfer_decode_attention, but written at row len_b - 1 (with
 *                         cfg.v_tiled the value codes of that token go to their tiled places)
 * Everything else, the workspace size and the errors as for vecinfer_decode_attention
 * (EINVAL also for NULL k_new_f16 / v_new_f16).
 */
int vecinfer_decode_step(const vecinfer_cfg *cfg, const void *q_f16, const void *k_new_f16,
                         const void *v_new_f16, const float *lambda, const void *cb_k_f16,
                         const void *cb_v_f16, uint8_t *k_idx, uint8_t *v_idx, const int32_t *seq_lens,
                         int32_t B, int64_t N, int64_t n_cap, int32_t num_splits, int32_t variant,
                         void *workspace, size_t workspace_bytes, void *out_f16, float *lse, void *stream);

/*
 * Sizes that follow from cfg (host-only; 0 for an invalid cfg).  keys != 0: the key side.
 *   vecinfer_index_row_bytes  bytes of one token's code row, M b / 8 (Sec. 2.2): the innermost
 *                             extent of k_idx / v_idx
 *   vecinfer_codebook_elems   fp16 elements of the whole codebook tensor cb_k / cb_v:
 *                             H_kv M 256 d at 8 bits, H_kv 2^b d above
 */
size_t vecinfer_index_row_bytes(const vecinfer_cfg *cfg, int32_t keys);
size_t vecinfer_codebook_elems(const vecinfer_cfg *cfg, int32_t keys);

/*
 * Tiled value codes -> rows: writes the N x M_v code matrix of every (sequence, KV head) of a cache
 * kept in the tiled layout (cfg.v_tiled, see "Tiled value codes") as rows, [B, H_kv, n_cap, M_v],
 * rows 0 .. N-1.  For callers that inspect or move a cache (and for the parity tests); the attention
 * path never needs it.  The flag in cfg is not consulted: the source is taken to be tiled.
 *   v_idx_tiled  [B, H_kv, n_cap * M_v] bytes, tiled     v_idx_rows  [B, H_kv, n_cap, M_v], another buffer
 * Errors: EINVAL (null or identical pointers, B < 1, N < 1, N > n_cap, n_cap not a multiple of 64),
 * EUNSUPPORTED (cfg; v_bits other than 8).
 */
int vecinfer_export_value_codes(const vecinfer_cfg *cfg, const uint8_t *v_idx_tiled, uint8_t *v_idx_rows,
                                int32_t B, int64_t N, int64_t n_cap, void *stream);

/*
 * Measurement aid: a plain streaming read of `bytes` bytes at `src` (16-byte loads from every CU,
 * nothing else), i.e. the read rate HBM delivers on this device to a kernel with no other work.
 * Benchmarks print it beside the attention kernel's rate (the roofline's measured counterpart of
 * the published peak).  The result of the reads is discarded; `sink` (device, 4 bytes) is written
 * at most in the unlikely case of one particular checksum.
 * Errors: EINVAL for null or misaligned pointers (src 16, sink 4 bytes) or bytes < 16.
 */
int vecinfer_read_probe(const void *src, size_t bytes, uint32_t *sink, void *stream);

/* Human-readable text for a return code (static storage). */
const char *vecinfer_strerror(int code);

/* VECINFER_VERSION of the built library. */
int vecinfer_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VECINFER_H */
