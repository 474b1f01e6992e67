// Shared device-side definitions of the gfx950 VQ decode-attention kernels.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vecinfer {

constexpr int kCentroids = 256;                    // 8-bit codes (Sec. 2.2)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Arguments of one decode step.  Scores are kept in log2 units throughout the
// kernels: s2 = s * log2(e), so that p = exp2(s2 - m2); the natural-log L of
// Alg. 1 step 22 is (m2 + log2 l) * ln 2.
struct DecodeParams {
    const __half *q;         // [B, Hq, D]
    const float *lam;        // [Hkv, D]
    const __half *cb_k;      // [Hkv, Mk, 256, dk]; codes wider than 8 bits: [Hkv, 2^bk, dk]
    const __half *cb_v;      // [Hkv, Mv, 256, dv]; codes wider than 8 bits: [Hkv, 2^bv, dv]
    const uint8_t *k_idx;    // [B, Hkv, n_cap, Mk * bk / 8]: a token's codes end to end, bk bits each
    const uint8_t *v_idx;    // [B, Hkv, n_cap, Mv * bv / 8]
    const int32_t *seq_lens; // [B] or nullptr
    int B, Hq, Hkv, G, D, dk, dv, Mk, Mv;
    int bk, bv;              // code widths: 8, 10 or 12 bits
    int v_tiled;             // value codes stored in tiles of 64 tokens (v_tiled_offset), 8-bit codes only
    long long N, n_cap;
    int S;                   // number of sequence splits
    float *part_o;           // [B, Hkv, S, G, D]  unnormalised partial outputs
    float *part_m;           // [B, Hkv, S, G]     partial running max (log2 units)
    float *part_l;           // [B, Hkv, S, G]     partial sum of exp2(s2 - m)
    __half *out;             // [B, Hq, D]
    float *lse;              // [B, Hq] or nullptr
    // full-precision residual window (Sec. 4.1, residual length); k_res == nullptr: none
    const __half *k_res;     // [B, Hkv, r_cap, D] raw keys of the most recent tokens
    const __half *v_res;     // [B, Hkv, r_cap, D] raw values
    const int32_t *res_lens; // [B] or nullptr
    int R;                   // window rows attended (upper bound when res_lens is given)
    long long r_cap;
    // fused append of the step's new token (Eq. 9 inside the decode step); k_new == nullptr: none.
    // The new token is the last one of each sequence (position len_b - 1): the attention kernel
    // reads codes of the len_b - 1 older tokens only, its workgroups share out the sub-spaces of
    // the new token (nearest centroid, code byte, score share, dequantized value) and the merge
    // kernel joins the new token as one more partial.
    const __half *k_new;     // [B, Hkv, 1, D] raw key of the new token
    const __half *v_new;     // [B, Hkv, 1, D] raw value
    uint8_t *k_idx_w;        // = k_idx, writable: row len_b - 1 receives the key codes
    uint8_t *v_idx_w;        // = v_idx, writable
    float *new_sc;           // [B, Hkv, Mk, G] score share of each key sub-space (log2 units)
    float *new_v;            // [B, Hkv, D]     dequantized value of the new token
};

// Tiled value codes: byte offset of (token n, sub-space m) in the cache of one (sequence, KV head).
// Blocks of 64 tokens.  Lane (k-group kg, column col) of the matrix-core kernel consumes, of a
// block, 16 R bytes (R = M / 16): for sub-tile st and token 4 v + kg of it, the bytes of sub-spaces
// R col .. R col + R - 1, in the order j = (st, v, r).  The block is stored as R slabs of 1 KB: slab
// j / 16 holds bytes j % 16 .. of every lane, lane after lane, so that one 16-byte load per lane
// reads a whole slab (8 full cache lines).
__host__ __device__ __forceinline__ size_t v_tiled_offset(long long n, int m, int M)
{
    const int R = M / 16, i = (int)(n & 63);
    const int st = i >> 4, v = (i & 15) >> 2, kg = i & 3, col = m / R, r = m % R;
    const int j = (st * 4 + v) * R + r;
    return (size_t)(n >> 6) * 64 * M + (size_t)(j >> 4) * 1024 + (kg * 16 + col) * 16 + (j & 15);
}

// Token range [n0, n1) of split s for a sequence of `len` tokens: equal chunks rounded
// up to a multiple of `align` tokens; trailing splits may be empty.
__device__ __forceinline__ void split_range(long long len, int S, int s, int align,
                                            long long &n0, long long &n1)
{
    long long chunk = (len + S - 1) / S;
    chunk = (chunk + align - 1) / align * align;
    n0 = (long long)s * chunk;
    n1 = n0 + chunk;
    if (n0 > len) n0 = len;
    if (n1 > len) n1 = len;
}

__device__ __forceinline__ long long seq_len_of(const DecodeParams &p, int b)
{
    long long len = p.N;
    if (p.seq_lens) {
        // b is the same for the whole workgroup: read through the constant address space, i.e. by a
        // scalar load, which does not queue behind the wavefront's vector loads
        typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
        long long v = ((const_i32_ptr)(uintptr_t)p.seq_lens)[b];
        len = v < 0 ? 0 : (v > p.N ? p.N : v);
    }
    return len;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Log-sum-exp merge of the S partials of one (b, g) into the final output rows (the paper
// returns L from each tile loop, Alg. 1 step 22, but leaves the merge to the reader):
//   M = max_s m_s,  w_s = 2^(m_s - M),  o = sum_s w_s o_s / sum_s w_s l_s,  L = (M + log2 sum) ln 2.
// reduce_partials folds the S workspace partials of output element e = hh * D + c into the
// running (mx, den, acc).  Partials are read in batches of independent loads so that the
// S-long reduction costs a few memory latencies, not S of them.
__device__ __forceinline__ void reduce_partials(const DecodeParams &p, int b, int g, int e, float &mx,
                                                float &den, float &acc)
{
    constexpr int kBatch = 32;
    const int GD = p.G * p.D;
    const size_t bg = (size_t)b * p.Hkv + g;
    const float *po = p.part_o + bg * p.S * GD;
    const float *pm = p.part_m + bg * p.S * p.G;
    const float *pl = p.part_l + bg * p.S * p.G;
    const int hh = e / p.D;
    for (int s0 = 0; s0 < p.S; s0 += kBatch) {
        float vm[kBatch], vl[kBatch], vo[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int s = s0 + i < p.S ? s0 + i : p.S - 1;
            vm[i] = pm[s * p.G + hh];
            vl[i] = pl[s * p.G + hh];
            vo[i] = po[(size_t)s * GD + e];
        }
        float bmx = mx;
#pragma unroll
        for (int i = 0; i < kBatch; ++i)
            if (s0 + i < p.S) bmx = fmaxf(bmx, vm[i]);
        if (bmx > -INFINITY) {
            const float rescale = exp2f(mx - bmx);        // 0 when nothing was accumulated yet
            den *= rescale;
            acc *= rescale;
#pragma unroll
            for (int i = 0; i < kBatch; ++i)
                if (s0 + i < p.S) {
                    const float w = exp2f(vm[i] - bmx);
                    den += w * vl[i];
                    acc += w * vo[i];
                }
            mx = bmx;
        }
    }
}

// Normalises the merged (mx, den, acc) of output element e and writes out (and lse once per row).
__device__ __forceinline__ void store_merged(const DecodeParams &p, int b, int g, int e, float mx, float den,
                                             float acc)
{
    const int hh = e / p.D, c = e - hh * p.D;
    const size_t row = (size_t)b * p.Hq + g * p.G + hh;
    p.out[row * p.D + c] = __float2half(den > 0.f ? acc / den : 0.f);
    if (c == 0 && p.lse) p.lse[row] = den > 0.f ? (mx + log2f(den)) * kLn2 : -INFINITY;
}

// Called by all BLOCK threads of one workgroup.
template <int BLOCK>
__device__ __forceinline__ void merge_splits(const DecodeParams &p, int b, int g)
{
    for (int e = threadIdx.x; e < p.G * p.D; e += BLOCK) {
        float mx = -INFINITY, den = 0.f, acc = 0.f;
        reduce_partials(p, b, g, e, mx, den, acc);
        store_merged(p, b, g, e, mx, den, acc);
    }
}

// End of a decode workgroup.  With a single split and no residual window the workgroup's own
// partial is the whole answer and it finalises the output rows itself; otherwise a merge kernel follows
// in the same stream (a device-scope release inside the kernel would write the whole L2 of the
// XCD back per workgroup, which costs more than the kernel boundary does).
template <int BLOCK>
__device__ __forceinline__ void finish_split(const DecodeParams &p, int b, int g)
{
    if (p.S > 1 || p.k_res) return;
    __syncthreads();                       // this workgroup's partial stores, visible to itself
    merge_splits<BLOCK>(p, b, g);
}

constexpr int kMaxResidual = 128;                  // rows of the residual window (the paper's setting)

int num_cus();   // compute units of the chip (queried once per process; sizes grids only)

// launchers (one translation unit each)
int launch_merge(const DecodeParams &p, hipStream_t stream);   // splits (+ residual window) -> out, lse
int launch_decode_lut(const DecodeParams &p, hipStream_t stream);
int launch_decode_mfma(const DecodeParams &p, hipStream_t stream);
int launch_decode_mfma_wide128(const DecodeParams &p, hipStream_t stream);   // 10- / 12-bit codes, D = 128
int launch_decode_mfma_wide64(const DecodeParams &p, hipStream_t stream);    // 10- / 12-bit codes, D = 64
int launch_decode_mfma_tiled(const DecodeParams &p, hipStream_t stream);  // 8-bit codes, tiled value codes
bool decode_mfma_supports(const DecodeParams &p);
bool decode_roles_supports(const DecodeParams &p);                        // score / value wavefront kernel
int launch_decode_roles(const DecodeParams &p, hipStream_t stream);

struct EncodeParams {
    const __half *x;      // [B, Hkv, T, D]
    const float *lam;     // [Hkv, D] or nullptr (values: no transform)
    const __half *cb;     // [Hkv, M, 256, d]; bits > 8: [Hkv, 2^bits, d], shared by the sub-spaces
    uint8_t *idx;         // [B, Hkv, n_cap, M * bits / 8]
    int B, Hkv, D, d, M;
    int bits;             // code width: 8, 10 or 12
    int tiled;            // 8-bit value codes written in tiles of 64 tokens (v_tiled_offset)
    long long T, pos0, n_cap;
    // per-sequence append position (T = 1 only): when seq_lens != nullptr the token of sequence b
    // goes to row clamp(seq_lens[b], 0, len_max) - 1, and a sequence of length 0 is skipped
    const int32_t *seq_lens;
    long long len_max;
    // K-Means training: when km_sums != nullptr the wide tiled kernel also adds every (transformed)
    // sub-vector into the sum of the centroid it was assigned to and its squared distance to the
    // iteration's error in km_state (8-bit codes: launch_kmeans_assign)
    float *km_sums;       // [Hkv, M, 256, d] fp32 (wide codes: [Hkv, 2^b, d]), cleared by launch_kmeans_begin
    int32_t *km_counts;   // [Hkv, M, 256]         (wide codes: [Hkv, 2^b])
    void *km_state;       // kmeans_state_bytes() of device memory
    int km_iter;          // iteration the launch belongs to (a launch behind the stop does nothing)
};
// K-Means training iteration: begin (clear), assign + accumulate (8-bit codes: launch_kmeans_assign; wide
// codes: launch_encode with km_sums set), end (update in place, error, stopping rule); `state` is
// kmeans_state_bytes() of device memory
size_t kmeans_state_bytes();
int launch_kmeans_begin(float *sums, int32_t *counts, size_t n_sums, size_t n_counts, int iter, void *state,
                        hipStream_t stream);
int launch_kmeans_assign(const EncodeParams &p, int iter, void *state, hipStream_t stream);
int launch_kmeans_end(const float *sums, const int32_t *counts, __half *cb, int32_t *counts_out, size_t n_centroids,
                      int d, int iter, float tol, void *state, int32_t *iters_run, double *errors, hipStream_t stream);
int launch_encode(const EncodeParams &p, hipStream_t stream);
int launch_export_value_codes(const uint8_t *tiled, uint8_t *rows, int BH, int M, long long N, long long n_cap,
                              hipStream_t stream);
int launch_read_probe(const void *src, size_t bytes, unsigned *sink, int num_cus, hipStream_t stream);
int launch_calibrate_lambda(const __half *k, float *lam, int B, int Hkv, int D, long long T, float floor_value,
                            hipStream_t stream);
int launch_append(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream);
int append_max_tokens();

} // namespace vecinfer
