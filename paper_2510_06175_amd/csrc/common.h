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
    const __half *cb_k;      // [Hkv, Mk, 256, dk]
    const __half *cb_v;      // [Hkv, Mv, 256, dv]
    const uint8_t *k_idx;    // [B, Hkv, n_cap, Mk]
    const uint8_t *v_idx;    // [B, Hkv, n_cap, Mv]
    const int32_t *seq_lens; // [B] or nullptr
    int B, Hq, Hkv, G, D, dk, dv, Mk, Mv;
    long long N, n_cap;
    int S;                   // number of sequence splits
    float *part_o;           // [B, Hkv, S, G, D]  unnormalised partial outputs
    float *part_m;           // [B, Hkv, S, G]     partial running max (log2 units)
    float *part_l;           // [B, Hkv, S, G]     partial sum of exp2(s2 - m)
    unsigned *counters;      // [B * Hkv]          arrivals per (b, g); zero between launches
    __half *out;             // [B, Hq, D]
    float *lse;              // [B, Hq] or nullptr
};

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
        long long v = p.seq_lens[b];
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

// Split merge (log-sum-exp over the S partials of one (b, g)), executed by the workgroup
// that arrives last.  Every workgroup calls this after its partials are written.
// Returns after the output rows of (b, g) are written by the last arrival; other
// workgroups return immediately.  `flag` is one int of LDS.
template <int BLOCK>
__device__ __forceinline__ void merge_if_last(const DecodeParams &p, int b, int g, int *flag)
{
    const int tid = threadIdx.x;
    __threadfence();                       // release: partials visible device-wide
    __syncthreads();
    if (tid == 0) {
        unsigned old = __hip_atomic_fetch_add(&p.counters[b * p.Hkv + g], 1u, __ATOMIC_ACQ_REL,
                                              __HIP_MEMORY_SCOPE_AGENT);
        *flag = (old == (unsigned)(p.S - 1));
    }
    __syncthreads();
    if (!*flag) return;
    __threadfence();                       // acquire: see the other workgroups' partials

    const int GD = p.G * p.D;
    const size_t bg = (size_t)b * p.Hkv + g;
    const float *po = p.part_o + bg * p.S * GD;
    const float *pm = p.part_m + bg * p.S * p.G;
    const float *pl = p.part_l + bg * p.S * p.G;
    for (int e = tid; e < GD; e += BLOCK) {
        const int hh = e / p.D, c = e - hh * p.D;
        float mx = -INFINITY;
        for (int s = 0; s < p.S; ++s) mx = fmaxf(mx, pm[s * p.G + hh]);
        float den = 0.f, acc = 0.f;
        if (mx > -INFINITY) {
            for (int s = 0; s < p.S; ++s) {
                const float w = exp2f(pm[s * p.G + hh] - mx);
                den += w * pl[s * p.G + hh];
                acc += w * po[(size_t)s * GD + e];
            }
        }
        const int h = g * p.G + hh;
        const size_t row = (size_t)b * p.Hq + h;
        p.out[row * p.D + c] = __float2half(den > 0.f ? acc / den : 0.f);
        if (c == 0 && p.lse) p.lse[row] = den > 0.f ? (mx + log2f(den)) * kLn2 : -INFINITY;
    }
    if (tid == 0)
        __hip_atomic_store(&p.counters[b * p.Hkv + g], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// launchers (one translation unit each)
int launch_decode_lut(const DecodeParams &p, hipStream_t stream);
int launch_decode_mfma(const DecodeParams &p, hipStream_t stream);
bool decode_mfma_supports(const DecodeParams &p);
int decode_align(const DecodeParams &p, int variant);

struct EncodeParams {
    const __half *x;      // [B, Hkv, T, D]
    const float *lam;     // [Hkv, D] or nullptr (values: no transform)
    const __half *cb;     // [Hkv, M, 256, d]
    uint8_t *idx;         // [B, Hkv, n_cap, M]
    int B, Hkv, D, d, M;
    long long T, pos0, n_cap;
};
int launch_encode(const EncodeParams &p, hipStream_t stream);

} // namespace vecinfer
