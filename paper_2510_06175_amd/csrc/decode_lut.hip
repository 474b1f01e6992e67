// Lookup-table decode attention on the vector ALU (Alg. 1 steps 4-23 taken literally).
//
// One workgroup per (split, KV head, batch).  For each of the G query heads of the
// group in turn: transform the query (Eq. 3, 6), build lut = q~' C_k^T in LDS with the
// 1/sqrt(D) * log2(e) factor folded in (Alg. 1 step 4), then walk the split's tokens in
// tiles of BLOCK: one thread per token sums its M_k table entries (step 11), the block
// reduces max and sum (steps 12-13), and the P.V update (step 16) runs with one thread
// per output channel gathering value centroids from the LDS copy of C_v.
//
// This kernel covers every supported configuration (D 64/128, d 2/4/8, G 1..8) and is
// the plain-LUT baseline the matrix-core kernel is measured against.
#include "common.h"

namespace vecinfer {

namespace {

constexpr int kBlock = 256;

struct LutSmem {
    float *lut;     // [Mk * 256]
    __half *cv;     // [Mv * 256 * dv] = 256 * D halves
    float *qt;      // [D]
    float *ptile;   // [kBlock]
    float *red;     // [2 * kBlock / 64]
    float *osum;    // [kBlock]  cross-slice reduction of the output
};

__device__ __forceinline__ LutSmem carve(unsigned char *base, int Mk, int D)
{
    LutSmem s;
    s.lut = reinterpret_cast<float *>(base);
    base += sizeof(float) * Mk * kCentroids;
    s.cv = reinterpret_cast<__half *>(base);
    base += sizeof(__half) * kCentroids * D;
    s.qt = reinterpret_cast<float *>(base);
    base += sizeof(float) * D;
    s.ptile = reinterpret_cast<float *>(base);
    base += sizeof(float) * kBlock;
    s.red = reinterpret_cast<float *>(base);
    base += sizeof(float) * 2 * (kBlock / 64);
    s.osum = reinterpret_cast<float *>(base);
    base += sizeof(float) * kBlock;
    return s;
}

size_t lut_smem_bytes(int Mk, int D)
{
    return sizeof(float) * Mk * kCentroids + sizeof(__half) * kCentroids * D + sizeof(float) * D +
           sizeof(float) * kBlock + sizeof(float) * 2 * (kBlock / 64) + sizeof(float) * kBlock + 16;
}

__global__ __launch_bounds__(kBlock) void decode_lut_kernel(DecodeParams p)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const LutSmem sm = carve(smem_raw, p.Mk, p.D);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int s = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int D = p.D, Mk = p.Mk, Mv = p.Mv, dk = p.dk, dv = p.dv;

    long long n0, n1;
    split_range(seq_len_of(p, b), p.S, s, kBlock, n0, n1);

    const size_t bg = (size_t)b * p.Hkv + g;
    const uint8_t *krow = p.k_idx + bg * p.n_cap * Mk;
    const uint8_t *vrow = p.v_idx + bg * p.n_cap * Mv;

    // value codebook of this KV head -> LDS (Alg. 1 step 7)
    {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(p.cb_v + (size_t)g * kCentroids * D);
        uint32_t *dst = reinterpret_cast<uint32_t *>(sm.cv);
        for (int e = tid; e < kCentroids * D / 2; e += kBlock) dst[e] = src[e];
    }

    const float fold = kLog2e / sqrtf((float)D);
    const float hscale = 1.0f / sqrtf((float)D);
    const int c_out = tid % D;            // output channel of this thread in the P.V phase
    const int slice = tid / D;            // token slice of this thread in the P.V phase
    const int nslice = kBlock / D;
    const int mv_out = c_out / dv, jv_out = c_out - mv_out * dv;

    for (int hh = 0; hh < p.G; ++hh) {
        const int h = g * p.G + hh;
        __syncthreads();                  // previous head is done with qt / lut
        // ---- query side of the dual transform: q~ = (q * lambda) H_D
        if (tid < D) sm.qt[tid] = __half2float(p.q[((size_t)b * p.Hq + h) * D + tid]) * p.lam[(size_t)g * D + tid];
        __syncthreads();
        for (int st = 1; st < D; st <<= 1) {
            float mine = 0.f, other = 0.f;
            if (tid < D) {
                mine = sm.qt[tid];
                other = sm.qt[tid ^ st];
            }
            __syncthreads();
            if (tid < D) sm.qt[tid] = (tid & st) ? (other - mine) : (mine + other);
            __syncthreads();
        }
        // ---- lut[m][c] = q~_m . C_k[m][c], scaled so that sums are scores in log2 units
        {
            const __half *cb = p.cb_k + (size_t)g * Mk * kCentroids * dk;
            for (int e = tid; e < Mk * kCentroids; e += kBlock) {
                const int m = e >> 8;
                float acc = 0.f;
                for (int j = 0; j < dk; ++j) acc += sm.qt[m * dk + j] * __half2float(cb[(size_t)e * dk + j]);
                sm.lut[e] = acc * (hscale * fold);
            }
        }
        __syncthreads();

        float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
        for (long long t0 = n0; t0 < n1; t0 += kBlock) {
            const long long n = t0 + tid;
            const int nb = (int)((n1 - t0 < kBlock) ? (n1 - t0) : kBlock);
            // ---- score by table lookup (Alg. 1 step 11)
            float sc = -INFINITY;
            if (n < n1) {
                const uint32_t *codes = reinterpret_cast<const uint32_t *>(krow + (size_t)n * Mk);
                float a = 0.f;
                for (int w = 0; w < Mk / 4; ++w) {
                    const uint32_t cw = codes[w];
                    a += sm.lut[(4 * w + 0) * kCentroids + (cw & 255u)];
                    a += sm.lut[(4 * w + 1) * kCentroids + ((cw >> 8) & 255u)];
                    a += sm.lut[(4 * w + 2) * kCentroids + ((cw >> 16) & 255u)];
                    a += sm.lut[(4 * w + 3) * kCentroids + (cw >> 24)];
                }
                sc = a;
            }
            // ---- online softmax (steps 12-13)
            float tmax = wave_max(sc);
            if (lane == 0) sm.red[wave] = tmax;
            __syncthreads();
            float m_new = m_run;
            for (int w = 0; w < kBlock / 64; ++w) m_new = fmaxf(m_new, sm.red[w]);
            const float pr = (n < n1) ? exp2f(sc - m_new) : 0.f;
            sm.ptile[tid] = pr;
            const float tsum = wave_sum(pr);
            if (lane == 0) sm.red[kBlock / 64 + wave] = tsum;
            __syncthreads();
            const float alpha = exp2f(m_run - m_new);   // 0 on the first tile
            float rowsum = 0.f;
            for (int w = 0; w < kBlock / 64; ++w) rowsum += sm.red[kBlock / 64 + w];
            l_run = alpha * l_run + rowsum;
            m_run = m_new;
            // ---- o = alpha * o + p . VQ^-1(V_q)  (step 16)
            acc *= alpha;
            for (int r = slice; r < nb; r += nslice) {
                const unsigned code = vrow[(size_t)(t0 + r) * Mv + mv_out];
                acc += sm.ptile[r] * __half2float(sm.cv[(mv_out * kCentroids + code) * dv + jv_out]);
            }
            __syncthreads();              // ptile / red are rewritten by the next tile
        }
        // ---- cross-slice sum, then the partial (o, m, l) of this split
        sm.osum[tid] = acc;
        __syncthreads();
        if (tid < D) {
            float o = 0.f;
            for (int sl = 0; sl < nslice; ++sl) o += sm.osum[sl * D + tid];
            const size_t pi = (bg * p.S + s) * p.G + hh;
            p.part_o[pi * D + tid] = o;
            if (tid == 0) {
                p.part_m[pi] = m_run;
                p.part_l[pi] = l_run;
            }
        }
    }
    finish_split<kBlock>(p, b, g);
}

} // namespace

int launch_decode_lut(const DecodeParams &p, hipStream_t stream)
{
    const size_t smem = lut_smem_bytes(p.Mk, p.D);
    if (smem > 160 * 1024) return -2;
    static thread_local size_t configured = 0;
    if (smem > configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(decode_lut_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return -4;
        configured = smem;
    }
    dim3 grid(p.S, p.Hkv, p.B);
    hipLaunchKernelGGL(decode_lut_kernel, grid, dim3(kBlock), smem, stream, p);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

} // namespace vecinfer
