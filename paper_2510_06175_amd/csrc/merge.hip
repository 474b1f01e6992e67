// Second kernel of a decode step: log-sum-exp merge of the split partials, and, when the caller
// keeps the most recent tokens unquantized (Sec. 4.1, residual length), attention over that
// fp16 window computed here and merged in with them.
//
// The kernel runs right behind the attention kernel on data that sits in other compute units'
// caches or in memory, so what it costs is dependent memory round trips, not arithmetic: every
// global load it needs is issued up front, back to back, and consumed after one barrier.
#include "common.h"

namespace vecinfer {
namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxSplits = 256;                         // VECINFER_MAX_SPLITS
constexpr int kBatch = 32;                              // split partials a thread keeps in flight
constexpr int kRowsPerWave = kMaxResidual / kWaves;     // 16: one MFMA column block of window rows per wave
static_assert(kRowsPerWave == 16, "a wave scores 16 window rows with 16x16x32 MFMAs");

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// x of the lane N places further on in its row of 16 lanes (DPP row_ror)
template <int N>
__device__ __forceinline__ float row_ror(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0x120 + N, 0xf, 0xf, true));
}

// One workgroup per (KV head g, sequence b); D = head dim, HB = bound on G (4 or 8), MODE below.
//
// Merge (the paper returns L from each tile loop, Alg. 1 step 22, and leaves the merge to the reader):
//   M = max_s m_s,  w_s = 2^(m_s - M),  o = sum_s w_s o_s / sum_s w_s l_s,  L = (M + log2 sum) ln 2.
// A thread owns output elements e = hh * D + c; it loads its o_s for the first kBatch splits at
// once (clamped to the last split; the (m, l) table in LDS is padded with m = -inf so that the
// surplus gets weight 0), the (m, l) pairs go through LDS.
//
// Window (WINDOW = true): rows are scored with the raw query against the raw keys,
// q . k = (q * lambda) H . (k / lambda) H (Eq. 7), so the scores live on the same scale as the
// quantized tokens' and share their softmax.  Wave w owns rows 16 w .. 16 w + 15 and turns them
// into one more partial (m, l, o):
//   scores  S[hh][r] = q[hh] . k[r] on the matrix cores.  v_mfma_f32_16x16x32_f16 wants, per lane
//           l, eight consecutive k-values of row / column l % 16 starting at 8 (l / 16): for both
//           the query rows and the row-major window keys that is one 16-byte global load, so the
//           operands come straight from memory.  The result lands with window row l % 16 in lane l
//           and head 4 (l / 16) + v in register v.
//   softmax over the 16 rows: DPP row rotations inside each 16-lane group.
//   o[hh][c] = sum_r p[hh][r] v[r][c] on the vector ALU: a lane owns two adjacent channels, p comes
//           from the owning lane by v_readlane.
// Window loads are clamped to row R - 1 (always inside the allocation) and masked by the
// sequence's own window length afterwards, so they do not wait for that length to arrive.
//
// New token (MODE = kNewToken, the fused append of Eq. 9): the attention kernel left, per key
// sub-space, the new token's score share for each head and, per channel, its dequantized
// value; the token joins as the partial (m = sum of the shares, l = 1, o = value).
enum { kPlain = 0, kWindow = 1, kNewToken = 2 };

//
// Arguments.  The first 14 dwords of a kernel's arguments can reach the wavefront in scalar
// registers (kernel-argument preloading), everything behind them costs a cold trip to the argument
// buffer before the loads that need it can leave.  They are therefore exactly what the first
// requests of each mode use: the three partial arrays; three mode pointers xa, xb, xc (window: q,
// k_res, v_res; new token: its score shares, its value, seq_lens); one packed dword
// S | G << 9 | min(Hkv, 2047) << 13 | i0 << 24 (i0: window rows R, or M_k of the new token; 2047
// stands for "read the grid's x extent", which is Hkv); and i1 (window: r_cap; new token: N clamped
// to an int).  `out`, `lse` and the window's own lengths are needed at the end and ride behind.
template <int D, int HB, int MODE>
__global__ __launch_bounds__(kThreads) void merge_kernel(const float *part_o, const float *part_m, const float *part_l,
                                                         const void *xa, const void *xb, const void *xc, unsigned packed,
                                                         int i1, __half *out, float *lse, const int32_t *res_lens)
{
    const int S = (int)(packed & 0x1ffu), G = (int)(packed >> 9 & 0xfu);
    const int Hkv = (packed >> 13 & 0x7ffu) < 0x7ffu ? (int)(packed >> 13 & 0x7ffu) : (int)gridDim.x;
    const int i0 = (int)(packed >> 24), Hq = Hkv * G;
    constexpr bool WINDOW = MODE == kWindow;
    constexpr int kMaxM = D / 2;                                      // key sub-spaces at d = 2
    constexpr int kSteps = D / 32;                                   // MFMA k-steps over the head dimension
    constexpr int kElems = (HB * D + kThreads - 1) / kThreads;       // output elements per thread
    constexpr int kML = kMaxSplits * HB / kThreads;                  // (m, l) table entries per thread
    __shared__ float pm_s[kMaxSplits * HB], pl_s[kMaxSplits * HB];   // [s][hh], padded to a multiple of kBatch splits
    __shared__ float wo_s[WINDOW ? kWaves * HB * D : 1];             // wave partial outputs, [wave][hh][c]
    __shared__ float wm_s[kWaves * HB], wl_s[kWaves * HB];
    __shared__ float ns_s[MODE == kNewToken ? kMaxM * HB : 1];      // [m][hh] score shares of the new token
    __shared__ float nv_s[MODE == kNewToken ? D : 1];

    const int g = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
    const int w = t >> 6, lane = t & 63;
    const int GD = G * D;
    const size_t bg = (size_t)b * Hkv + g;

    // ---- 1. split partials: this thread's o_s of the first kBatch splits, and its share of the (m, l)
    // table.  These requests use the leading kernel arguments only, which the command processor can
    // hand over in scalar registers (kernel-argument preloading): they leave before the rest of
    // `p` has made its trip from the argument buffer.
    float vo[kElems][kBatch], tm[kML], tl[kML];
    const int SG = S * G;
    if (S > 0) {
        const float *po = part_o + bg * S * GD;
        const float *pm = part_m + bg * SG;
        const float *pl = part_l + bg * SG;
#pragma unroll
        for (int i = 0; i < kElems; ++i) {
            const int e = t + i * kThreads < GD ? t + i * kThreads : 0;
#pragma unroll
            for (int j = 0; j < kBatch; ++j) vo[i][j] = po[(size_t)(j < S ? j : S - 1) * GD + e];
        }
#pragma unroll
        for (int i = 0; i < kML; ++i) {
            const int idx = t + i * kThreads < SG ? t + i * kThreads : SG - 1;
            tm[i] = pm[idx];
            tl[i] = pl[idx];
        }
    }

    // ---- 2. window operands -> registers
    half8 qa[kSteps], kb[kSteps];
    unsigned vv[kRowsPerWave];
    const int row0 = w * kRowsPerWave;
    const int R = WINDOW ? i0 : 0, r_cap = i1;
    const bool wave_loads = WINDOW && row0 < R;              // wave-uniform
    int r_len = 0;
    if (WINDOW) {
        r_len = R;
        if (res_lens) {
            const int v = res_lens[b];
            r_len = v < 0 ? 0 : (v > R ? R : v);
        }
        if (wave_loads) {
            const __half *kg = static_cast<const __half *>(xb) + bg * r_cap * D;
            const __half *vg = static_cast<const __half *>(xc) + bg * r_cap * D;
            const __half *qg = static_cast<const __half *>(xa) + ((size_t)b * Hq + (size_t)g * G) * D;
            const int last = R - 1;
            const int qrow = (lane & 15) < G ? (lane & 15) : 0;
            const int krow = row0 + (lane & 15) < last ? row0 + (lane & 15) : last;
#pragma unroll
            for (int ks = 0; ks < kSteps; ++ks) {
                const int col = ks * 32 + 8 * (lane >> 4);
                qa[ks] = *reinterpret_cast<const half8 *>(qg + qrow * D + col);
                kb[ks] = *reinterpret_cast<const half8 *>(kg + (size_t)krow * D + col);
            }
            const int c2 = 2 * lane < D ? 2 * lane : 0;
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r) {
                const int vrow = row0 + r < last ? row0 + r : last;
                vv[r] = *reinterpret_cast<const unsigned *>(vg + (size_t)vrow * D + c2);
            }
        }
    }

    // new token: its shares and value (read unconditionally; ignored for an empty sequence)
    const int Mk = MODE == kNewToken ? i0 : 0;
    int len_b = MODE == kNewToken ? i1 : 0;                  // only its sign matters here
    float nsc = 0.f, nvv = 0.f;
    if (MODE == kNewToken) {
        if (xc) {
            // b is the same for the whole workgroup: read through the constant address space, i.e. by
            // a scalar load, which does not queue behind the wavefront's vector loads
            typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
            const int v = ((const_i32_ptr)(uintptr_t)xc)[b];
            len_b = v < len_b ? v : len_b;
        }
        if (t < Mk * G) nsc = static_cast<const float *>(xa)[bg * Mk * G + t];
        if (t < D) nvv = static_cast<const float *>(xb)[bg * D + t];
    }

    // ---- 3. the wave's window partial -> LDS
    if (WINDOW && row0 < r_len) {
        floatx4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < kSteps; ++ks) sc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[ks], kb[ks], sc, 0, 0, 0);
        const float scale = kLog2e * rsqrtf((float)D);
        const bool valid = row0 + (lane & 15) < r_len;
        float pr[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float s2 = valid ? sc[v] * scale : -INFINITY;
            // (all-reduce over the 16-lane row by DPP rotations: no trip through the LDS crossbar)
            float m = s2;
            m = fmaxf(m, row_ror<8>(m));
            m = fmaxf(m, row_ror<4>(m));
            m = fmaxf(m, row_ror<2>(m));
            m = fmaxf(m, row_ror<1>(m));
            pr[v] = __builtin_amdgcn_exp2f(s2 - m);          // row row0 is valid, so m is finite
            float l = pr[v];
            l += row_ror<8>(l);
            l += row_ror<4>(l);
            l += row_ror<2>(l);
            l += row_ror<1>(l);
            const int hh = 4 * (lane >> 4) + v;
            if ((lane & 15) == 0 && hh < HB) {               // heads G .. HB - 1 hold finite filler
                wm_s[w * HB + hh] = m;
                wl_s[w * HB + hh] = l;
            }
        }
        float o2[HB][2];
#pragma unroll
        for (int hh = 0; hh < HB; ++hh) o2[hh][0] = o2[hh][1] = 0.f;
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) {
            const float2 vf = __half22float2(*reinterpret_cast<const __half2 *>(&vv[r]));
#pragma unroll
            for (int hh = 0; hh < HB; ++hh) {
                const float ph = __uint_as_float(
                    __builtin_amdgcn_readlane(__float_as_uint(pr[hh & 3]), 16 * (hh >> 2) + r));
                o2[hh][0] = fmaf(ph, vf.x, o2[hh][0]);
                o2[hh][1] = fmaf(ph, vf.y, o2[hh][1]);
            }
        }
        if (2 * lane < D) {
#pragma unroll
            for (int hh = 0; hh < HB; ++hh)
                *reinterpret_cast<float2 *>(&wo_s[(w * HB + hh) * D + 2 * lane]) = make_float2(o2[hh][0], o2[hh][1]);
        }
    }

    if (MODE == kNewToken) {
        if (t < Mk * G) ns_s[t] = nsc;
        if (t < D) nv_s[t] = nvv;
    }

    // ---- 4. (m, l) table -> LDS, padded with empty splits up to a multiple of kBatch
    const int Spad = (S + kBatch - 1) / kBatch * kBatch;
#pragma unroll
    for (int i = 0; i < kML; ++i) {
        const int idx = t + i * kThreads;
        if (idx < Spad * G) {
            pm_s[idx] = idx < SG ? tm[i] : -INFINITY;
            pl_s[idx] = idx < SG ? tl[i] : 0.f;
        }
    }
    __syncthreads();

    // ---- 5. merge and write the rows
    const int n_waves = WINDOW ? (r_len + kRowsPerWave - 1) / kRowsPerWave : 0;
    const bool new_tok = MODE == kNewToken && len_b > 0;
#pragma unroll
    for (int i = 0; i < kElems; ++i) {
        const int e = t + i * kThreads;
        if (e >= GD) continue;
        const int hh = e / D, c = e % D;
        float M = -INFINITY;
        for (int s = 0; s < S; ++s) M = fmaxf(M, pm_s[s * G + hh]);
        for (int ww = 0; ww < n_waves; ++ww) M = fmaxf(M, wm_s[ww * HB + hh]);
        float s_new = -INFINITY;
        if (new_tok) {
            s_new = 0.f;
            for (int m = 0; m < Mk; ++m) s_new += ns_s[m * G + hh];
            M = fmaxf(M, s_new);
        }
        const float Mc = M > -INFINITY ? M : 0.f;            // nothing to attend to: all weights 0
        float den = 0.f, acc = 0.f;
        if (S > 0) {
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const float wgt = __builtin_amdgcn_exp2f(pm_s[j * G + hh] - Mc);
                den = fmaf(wgt, pl_s[j * G + hh], den);
                acc = fmaf(wgt, vo[i][j], acc);
            }
            const float *po = part_o + bg * S * GD;
            for (int s0 = kBatch; s0 < S; s0 += kBatch) {    // more than kBatch splits: further rounds
                float vx[kBatch];
#pragma unroll
                for (int j = 0; j < kBatch; ++j) vx[j] = po[(size_t)(s0 + j < S ? s0 + j : S - 1) * GD + e];
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    const float wgt = __builtin_amdgcn_exp2f(pm_s[(s0 + j) * G + hh] - Mc);
                    den = fmaf(wgt, pl_s[(s0 + j) * G + hh], den);
                    acc = fmaf(wgt, vx[j], acc);
                }
            }
        }
        for (int ww = 0; ww < n_waves; ++ww) {
            const float wgt = __builtin_amdgcn_exp2f(wm_s[ww * HB + hh] - Mc);
            den = fmaf(wgt, wl_s[ww * HB + hh], den);
            acc = fmaf(wgt, wo_s[(ww * HB + hh) * D + c], acc);
        }
        if (new_tok) {
            const float wgt = __builtin_amdgcn_exp2f(s_new - Mc);
            den += wgt;
            acc = fmaf(wgt, nv_s[c], acc);
        }
        const size_t row = (size_t)b * Hq + g * G + hh;
        out[row * D + c] = __float2half(den > 0.f ? acc / den : 0.f);
        if (c == 0 && lse) lse[row] = den > 0.f ? (M + log2f(den)) * kLn2 : -INFINITY;
    }
}

template <int D, int HB>
int launch_for(const DecodeParams &p, hipStream_t stream)
{
    const dim3 grid(p.Hkv, p.B), block(kThreads);
    const unsigned base = (unsigned)p.S | (unsigned)p.G << 9 | (unsigned)(p.Hkv < 2047 ? p.Hkv : 2047) << 13;
    if (p.k_res)
        hipLaunchKernelGGL((merge_kernel<D, HB, kWindow>), grid, block, 0, stream, p.part_o, p.part_m, p.part_l,
                           (const void *)p.q, (const void *)p.k_res, (const void *)p.v_res, base | (unsigned)p.R << 24, (int)p.r_cap,
                           p.out, p.lse, p.res_lens);
    else if (p.k_new)
        hipLaunchKernelGGL((merge_kernel<D, HB, kNewToken>), grid, block, 0, stream, p.part_o, p.part_m, p.part_l,
                           (const void *)p.new_sc, (const void *)p.new_v, (const void *)p.seq_lens, base | (unsigned)p.Mk << 24,
                           (int)(p.N < 0x7fffffffLL ? p.N : 0x7fffffffLL), p.out, p.lse, (const int32_t *)nullptr);
    else
        hipLaunchKernelGGL((merge_kernel<D, HB, kPlain>), grid, block, 0, stream, p.part_o, p.part_m, p.part_l,
                           (const void *)nullptr, (const void *)nullptr, (const void *)nullptr, base, 0, p.out, p.lse,
                           (const int32_t *)nullptr);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

} // namespace

int launch_merge(const DecodeParams &p, hipStream_t stream)
{
    // (field widths of the kernel's packed argument)
    if (p.S > kMaxSplits || p.G > 8 || p.Hq != p.Hkv * p.G || p.Mk > 255 ||
        (p.k_res && (p.R > kMaxResidual || p.r_cap > 0x7fffffffLL))) return -2;
    static_assert(kMaxSplits < 512 && kMaxResidual < 256, "packed merge argument");
    if (p.D == 128) return p.G <= 4 ? launch_for<128, 4>(p, stream) : launch_for<128, 8>(p, stream);
    if (p.D == 64) return p.G <= 4 ? launch_for<64, 4>(p, stream) : launch_for<64, 8>(p, stream);
    return -2;
}

} // namespace vecinfer
