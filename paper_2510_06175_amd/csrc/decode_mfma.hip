// Matrix-core decode attention for gfx950: D = 128, G = 4 query heads per KV head,
// sub-vector dim d = 4 (32 sub-spaces) or d = 2 (64 sub-spaces), 8-bit codes.
//
// Both codebooks of the KV head live in LDS for the whole kernel.  A token's dequantized
// row is never assembled: each lane gathers a few centroids with ds_read and hands them
// straight to v_mfma_f32_16x16x32_f16 as an operand, so the matrix cores do the
// cross-lane summation that the lookup formulation needs.
//
//   scores (Eq. 10 / Alg. 1 step 11).  A 16-token tile is the A operand: lane (i, kg) owns
//   token row i and the k-range [8kg, 8kg+8), which it fills with the centroids of 8/d
//   consecutive sub-spaces of that token.  The B operand holds the transformed query:
//   column j = 4h + t0 carries q~_h (the same vector for the four t0), so the product's
//   column j is the score of head h and every lane ends up with the scores it will need as
//   a P.V operand.  q~ is split into an fp16 high and low part (two MFMAs) so that the
//   scores are fp32-accurate; 1/sqrt(D) and log2(e) are folded into q~.
//
//   P.V (Alg. 1 step 16).  Row 4h + t0 of the A operand holds p_h of 8/d tokens, placed
//   only in the k-slots whose channel-in-sub-vector equals t0; the B operand's column n
//   holds the gathered value centroids of those tokens for one sub-space.  The product's
//   row (h, t0), column n is then o_h[channel d*m(n) + t0].  3/4 of the A operand is
//   zero: the matrix cores have the headroom, and no cross-lane shuffle or transpose is
//   needed anywhere.
//
// Each wavefront runs its own online softmax (steps 12-13) over the 64-token tiles it owns;
// wavefronts are merged through LDS at the end of the split, splits through the workspace.
#include "common.h"

namespace vecinfer {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kG = 4;
constexpr int kTile = 64;          // tokens per wavefront iteration (4 sub-tiles of 16)

__device__ __forceinline__ half8 as_half8(unsigned a, unsigned b, unsigned c, unsigned d)
{
    uintx4 u = {a, b, c, d};
    return __builtin_bit_cast(half8, u);
}

__device__ __forceinline__ unsigned pack_dup_f16(float p)
{
    // (p, p) as two fp16, round-to-nearest-even
    const _Float16 h = (_Float16)p;
    const unsigned short b = __builtin_bit_cast(unsigned short, h);
    return (unsigned)b | ((unsigned)b << 16);
}

template <int DSUB, int NW>
__global__ __launch_bounds__(NW * 64) void decode_mfma_kernel(DecodeParams p)
{
    constexpr int BLOCK = NW * 64;
    constexpr int M = kD / DSUB;                       // sub-spaces: 32 or 64
    constexpr int CB_BYTES = kCentroids * kD * 2;      // one codebook set of a KV head: 64 KB
    constexpr int ENTRY = DSUB * 2;                    // bytes per centroid: 8 or 4
    constexpr int SUBSPACE_BYTES = kCentroids * ENTRY; // 2048 or 1024
    constexpr int KW = M / 16;                         // key-code dwords per lane per sub-tile: 2 or 4
    constexpr int NROUND_V = M / 16;                   // value MFMA rounds per P.V step: 2 or 4
    constexpr int PV_STEPS = DSUB / 2;                 // P.V steps per sub-tile: 2 (d=4) or 1 (d=2)

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *const sm_k = smem;
    unsigned char *const sm_v = smem + CB_BYTES;
    float *const sm_qt = reinterpret_cast<float *>(smem + 2 * CB_BYTES);   // [4][128]
    int *const sm_flag = reinterpret_cast<int *>(smem + 2 * CB_BYTES + sizeof(float) * kG * kD);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int s = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int col = lane & 15;       // MFMA row (A) / column (B, D) index of this lane
    const int kg = lane >> 4;        // k-group (A, B) / row group (D) of this lane
    const size_t bg = (size_t)b * p.Hkv + g;

    long long n0, n1;
    split_range(seq_len_of(p, b), p.S, s, kTile, n0, n1);

    if (n0 >= n1) {                                    // empty split: neutral partial
        for (int e = tid; e < kG * kD; e += BLOCK) p.part_o[(bg * p.S + s) * kG * kD + e] = 0.f;
        if (tid < kG) {
            p.part_m[(bg * p.S + s) * kG + tid] = -INFINITY;
            p.part_l[(bg * p.S + s) * kG + tid] = 0.f;
        }
        merge_if_last<BLOCK>(p, b, g, sm_flag);
        return;
    }

    // ---- stage both codebooks of this KV head in LDS (Alg. 1 step 7, and C_k likewise)
    {
        const uint4 *srck = reinterpret_cast<const uint4 *>(p.cb_k + (size_t)g * kCentroids * kD);
        const uint4 *srcv = reinterpret_cast<const uint4 *>(p.cb_v + (size_t)g * kCentroids * kD);
        uint4 *dk = reinterpret_cast<uint4 *>(sm_k);
        uint4 *dv = reinterpret_cast<uint4 *>(sm_v);
        for (int e = tid; e < CB_BYTES / 16; e += BLOCK) {
            dk[e] = srck[e];
            dv[e] = srcv[e];
        }
    }
    // ---- q~ = (q * lambda) H_D for the 4 heads of the group (un-normalised butterflies)
    for (int e = tid; e < kG * kD; e += BLOCK) {
        const int hh = e >> 7, c = e & 127;
        sm_qt[e] = __half2float(p.q[((size_t)b * p.Hq + g * kG + hh) * kD + c]) * p.lam[(size_t)g * kD + c];
    }
    __syncthreads();
    for (int st = 1; st < kD; st <<= 1) {
        float nv[(kG * kD + BLOCK - 1) / BLOCK];
        int it = 0;
        for (int e = tid; e < kG * kD; e += BLOCK, ++it) {
            const float mine = sm_qt[e], other = sm_qt[e ^ st];
            nv[it] = (e & st) ? (other - mine) : (mine + other);
        }
        __syncthreads();
        it = 0;
        for (int e = tid; e < kG * kD; e += BLOCK, ++it) sm_qt[e] = nv[it];
        __syncthreads();
    }

    // ---- B operands of the score MFMAs: q~_h[32kg + 8r .. +8), hi and lo fp16 parts.
    // fold = (1/sqrt D of H_D) * (1/sqrt D of the score) * log2 e
    half8 bq_hi[4], bq_lo[4];
    {
        const float fold = kLog2e / (float)kD;
        const int hh = col >> 2;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = sm_qt[hh * kD + 32 * kg + 8 * r + e] * fold;
                const _Float16 hi = (_Float16)x;
                bq_hi[r][e] = hi;
                bq_lo[r][e] = (_Float16)(x - (float)hi);
            }
    }

    // ---- per-lane constants
    const int t0 = col & 3;                              // channel-in-sub-vector this A row serves
    unsigned mask_a, mask_b;                             // select the fp16 slot(s) of (p, p)
    if (DSUB == 4) {
        mask_a = t0 == 0 ? 0x0000ffffu : (t0 == 1 ? 0xffff0000u : 0u);
        mask_b = t0 == 2 ? 0x0000ffffu : (t0 == 3 ? 0xffff0000u : 0u);
    } else {
        mask_a = t0 == 0 ? 0x0000ffffu : (t0 == 1 ? 0xffff0000u : 0u);
        mask_b = 0u;
    }
    // LDS byte offsets: keys  sub-space (8/d)*(8kg.. ) i.e. M/4 sub-spaces per kg
    //                   values sub-space NROUND_V*col + r
    const unsigned lds_k = (unsigned)(kg * (M / 4) * SUBSPACE_BYTES);
    const unsigned lds_v = (unsigned)(CB_BYTES + col * NROUND_V * SUBSPACE_BYTES);

    const uint8_t *krow = p.k_idx + bg * p.n_cap * M;
    const uint8_t *vrow = p.v_idx + bg * p.n_cap * M;
    const long long last = n1 - 1;

    // token owned by A-row i of sub-tile st: base + 16 st + 4 (i % 4) + i / 4, so that D-register v
    // of row group rg is token base + 16 st + 4 v + rg
    const int krow_tok = 4 * (col & 3) + (col >> 2);

    float m_run = -INFINITY;          // running max of head col/4 (log2 units), same in all its lanes
    float l_part = 0.f;               // this lane's share of the running sum
    floatx4 acc_o[NROUND_V];
#pragma unroll
    for (int r = 0; r < NROUND_V; ++r) acc_o[r] = floatx4{0.f, 0.f, 0.f, 0.f};

    for (long long tb = n0 + (long long)wave * kTile; tb < n1; tb += (long long)NW * kTile) {
        // ---- codes of this tile
        unsigned kc[4][KW];
        unsigned vc[4][4];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            long long tk = tb + 16 * st + krow_tok;
            tk = tk > last ? last : tk;
            const unsigned char *src = krow + (size_t)tk * M + kg * (M / 4);
            if (DSUB == 4) {
                const uint2 w = *reinterpret_cast<const uint2 *>(src);
                kc[st][0] = w.x;
                kc[st][1] = w.y;
            } else {
                const uint4 w = *reinterpret_cast<const uint4 *>(src);
                kc[st][0] = w.x; kc[st][1] = w.y; kc[st][KW - 2] = w.z; kc[st][KW - 1] = w.w;
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                long long tv = tb + 16 * st + 4 * v + kg;
                tv = tv > last ? last : tv;
                const unsigned char *vs = vrow + (size_t)tv * M + col * NROUND_V;
                if (DSUB == 4)
                    vc[st][v] = *reinterpret_cast<const unsigned short *>(vs);
                else
                    vc[st][v] = *reinterpret_cast<const unsigned *>(vs);
            }
        }

        // ---- scores: 4 sub-tiles x 4 rounds x (hi, lo)
        floatx4 sacc[4];
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                half8 a;
                if (DSUB == 4) {
                    // sub-spaces 8kg + 2r, 8kg + 2r + 1: code bytes 2r, 2r+1 of the lane's 8
                    const unsigned w = kc[st][r >> 1];
                    const unsigned c0 = (w >> (16 * (r & 1))) & 255u;
                    const unsigned c1 = (w >> (16 * (r & 1) + 8)) & 255u;
                    const uint2 x0 = *reinterpret_cast<const uint2 *>(smem + lds_k + (2 * r) * SUBSPACE_BYTES + c0 * ENTRY);
                    const uint2 x1 = *reinterpret_cast<const uint2 *>(smem + lds_k + (2 * r + 1) * SUBSPACE_BYTES + c1 * ENTRY);
                    a = as_half8(x0.x, x0.y, x1.x, x1.y);
                } else {
                    // sub-spaces 16kg + 4r .. +3: the 4 code bytes of dword r
                    const unsigned w = kc[st][r];
                    unsigned x[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const unsigned c = (w >> (8 * q)) & 255u;
                        x[q] = *reinterpret_cast<const unsigned *>(smem + lds_k + (4 * r + q) * SUBSPACE_BYTES + c * ENTRY);
                    }
                    a = as_half8(x[0], x[1], x[2], x[3]);
                }
                sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq_hi[r], sacc[st], 0, 0, 0);
                sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq_lo[r], sacc[st], 0, 0, 0);
            }

        // ---- online softmax of this wavefront (Alg. 1 steps 12-13)
        float tmax = -INFINITY;
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const long long tok = tb + 16 * st + 4 * v + kg;
                if (tok > last) sacc[st][v] = -INFINITY;
                tmax = fmaxf(tmax, sacc[st][v]);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        if (__any(m_new > m_run)) {
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first tile
            l_part *= alpha;
            const float alpha_o = __shfl(alpha, 4 * kg);                 // head kg's factor (lane 4kg serves head kg)
#pragma unroll
            for (int r = 0; r < NROUND_V; ++r) acc_o[r] *= alpha_o;
            m_run = m_new;
        }
        unsigned pp[4][4];
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float pr = __builtin_amdgcn_exp2f(sacc[st][v] - m_run);
                l_part += pr;
                pp[st][v] = pack_dup_f16(pr);
            }

        // ---- o += P . VQ^-1(V_q)  (step 16)
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            if (DSUB == 4) {
#pragma unroll
                for (int u = 0; u < PV_STEPS; ++u) {
                    const half8 a = as_half8(pp[st][2 * u] & mask_a, pp[st][2 * u] & mask_b,
                                             pp[st][2 * u + 1] & mask_a, pp[st][2 * u + 1] & mask_b);
#pragma unroll
                    for (int r = 0; r < NROUND_V; ++r) {
                        const unsigned c0 = (vc[st][2 * u] >> (8 * r)) & 255u;
                        const unsigned c1 = (vc[st][2 * u + 1] >> (8 * r)) & 255u;
                        const uint2 x0 = *reinterpret_cast<const uint2 *>(smem + lds_v + r * SUBSPACE_BYTES + c0 * ENTRY);
                        const uint2 x1 = *reinterpret_cast<const uint2 *>(smem + lds_v + r * SUBSPACE_BYTES + c1 * ENTRY);
                        acc_o[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, as_half8(x0.x, x0.y, x1.x, x1.y), acc_o[r], 0, 0, 0);
                    }
                }
            } else {
                const half8 a = as_half8(pp[st][0] & mask_a, pp[st][1] & mask_a, pp[st][2] & mask_a, pp[st][3] & mask_a);
#pragma unroll
                for (int r = 0; r < NROUND_V; ++r) {
                    unsigned x[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const unsigned c = (vc[st][v] >> (8 * r)) & 255u;
                        x[v] = *reinterpret_cast<const unsigned *>(smem + lds_v + r * SUBSPACE_BYTES + c * ENTRY);
                    }
                    acc_o[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, as_half8(x[0], x[1], x[2], x[3]), acc_o[r], 0, 0, 0);
                }
            }
        }
    }

    // ---- merge the wavefronts of this split through LDS (the codebooks are no longer needed)
    float l_head = l_part + __shfl_xor(l_part, 16);
    l_head += __shfl_xor(l_head, 32);
    __syncthreads();
    float *const sm_o = reinterpret_cast<float *>(smem);                  // [NW][4][128]
    float *const sm_m = sm_o + NW * kG * kD;                              // [NW][4]
    float *const sm_l = sm_m + NW * kG;                                   // [NW][4]
    {
        // acc_o[r] register v of lane (col, kg): head kg, channel d * (NROUND_V * col + r) + v
#pragma unroll
        for (int r = 0; r < NROUND_V; ++r)
#pragma unroll
            for (int v = 0; v < DSUB; ++v)
                sm_o[(wave * kG + kg) * kD + DSUB * (NROUND_V * col + r) + v] = acc_o[r][v];
        if (kg == 0 && (col & 3) == 0) {
            sm_m[wave * kG + (col >> 2)] = m_run;
            sm_l[wave * kG + (col >> 2)] = l_head;
        }
    }
    __syncthreads();
    for (int e = tid; e < kG * kD; e += BLOCK) {
        const int hh = e >> 7;
        float mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) mx = fmaxf(mx, sm_m[w * kG + hh]);
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = sm_m[w * kG + hh];
            const float f = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - mx) : 0.f;
            o += f * sm_o[w * kG * kD + e];
            l += f * sm_l[w * kG + hh];
        }
        const size_t pi = (bg * p.S + s) * kG;
        p.part_o[pi * kD + e] = o;
        if ((e & 127) == 0) {
            p.part_m[pi + hh] = mx;
            p.part_l[pi + hh] = l;
        }
    }
    merge_if_last<BLOCK>(p, b, g, sm_flag);
}

constexpr int kWaves = 8;

template <int DSUB>
int launch_typed(const DecodeParams &p, hipStream_t stream)
{
    constexpr size_t smem = 2 * (size_t)kCentroids * kD * 2 + sizeof(float) * kG * kD + 16;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(decode_mfma_kernel<DSUB, kWaves>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return -4;
        configured = true;
    }
    dim3 grid(p.S, p.Hkv, p.B);
    hipLaunchKernelGGL((decode_mfma_kernel<DSUB, kWaves>), grid, dim3(kWaves * 64), smem, stream, p);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

} // namespace

bool decode_mfma_supports(const DecodeParams &p)
{
    return p.D == kD && p.G == kG && p.dk == p.dv && (p.dk == 4 || p.dk == 2);
}

int launch_decode_mfma(const DecodeParams &p, hipStream_t stream)
{
    if (!decode_mfma_supports(p)) return -2;
    return p.dk == 4 ? launch_typed<4>(p, stream) : launch_typed<2>(p, stream);
}

} // namespace vecinfer
