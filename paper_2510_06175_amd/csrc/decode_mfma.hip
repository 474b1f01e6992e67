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

#ifdef VECINFER_PHASE_TIMING
__device__ unsigned long long *g_phase_buf = nullptr;
#define STAMP(i) do { if (g_phase_buf && threadIdx.x == 0) g_phase_buf[((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 8 + (i)] = wall_clock64(); } while (0)
#else
#define STAMP(i)
#endif

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

    STAMP(0);
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
    __syncthreads(); STAMP(1);
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

    STAMP(2);
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

    // Codes of one 64-token tile as this lane needs them: kc = the key-code bytes of the lane's
    // A row in each sub-tile, vc = the value-code bytes of the 4 tokens of its k-group.
    struct Codes {
        unsigned kc[4][KW];
        unsigned vc[4][4];
    };
    // 32-bit byte offsets into the (b, g) code rows (the host checks n_cap * M < 2^31)
    const unsigned koff_lane = (unsigned)(krow_tok * M + kg * (M / 4));
    const unsigned voff_lane = (unsigned)(kg * M + col * NROUND_V);
    const unsigned last_off = (unsigned)last * M;

    auto load_codes = [&](Codes &cd, long long tb) {
        if (tb + kTile <= n1) {                 // whole tile in range (uniform over the wavefront)
            const unsigned base = (unsigned)tb * M;
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const unsigned char *src = krow + (base + koff_lane + 16 * st * M);
                if (DSUB == 4) {
                    const uint2 w = *reinterpret_cast<const uint2 *>(src);
                    cd.kc[st][0] = w.x; cd.kc[st][1] = w.y;
                } else {
                    const uint4 w = *reinterpret_cast<const uint4 *>(src);
                    cd.kc[st][0] = w.x; cd.kc[st][1] = w.y; cd.kc[st][KW - 2] = w.z; cd.kc[st][KW - 1] = w.w;
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const unsigned char *vs = vrow + (base + voff_lane + (16 * st + 4 * v) * M);
                    if (DSUB == 4)
                        cd.vc[st][v] = *reinterpret_cast<const unsigned short *>(vs);
                    else
                        cd.vc[st][v] = *reinterpret_cast<const unsigned *>(vs);
                }
            }
        } else {                                // tail (or past the end): clamp to the last token
            const long long tbc = tb > last ? last : tb;
            const unsigned base = (unsigned)tbc * M;
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                unsigned ko = base + (16 * st + krow_tok) * M;
                ko = (ko > last_off ? last_off : ko) + kg * (M / 4);
                const unsigned char *src = krow + ko;
                if (DSUB == 4) {
                    const uint2 w = *reinterpret_cast<const uint2 *>(src);
                    cd.kc[st][0] = w.x; cd.kc[st][1] = w.y;
                } else {
                    const uint4 w = *reinterpret_cast<const uint4 *>(src);
                    cd.kc[st][0] = w.x; cd.kc[st][1] = w.y; cd.kc[st][KW - 2] = w.z; cd.kc[st][KW - 1] = w.w;
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    unsigned vo = base + (16 * st + 4 * v + kg) * M;
                    vo = (vo > last_off ? last_off : vo) + col * NROUND_V;
                    const unsigned char *vs = vrow + vo;
                    if (DSUB == 4)
                        cd.vc[st][v] = *reinterpret_cast<const unsigned short *>(vs);
                    else
                        cd.vc[st][v] = *reinterpret_cast<const unsigned *>(vs);
                }
            }
        }
    };

    // A operand of the score MFMA for sub-tile st, round r: the centroids of 8/d consecutive
    // key sub-spaces of the lane's token (pure LDS gathers, no arithmetic).
    auto gather_k = [&](const Codes &cd, int st, int r) -> half8 {
        if (DSUB == 4) {
            // sub-spaces 8kg + 2r, 8kg + 2r + 1: code bytes 2r, 2r+1 of the lane's 8
            const unsigned w = cd.kc[st][r >> 1];
            const unsigned c0 = (w >> (16 * (r & 1))) & 255u;
            const unsigned c1 = (w >> (16 * (r & 1) + 8)) & 255u;
            const uint2 x0 = *reinterpret_cast<const uint2 *>(smem + lds_k + (2 * r) * SUBSPACE_BYTES + c0 * ENTRY);
            const uint2 x1 = *reinterpret_cast<const uint2 *>(smem + lds_k + (2 * r + 1) * SUBSPACE_BYTES + c1 * ENTRY);
            return as_half8(x0.x, x0.y, x1.x, x1.y);
        } else {
            // sub-spaces 16kg + 4r .. +3: the 4 code bytes of dword r
            const unsigned w = cd.kc[st][r];
            unsigned x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned c = (w >> (8 * q)) & 255u;
                x[q] = *reinterpret_cast<const unsigned *>(smem + lds_k + (4 * r + q) * SUBSPACE_BYTES + c * ENTRY);
            }
            return as_half8(x[0], x[1], x[2], x[3]);
        }
    };
    // B operand q (0..3) of the P.V MFMAs of sub-tile st.  d = 4: q = 2u + r (step u, round r):
    // centroids of sub-space 2 col + r for tokens 2u, 2u+1 of the k-group.  d = 2: q = r:
    // centroids of sub-space 4 col + r for the 4 tokens of the k-group.
    auto gather_v = [&](const Codes &cd, int st, int q) -> half8 {
        if (DSUB == 4) {
            const int u = q >> 1, r = q & 1;
            const unsigned c0 = (cd.vc[st][2 * u] >> (8 * r)) & 255u;
            const unsigned c1 = (cd.vc[st][2 * u + 1] >> (8 * r)) & 255u;
            const uint2 x0 = *reinterpret_cast<const uint2 *>(smem + lds_v + r * SUBSPACE_BYTES + c0 * ENTRY);
            const uint2 x1 = *reinterpret_cast<const uint2 *>(smem + lds_v + r * SUBSPACE_BYTES + c1 * ENTRY);
            return as_half8(x0.x, x0.y, x1.x, x1.y);
        } else {
            unsigned x[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const unsigned c = (cd.vc[st][v] >> (8 * q)) & 255u;
                x[v] = *reinterpret_cast<const unsigned *>(smem + lds_v + q * SUBSPACE_BYTES + c * ENTRY);
            }
            return as_half8(x[0], x[1], x[2], x[3]);
        }
    };

    half8 ka[8];                     // score operands of rounds 0-1 of the tile about to be processed
    // One tile.  LDS gathers are issued one stage ahead of the MFMAs that consume them, in the
    // order: [rounds 2-3 of K] MFMA(K 0-1) [V of sub-tiles 0-1] MFMA(K 2-3) softmax
    // [V of sub-tiles 2-3] MFMA(V 0-1) [rounds 0-1 of K of the NEXT tile] MFMA(V 2-3).
    auto process_tile = [&](Codes &cd, const Codes &next, long long tb, long long tb_refill) {
        half8 kb[8], va[8], vb[8];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            kb[2 * st] = gather_k(cd, st, 2);
            kb[2 * st + 1] = gather_k(cd, st, 3);
        }
        __builtin_amdgcn_sched_barrier(0);
        floatx4 sacc[4];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[2 * st], bq_hi[0], floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[2 * st], bq_lo[0], sacc[st], 0, 0, 0);
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[2 * st + 1], bq_hi[1], sacc[st], 0, 0, 0);
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[2 * st + 1], bq_lo[1], sacc[st], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            va[q] = gather_v(cd, 0, q);
            va[4 + q] = gather_v(cd, 1, q);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb[2 * st], bq_hi[2], sacc[st], 0, 0, 0);
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb[2 * st], bq_lo[2], sacc[st], 0, 0, 0);
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb[2 * st + 1], bq_hi[3], sacc[st], 0, 0, 0);
#pragma unroll
        for (int st = 0; st < 4; ++st) sacc[st] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb[2 * st + 1], bq_lo[3], sacc[st], 0, 0, 0);

        // ---- online softmax of this wavefront (Alg. 1 steps 12-13)
        if (tb + kTile > n1) {                  // tail tile: tokens past the end get p = 0
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (tb + 16 * st + 4 * v + kg > last) sacc[st][v] = -INFINITY;
        }
        float tmax = fmaxf(fmaxf(sacc[0][0], sacc[0][1]), fmaxf(sacc[0][2], sacc[0][3]));
#pragma unroll
        for (int st = 1; st < 4; ++st)
            tmax = fmaxf(tmax, fmaxf(fmaxf(sacc[st][0], sacc[st][1]), fmaxf(sacc[st][2], sacc[st][3])));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        if (__any(m_new > m_run)) {
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first tile
            l_part *= alpha;
            const float alpha_o = __shfl(alpha, 4 * kg);                 // lane 4kg serves head kg
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
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            vb[q] = gather_v(cd, 2, q);
            vb[4 + q] = gather_v(cd, 3, q);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_codes(cd, tb_refill);                // cd is consumed: refill it two tiles ahead
        __builtin_amdgcn_sched_barrier(0);

        // ---- o += P . VQ^-1(V_q)  (step 16)
        auto pv = [&](int st, const half8 *vops) {
            if (DSUB == 4) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const half8 a = as_half8(pp[st][2 * u] & mask_a, pp[st][2 * u] & mask_b,
                                             pp[st][2 * u + 1] & mask_a, pp[st][2 * u + 1] & mask_b);
#pragma unroll
                    for (int r = 0; r < 2; ++r)
                        acc_o[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, vops[2 * u + r], acc_o[r], 0, 0, 0);
                }
            } else {
                const half8 a = as_half8(pp[st][0] & mask_a, pp[st][1] & mask_a, pp[st][2] & mask_a, pp[st][3] & mask_a);
#pragma unroll
                for (int r = 0; r < NROUND_V; ++r)
                    acc_o[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, vops[r], acc_o[r], 0, 0, 0);
            }
        };
        pv(0, va);
        pv(1, va + 4);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < 4; ++st) {          // first half of the next tile's score operands
            ka[2 * st] = gather_k(next, st, 0);
            ka[2 * st + 1] = gather_k(next, st, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        pv(2, vb);
        pv(3, vb + 4);
    };

    // Two tiles of codes in flight: a tile's registers are refilled (two tiles ahead) as soon as
    // its last gather has been issued.  Loads past the end of the split are clamped to its last
    // token, so the refill and the look-ahead gathers need no bounds branch.
    {
        const long long stride = (long long)NW * kTile;
        long long tb = n0 + (long long)wave * kTile;
        Codes ca, cb;
        load_codes(ca, tb);
        load_codes(cb, tb + stride);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            ka[2 * st] = gather_k(ca, st, 0);
            ka[2 * st + 1] = gather_k(ca, st, 1);
        }
        for (; tb < n1; tb += 2 * stride) {
            process_tile(ca, cb, tb, tb + 2 * stride);
            if (tb + stride < n1) process_tile(cb, ca, tb + stride, tb + 3 * stride);
        }
    }

    STAMP(3);
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
    STAMP(4);
    merge_if_last<BLOCK>(p, b, g, sm_flag);
    STAMP(5);
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

#ifdef VECINFER_PHASE_TIMING
extern "C" int vecinfer_debug_phase_buffer(void *buf) { return hipMemcpyToSymbol(HIP_SYMBOL(g_phase_buf), &buf, sizeof(buf)) == hipSuccess ? 0 : -4; }
#endif

bool decode_mfma_supports(const DecodeParams &p)
{
    // code rows are addressed with 32-bit byte offsets
    return p.D == kD && p.G == kG && p.dk == p.dv && (p.dk == 4 || p.dk == 2) &&
           p.N * (long long)(kD / p.dk) < (1LL << 31);
}

int launch_decode_mfma(const DecodeParams &p, hipStream_t stream)
{
    if (!decode_mfma_supports(p)) return -2;
    return p.dk == 4 ? launch_typed<4>(p, stream) : launch_typed<2>(p, stream);
}

} // namespace vecinfer
