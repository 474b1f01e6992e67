// Matrix-core decode attention with score wavefronts and value wavefronts (8-bit codes, D = 128,
// up to 4 query heads per KV head, d_k and d_v = 4 or 2): VECINFER_VARIANT_ROLES.  Same arithmetic,
// operand layouts and results as decode_mfma_kernel.h; what differs is who does what.
//
// A workgroup is 16 wavefronts, four per SIMD, in 8 pairs.  Both codebooks of the KV head live in
// LDS.  Of a pair,
//   the score wavefront streams the key codes of the pair's 64-token tiles, gathers the key
//     centroids from LDS straight into v_mfma_f32_16x16x32_f16 operands (Eq. 10 / Alg. 1 step 11),
//     runs the online softmax (steps 12-13) and leaves the tile's probabilities (fp16) and the
//     rescale factor of each head in a small ring in LDS;
//   the value wavefront streams the value codes of the same tiles, gathers the value centroids,
//     takes the probabilities from the ring and accumulates P.V on the matrix cores (step 16).
// Each carries half of the state the single-role kernel keeps in one wavefront (under 128
// registers instead of ~180), which is what lets four wavefronts share a SIMD: while one waits
// for LDS or for its codes from HBM, three others have matrix-core, vector-ALU or LDS work to
// issue.  The ring decouples the two roles by up to kRing tiles; its head / tail counters are
// the only synchronisation inside the tile loop.
//
// The two tables are staged separately: every wavefront fetches its share of the key table first,
// the score wavefronts start as soon as that table is in LDS, and the value wavefronts bring in
// the value table meanwhile (Alg. 1 step 7).
#pragma once
#include "common.h"
#include "mfma_helpers.h"

namespace vecinfer {

namespace {

constexpr int kPairs = 8;          // (score wavefront, value wavefront) pairs per workgroup
constexpr int kRing = 4;           // tiles a score wavefront may run ahead of its value wavefront

// counters of the ring, and the count of value wavefronts that have staged their table share:
// plain LDS words, written by one wavefront and polled by another
__device__ __forceinline__ unsigned flag_load(const unsigned *f)
{
    return __hip_atomic_load(f, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void flag_store(unsigned *f, unsigned v)
{
    __hip_atomic_store(f, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// waits until *f >= want; every lane reads the same word, the decision is wave-uniform
__device__ __forceinline__ void flag_wait(const unsigned *f, unsigned want)
{
    while ((unsigned)__builtin_amdgcn_readfirstlane((int)flag_load(f)) < want) __builtin_amdgcn_s_sleep(1);
}

template <int kD, int DK, int DV, bool VT>
__global__ __launch_bounds__(2 * kPairs * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))
void decode_roles_kernel(const __half *q_arg, const float *lam_arg, const __half *cb_k_arg, const __half *cb_v_arg,
                         const __half *k_new_arg, const __half *v_new_arg, unsigned hkv_g_arg, int S_, DecodeParams p)
{
    static_assert(kD == 128 && (DK == 4 || DK == 2) && (DV == 4 || DV == 2), "shapes this kernel is laid out for");
    constexpr int NW = 2 * kPairs, BLOCK = NW * 64;
    constexpr int KG = kG;                             // head slots (one MFMA pass)
    constexpr int MK = kD / DK, MV = kD / DV;          // sub-spaces: 32 or 64
    constexpr int CBK_BYTES = kCentroids * kD * 2, CBV_BYTES = kCentroids * kD * 2;
    constexpr int ENTRY_K = DK * 2, ENTRY_V = DV * 2;  // bytes per centroid: 8 or 4
    constexpr int SUB_K = kCentroids * ENTRY_K, SUB_V = kCentroids * ENTRY_V;
    constexpr int NR = kD / 32;                        // score MFMA rounds per sub-tile = P.V operands per sub-tile: 4
    constexpr int NROUND_V = MV / 16;                  // value sub-spaces per MFMA column: 2 or 4
    constexpr int KW = (MK / 4 + 3) / 4;               // key-code dwords per lane per sub-tile (MK / 4 bytes)
    constexpr int VW = NROUND_V;                       // value-code dwords per lane per sub-tile (4 tokens x NROUND_V bytes)
    constexpr int NACC = NROUND_V;                     // P.V accumulators: one per value sub-space of the lane's column
    constexpr int ROW_V = 16 * ENTRY_V;                // value table in LDS: [r][code][col], rows of 128 or 64 bytes
    constexpr int PLANE_V = kCentroids * ROW_V;
    constexpr int SLOT = 64 * 8 + 16;                  // ring slot: 4 fp16 probabilities per lane + 4 rescale factors

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *const sm_k = smem;
    unsigned char *const sm_v = smem + CBK_BYTES;
    float *const sm_qt = reinterpret_cast<float *>(smem + CBK_BYTES + CBV_BYTES);   // [KG][D]
    float *const sm_new = sm_qt + KG * kD;                                 // [2][D]: k~ and v of the new token
    float *const sm_nsc = sm_new + 2 * kD;                                 // [MK][KG]: its score shares (log2 units)
    float *const sm_nv = sm_nsc + MK * KG;                                 // [D]:    its dequantized value
    unsigned char *const sm_ring = reinterpret_cast<unsigned char *>(sm_nv + kD);   // [kPairs][kRing][SLOT]
    unsigned *const sm_head = reinterpret_cast<unsigned *>(sm_ring + kPairs * kRing * SLOT);   // [kPairs] tiles produced
    unsigned *const sm_tail = sm_head + kPairs;                            // [kPairs] tiles consumed
    float *const sm_ml = reinterpret_cast<float *>(sm_tail + kPairs);      // [kPairs][2][KG]: (m, l) of each pair at the end

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const bool v_role = wave_u >= kPairs;              // wavefronts 0 .. 7 score, 8 .. 15 accumulate
    const int pr = wave_u & (kPairs - 1);              // pair
    const int Hkv_ = (int)(hkv_g_arg & 0xffffffu), G_ = (int)(hkv_g_arg >> 24);   // = p.Hkv, p.G
    // Workgroups are dealt to the 8 XCDs round-robin in linear order, so the KV head varies
    // fastest: with 8 KV heads every XCD serves one head and its L2 fetches one codebook set.
    const int lin = blockIdx.x + S_ * blockIdx.y;
    const int g = lin % Hkv_, s = lin / Hkv_, b = blockIdx.z;
    const int col = lane & 15;       // MFMA row (A) / column (B, D) index of this lane
    const int kg = lane >> 4;        // k-group (A, B) / row group (D) of this lane
    const size_t bg = (size_t)b * Hkv_ + g;

    // ---- first requests, from the preloaded leading arguments only.  Up to the role split below every
    // wavefront runs the same instruction stream with no branch between a request and its use: the
    // compiler then knows exactly how many younger requests may stay in flight at each use (loads
    // return in order), where requests issued under a condition make it wait for all of them.
    // The small input rows first (kept as raw bits: no conversion makes the wavefront wait for data
    // it has only just asked for): score wavefront hh < G takes query head hh, the last two value
    // wavefronts the key and the value row of a fused new token; the others read a row that exists
    // anyway and ignore it.
    auto raw16 = [](const __half *src) -> unsigned { return *reinterpret_cast<const unsigned short *>(src); };
    auto widen = [](unsigned bits) { return (float)__builtin_bit_cast(_Float16, (unsigned short)bits); };
    const bool q_role = wave_u < KG && wave_u < G_;
    const __half *const qsrc = q_arg + (((size_t)b * Hkv_ + g) * G_ + (q_role ? wave_u : 0)) * kD;
    const __half *const nsrc = (wave_u >= NW - 2 && k_new_arg) ? (wave_u == NW - 1 ? v_new_arg : k_new_arg) + bg * kD : qsrc;
    const unsigned xh0 = raw16(nsrc + lane), xh1 = raw16(nsrc + 64 + lane);
    const float ql0 = lam_arg[(size_t)g * kD + lane], ql1 = lam_arg[(size_t)g * kD + 64 + lane];
    asm volatile("" ::: "memory");                 // keep these loads ahead of the big ones below
    // .. then both tables, as items of 1 KB (one wavefront instruction each), 4 + 4 per wavefront
    constexpr int kStage = CBK_BYTES / 1024;           // 64 items per table
    constexpr int kItems = kStage / NW;
    constexpr int CPL = 16 / ENTRY_V;                  // codes per 16-byte load of the value codebook
    static_assert(NROUND_V * (kCentroids / (4 * CPL)) == kStage, "value items: (code group, r)");
    const int vq = lane >> 4, vcol = lane & 15;
    uintx4 kreg[kItems], vreg[kItems];
    {
        const unsigned char *srck = reinterpret_cast<const unsigned char *>(cb_k_arg) + (size_t)g * CBK_BYTES;
        const unsigned char *srcv = reinterpret_cast<const unsigned char *>(cb_v_arg) + (size_t)g * CBV_BYTES;
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            kreg[j] = *reinterpret_cast<const uintx4 *>(srck + (wave_u + NW * j) * 1024 + lane * 16);
        // the value table is transposed on the way into LDS ([r][code][col], see below): a lane loads
        // 16 bytes = CPL consecutive codes of sub-space NROUND_V vcol + r; the four 16-lane groups take
        // adjacent pieces.  Item `it` serves r = it % NROUND_V and the 4 CPL codes of code group it / NROUND_V.
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            const int it = wave_u + NW * j;
            const int r = it % NROUND_V, code = (it / NROUND_V) * 4 * CPL + vq * CPL;
            vreg[j] = *reinterpret_cast<const uintx4 *>(srcv + (NROUND_V * vcol + r) * SUB_V + code * ENTRY_V);
        }
    }
    // every other argument the prologue uses, in one batch of scalar loads
#define VECINFER_PIN(x) asm volatile("" ::"s"(x))
    VECINFER_PIN(p.seq_lens); VECINFER_PIN(p.N); VECINFER_PIN(p.n_cap); VECINFER_PIN(p.k_idx); VECINFER_PIN(p.v_idx);
#undef VECINFER_PIN

    // With a fused append the new token is the sequence's last one: its codes are produced in this
    // launch, the tile loop covers the len - 1 older tokens, workgroup s encodes sub-spaces
    // s, s + S, .. of the new token's key and value.
    const long long len = seq_len_of(p, b);
    const bool fused = k_new_arg != nullptr && len > 0;
    const bool has_new = fused && (s < MK || s < MV);
    long long n0, n1;
    split_range(fused ? len - 1 : len, S_, s, kTile, n0, n1);
    if (n0 >= n1 && !has_new) {                        // empty split: neutral partial
        for (int e = tid; e < G_ * kD; e += BLOCK) p.part_o[(bg * S_ + s) * G_ * kD + e] = 0.f;
        if (tid < G_) {
            p.part_m[(bg * S_ + s) * G_ + tid] = -INFINITY;
            p.part_l[(bg * S_ + s) * G_ + tid] = 0.f;
        }
        finish_split<BLOCK>(p, b, g);
        return;
    }

    // ---- per-lane constants
    const int t0 = col & 3;                              // channel-in-sub-vector this A row serves
    const unsigned lds_base = (unsigned)(uintptr_t)smem;          // LDS offset of the dynamic segment
    const unsigned lds_k = lds_base + (unsigned)(kg * (MK / 4) * SUB_K);
    const unsigned lds_v = lds_base + (unsigned)CBK_BYTES + (unsigned)(col * ENTRY_V);
    const uint8_t *krow = p.k_idx + bg * p.n_cap * MK;
    const uint8_t *vrow = p.v_idx + bg * p.n_cap * MV;
    const long long last = n1 - 1;
    // token owned by A-row i of sub-tile st: base + 16 st + 4 (i % 4) + i / 4, so that D-register v
    // of row group rg is token base + 16 st + 4 v + rg
    const int krow_tok = 4 * (col & 3) + (col >> 2);
    // The code rows of (b, g) are read through buffer descriptors whose extent ends at the split's
    // last token: loads past the end return 0 (a valid code) instead of needing a clamp.  The host
    // checks N * M < 2^31.
    const __amdgpu_buffer_rsrc_t rsrc_k =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(krow), 0, (int)((unsigned)n1 * MK), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_v = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(vrow), 0, (int)((unsigned)(VT ? (n1 + 63) / 64 * 64 : n1) * MV), 0x00020000);
    const unsigned koff_lane = (unsigned)(krow_tok * MK + kg * (MK / 4));
    const unsigned voff_lane = VT ? (unsigned)(lane * 16) : (unsigned)(kg * MV + col * NROUND_V);

    // codes of one 64-token tile as this lane needs them
    struct KCodes { unsigned c[4][KW]; };                // the key-code bytes of the lane's A row, per sub-tile
    struct VCodes { unsigned c[4][VW]; };                // the value-code bytes of the 4 tokens of its k-group
    auto load_codes_k = [&](KCodes &cd, long long tb) {
        const unsigned ko = (unsigned)tb * MK + koff_lane;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            if constexpr (MK / 4 == 8) {
                const uintx2 w = __builtin_amdgcn_raw_buffer_load_b64(rsrc_k, ko + 16 * st * MK, 0, kStreamPolicy);
                cd.c[st][0] = w[0]; cd.c[st][1] = w[1];
            } else {
                const uintx4 w = __builtin_amdgcn_raw_buffer_load_b128(rsrc_k, ko + 16 * st * MK, 0, kStreamPolicy);
                cd.c[st][0] = w[0]; cd.c[st][1] = w[1]; cd.c[st][2] = w[2]; cd.c[st][3] = w[3];
            }
        }
    };
    auto load_codes_v = [&](VCodes &cd, long long tb) {
        const unsigned vo = (unsigned)tb * MV + voff_lane;
        if constexpr (VT) {
            // the lane's 16 NROUND_V bytes of the tile, in the order (sub-tile, token v, round r), 16
            // from each of the block's NROUND_V slabs of 1 KB
            unsigned w[4 * NROUND_V];
#pragma unroll
            for (int j = 0; j < NROUND_V; ++j) {
                const uintx4 x = __builtin_amdgcn_raw_buffer_load_b128(rsrc_v, vo + 1024 * j, 0, kStreamPolicy);
                w[4 * j] = x[0]; w[4 * j + 1] = x[1]; w[4 * j + 2] = x[2]; w[4 * j + 3] = x[3];
            }
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int j = 0; j < NROUND_V; ++j) cd.c[st][j] = w[st * NROUND_V + j];
            return;
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            // NROUND_V bytes (sub-spaces NROUND_V col ..) of each of the tokens 4 v + kg, packed
            // token after token: byte v * NROUND_V + r
            if constexpr (NROUND_V == 2) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    ushortx2 t;
                    t[0] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rsrc_v, vo + (16 * st + 8 * u) * MV, 0, kStreamPolicy);
                    t[1] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rsrc_v, vo + (16 * st + 8 * u + 4) * MV, 0, kStreamPolicy);
                    cd.c[st][u] = __builtin_bit_cast(unsigned, t);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    cd.c[st][v] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_v, vo + (16 * st + 4 * v) * MV, 0, kStreamPolicy);
            }
        }
    };
    // The pair's k-th tile.  The wavefronts of a SIMD do not run at the same speed: those launched
    // first (pairs 0 .. 3) win the issue arbitration and get through a tile about a fifth sooner,
    // so an even deal leaves them idle at the end of a long split.  Tiles are therefore dealt in
    // periods of kFull + 1 rounds: kFull rounds to every pair in turn and one round to the first
    // half only, two tiles each ((kFull + 2) : kFull).  Short splits see the plain round-robin.
    // The deal is static, so results are reproducible.
    auto tile_base = [&](int k) -> long long {
        constexpr int kFull = 5, kPeriod = (kFull + 1) * kPairs;
        int per, off;
        if (pr < kPairs / 2) {
            per = k / (kFull + 2);
            const int i = k % (kFull + 2);
            off = i < kFull ? i * kPairs + pr : kFull * kPairs + (i - kFull) * (kPairs / 2) + pr;
        } else {
            per = k / kFull;
            off = (k % kFull) * kPairs + pr;
        }
        return n0 + ((long long)per * kPeriod + off) * kTile;
    };
    // second half of the staging, registers -> LDS.  Keys keep the [m][code] order of memory.  Values
    // are stored [r][code][col] with sub-space m = NROUND_V col + r: LDS serves a gather 16 lanes at a
    // time, and the 16 lanes of such a group read the same r and 16 different col, so with the 16
    // entries of a code in one ROW_V-byte row they fall on disjoint banks whatever their codes are.
    auto stage_tables = [&]() {
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            *reinterpret_cast<uintx4 *>(sm_k + (wave_u + NW * j) * 1024 + lane * 16) = kreg[j];
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            const int it = wave_u + NW * j;
            const int r = it % NROUND_V, code = (it / NROUND_V) * 4 * CPL + vq * CPL;
#pragma unroll
            for (int e = 0; e < CPL; ++e) {
                unsigned char *const d = sm_v + r * PLANE_V + (code + e) * ROW_V + vcol * ENTRY_V;
                if constexpr (DV == 4)
                    *reinterpret_cast<uintx2 *>(d) = uintx2{vreg[j][2 * e], vreg[j][2 * e + 1]};
                else
                    *reinterpret_cast<unsigned *>(d) = vreg[j][e];
            }
        }
    };

    const float fold = kLog2e / (float)kD;              // (1/sqrt D of H_D) (1/sqrt D of the score) log2 e
    auto lds_addr = [&](unsigned w, int k, unsigned base) -> unsigned {        // code byte k of w: code * ENTRY_K + base
        return __builtin_amdgcn_udot4(w, (unsigned)ENTRY_K << (8 * k), base, false);
    };
    auto lds_addr_v = [&](unsigned w, int k, unsigned base) -> unsigned {      // code * ROW_V + base
        if constexpr (ROW_V > 255)                  // the multiplier of v_dot4 is one byte: halve, then double
            return __builtin_amdgcn_udot4(w, (unsigned)(ROW_V / 2) << (8 * k), base >> 1, false) << 1;
        else
            return __builtin_amdgcn_udot4(w, (unsigned)ROW_V << (8 * k), base, false);
    };
    unsigned char *const ring = sm_ring + pr * kRing * SLOT;
    // what a pair leaves for the merge at the end of the split: the accumulators [KG][D] in the first
    // 2 KB of its own ring (free by then), (m, l) in sm_ml
    float *const pair_o = reinterpret_cast<float *>(ring);
    static_assert(kRing * SLOT >= (int)sizeof(float) * KG * kD, "a pair's accumulators fit in its ring");

    if (!v_role) {
        // =============================== score wavefront ===============================
        float m_run = -INFINITY;      // running max of head col / 4 (log2 units), same in all its lanes
        float l_part = 0.f;           // this lane's share of the running sum
        // the first two tiles' key codes start their trip from HBM now, behind the tables
        KCodes ka_c, kb_c;
        load_codes_k(ka_c, tile_base(0));
        load_codes_k(kb_c, tile_base(1));
        // q~ = (q * lambda) H_D for the heads of the group (un-normalised butterflies): wavefront hh
        // transforms head hh in registers, a lane holding channels `lane` and `lane + 64`
        if (wave_u < KG && wave_u >= G_) {
            sm_qt[wave_u * kD + lane] = 0.f;            // spare head slot: a zero query, never written out
            sm_qt[wave_u * kD + 64 + lane] = 0.f;
        } else if (wave_u < KG) {
            float x0 = widen(xh0) * ql0, x1 = widen(xh1) * ql1;
            {
                const float a = x0 + x1, d = x0 - x1;
                x0 = a;
                x1 = d;
            }
#pragma unroll
            for (int st = 1; st < 64; st <<= 1) {
                const float o0 = __shfl_xor(x0, st), o1 = __shfl_xor(x1, st);
                const bool up = (lane & st) != 0;
                x0 = up ? (o0 - x0) : (x0 + o0);
                x1 = up ? (o1 - x1) : (x1 + o1);
            }
            sm_qt[wave_u * kD + lane] = x0;
            sm_qt[wave_u * kD + 64 + lane] = x1;
        } else if (wave_u == KG && lane < 2 * kPairs) {
            sm_head[lane] = 0u;                          // ring counters
        }
        stage_tables();
        __syncthreads();                                // tables, q~, new token, counters
        // B operands of the score MFMAs: q~_h[32 kg + 8 r .. + 8); columns with t0 < 2 take the fp16
        // high part, columns with t0 >= 2 the low part (x - float(hi)); one DPP add across the quad
        // recombines them, so the scores are fp32-accurate.
        half8 bq[NR];
        {
            const int hh = col >> 2;
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = sm_qt[hh * kD + (kD / 4) * kg + 8 * r + e] * fold;
                    const _Float16 hi = (_Float16)x;
                    const _Float16 lo = (_Float16)(x - (float)hi);
                    bq[r][e] = (col & 2) ? lo : hi;
                }
        }
        // A operand of sub-tile st, round r: the centroids of 8 / d_k consecutive key sub-spaces of
        // the lane's token (pure LDS gathers)
        auto gather_k = [&](const KCodes &cd, int st, int r) -> half8 {
            if constexpr (DK == 4) {
                const unsigned w = cd.c[st][r >> 1];
                const int k0 = 2 * (r & 1);
                const uint2 x0 = lds_load_b64(lds_addr(w, k0, lds_k) + (2 * r) * SUB_K);
                const uint2 x1 = lds_load_b64(lds_addr(w, k0 + 1, lds_k) + (2 * r + 1) * SUB_K);
                return as_half8(x0.x, x0.y, x1.x, x1.y);
            } else {
                const unsigned w = cd.c[st][r];
                unsigned x[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) x[q] = lds_load_b32(lds_addr(w, q, lds_k) + (4 * r + q) * SUB_K);
                return as_half8(x[0], x[1], x[2], x[3]);
            }
        };
        const floatx4 kZero4 = {0.f, 0.f, 0.f, 0.f};
        half8 oa[NR], ob[NR];            // operands of the sub-tile at hand / of the one after it
        unsigned produced = 0;           // tiles this wavefront has put into the ring
        unsigned is_t[4];                // is_t[i] = all ones iff t0 == i
#pragma unroll
        for (int i = 0; i < 4; ++i) is_t[i] = t0 == i ? 0xffffffffu : 0u;
        auto bfi = [](unsigned m, unsigned a, unsigned b) -> unsigned { return (m & a) | (~m & b); };

        // One tile: four sub-tiles, each NR MFMAs on operands gathered while the sub-tile before ran;
        // the first sub-tile of the next tile is gathered under the last one.  The key-code
        // registers are refilled (two tiles ahead) right after their last gather.
        auto k_tile = [&](KCodes &cd, const KCodes &next, long long tb, long long tb_refill) {
            // Scores of sub-tile st: NR MFMAs.  The four lanes of a quad (same head, t0 = 0 .. 3) then
            // hold the high-part scores (t0 < 2) or the low-part scores (t0 >= 2) of the 16 tokens of
            // their row group; lane t0 keeps sub-tile t0's four (`mine`), and the copy of sub-tile
            // t0 ^ 2 that the lane two further on, which holds the other part, needs (`theirs`).
            // Branch-free picks with bit masks (v_bfi_b32 / v_cndmask).
            unsigned mine[4], theirs[4];
            auto scores = [&](auto st_c, const half8 *ops) {
                constexpr int st = decltype(st_c)::value;
                floatx4 acc = MFMA16(ops[0], bq[0], kZero4, 0, 0, 0);
#pragma unroll
                for (int r = 1; r < NR; ++r) acc = MFMA16(ops[r], bq[r], acc, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const unsigned x = __float_as_uint(acc[v]);
                    mine[v] = st == 0 ? x : bfi(is_t[st], x, mine[v]);
                    theirs[v] = st == 0 ? x : bfi(is_t[st ^ 2], x, theirs[v]);
                }
            };
#pragma unroll
            for (int r = 0; r < NR; ++r) ob[r] = gather_k(cd, 1, r);
            scores(std::integral_constant<int, 0>{}, oa);
#pragma unroll
            for (int r = 0; r < NR; ++r) oa[r] = gather_k(cd, 2, r);
            scores(std::integral_constant<int, 1>{}, ob);
#pragma unroll
            for (int r = 0; r < NR; ++r) ob[r] = gather_k(cd, 3, r);
            load_codes_k(cd, tb_refill);
            scores(std::integral_constant<int, 2>{}, oa);
#pragma unroll
            for (int r = 0; r < NR; ++r) oa[r] = gather_k(next, 0, r);
            scores(std::integral_constant<int, 3>{}, ob);

            // online softmax of this wavefront (Alg. 1 steps 12-13)
            float sc[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) sc[v] = __uint_as_float(mine[v]) + quad_xor<2>(__uint_as_float(theirs[v]));
            if (tb + kTile > n1) {                  // tail tile: tokens past the end get p = 0
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (tb + 16 * t0 + 4 * v + kg > last) sc[v] = -INFINITY;
            }
            float tmax = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
            tmax = fmaxf(tmax, quad_xor<1>(tmax));
            tmax = fmaxf(tmax, quad_xor<2>(tmax));
            tmax = rows_max(tmax);
            const float m_new = fmaxf(m_run, tmax);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);          // 0 on the first tile, 1 when the max stands
            m_run = m_new;
            float pr4[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) pr4[v] = __builtin_amdgcn_exp2f(sc[v] - m_new);
            l_part = l_part * alpha + ((pr4[0] + pr4[1]) + (pr4[2] + pr4[3]));
            typedef _Float16 half2v __attribute__((ext_vector_type(2)));
            const half2v h01 = {(_Float16)pr4[0], (_Float16)pr4[1]}, h23 = {(_Float16)pr4[2], (_Float16)pr4[3]};
            // hand the tile over: wait for the slot to be free, write, publish
            if (produced >= (unsigned)kRing) flag_wait(&sm_tail[pr], produced - kRing + 1);
            unsigned char *const slot = ring + (produced % kRing) * SLOT;
            *reinterpret_cast<uintx2 *>(slot + lane * 8) =
                uintx2{__builtin_bit_cast(unsigned, h01), __builtin_bit_cast(unsigned, h23)};
            if ((lane & 0x33) == 0) *reinterpret_cast<float *>(slot + 512 + col) = alpha;   // lanes 0, 4, 8, 12: heads 0 .. 3
            ++produced;
            flag_store(&sm_head[pr], produced);
        };
#pragma unroll
        for (int r = 0; r < NR; ++r) oa[r] = gather_k(ka_c, 0, r);
        long long ta = tile_base(0), tb = tile_base(1);
        for (int k = 2; ta < n1; k += 2) {
            const long long tc = tile_base(k), td = tile_base(k + 1);
            k_tile(ka_c, kb_c, ta, tc);
            if (tb < n1) k_tile(kb_c, ka_c, tb, td);
            ta = tc;
            tb = td;
        }
        float l_head = l_part + quad_xor<1>(l_part);
        l_head += quad_xor<2>(l_head);
        l_head += __shfl_xor(l_head, 16);
        l_head += __shfl_xor(l_head, 32);
        if (kg == 0 && (col & 3) == 0) {
            sm_ml[(pr * 2 + 0) * KG + (col >> 2)] = m_run;
            sm_ml[(pr * 2 + 1) * KG + (col >> 2)] = l_head;
        }
    } else {
        // =============================== value wavefront ===============================
        floatx4 acc_o[NACC];          // P.V accumulators
#pragma unroll
        for (int r = 0; r < NACC; ++r) acc_o[r] = floatx4{0.f, 0.f, 0.f, 0.f};
        // the first two tiles' value codes start their trip from HBM now, behind the tables
        VCodes va_c, vb_c;
        load_codes_v(va_c, tile_base(0));
        load_codes_v(vb_c, tile_base(1));
        // the new token's key and value (fused append): the last two wavefronts
        if (has_new && wave_u == NW - 2) {
            // k~ = (k / lambda) H_D of the new token (Eq. 9), operation for operation what the
            // cache-fill kernels compute, so that the fused step writes the codes a separate append would
            float x0 = widen(xh0) / ql0, x1 = widen(xh1) / ql1;
#pragma unroll
            for (int st = 1; st < 64; st <<= 1) {
                const float o0 = __shfl_xor(x0, st), o1 = __shfl_xor(x1, st);
                const bool up = (lane & st) != 0;
                x0 = up ? (o0 - x0) : (x0 + o0);
                x1 = up ? (o1 - x1) : (x1 + o1);
            }
            const float hs = 1.0f / sqrtf((float)kD);
            sm_new[lane] = (x0 + x1) * hs;
            sm_new[64 + lane] = (x0 - x1) * hs;
        } else if (has_new && wave_u == NW - 1) {
            sm_new[kD + lane] = widen(xh0);
            sm_new[kD + 64 + lane] = widen(xh1);
        }
        stage_tables();
        __syncthreads();                                // tables, q~, new token, counters
        // selectors of v_perm_b32 that place a probability (fp16, low or high half of a packed pair)
        // in the one k-slot of the A operand whose channel-in-sub-vector is t0, zero elsewhere
        constexpr unsigned kZ = 0x0c0c0c0cu;
        const unsigned lo_a = t0 == 0 ? 0x0c0c0100u : (t0 == 1 ? 0x01000c0cu : kZ);   // even token of the pair, slots 0-1
        const unsigned hi_a = t0 == 0 ? 0x0c0c0302u : (t0 == 1 ? 0x03020c0cu : kZ);   // odd token, slots 0-1
        const unsigned lo_b = t0 == 2 ? 0x0c0c0100u : (t0 == 3 ? 0x01000c0cu : kZ);   // even token, slots 2-3 (d = 4)
        const unsigned hi_b = t0 == 2 ? 0x0c0c0302u : (t0 == 3 ? 0x03020c0cu : kZ);   // odd token, slots 2-3
        // B operand q (0 .. NR-1) of the P.V MFMAs of sub-tile st; the code of (token v of the
        // k-group, round r) is byte v * NROUND_V + r of the packed value codes.  d = 4: q = u * 2 + r:
        // centroids of sub-space 2 col + r for tokens 2u, 2u + 1.  d = 2: q = r: centroids of
        // sub-space 4 col + r for the 4 tokens.
        auto gather_v = [&](const VCodes &cd, int st, int q) -> half8 {
            if constexpr (DV == 4) {
                const int u = q / NROUND_V, r = q % NROUND_V;
                const int b0 = 2 * u * NROUND_V + r, b1 = (2 * u + 1) * NROUND_V + r;
                const uint2 x0 = lds_load_b64(lds_addr_v(cd.c[st][b0 >> 2], b0 & 3, lds_v) + r * PLANE_V);
                const uint2 x1 = lds_load_b64(lds_addr_v(cd.c[st][b1 >> 2], b1 & 3, lds_v) + r * PLANE_V);
                return as_half8(x0.x, x0.y, x1.x, x1.y);
            } else {
                unsigned x[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int bi = v * NROUND_V + q;
                    x[v] = lds_load_b32(lds_addr_v(cd.c[st][bi >> 2], bi & 3, lds_v) + q * PLANE_V);
                }
                return as_half8(x[0], x[1], x[2], x[3]);
            }
        };
        unsigned p01 = 0, p23 = 0;       // this lane's slot word: probabilities of tokens 4 v + kg of sub-tile t0
        // o += P . VQ^-1(V_q) for sub-tile st (step 16): p of sub-tile st lives in quad lane st
        auto pv = [&](auto st_c, const half8 *vops) {
            constexpr int st = decltype(st_c)::value;
            const unsigned b01 = quad_bcast<st>(p01), b23 = quad_bcast<st>(p23);
            if constexpr (DV == 4) {
                const half8 a0 = as_half8(__builtin_amdgcn_perm(0u, b01, lo_a), __builtin_amdgcn_perm(0u, b01, lo_b),
                                          __builtin_amdgcn_perm(0u, b01, hi_a), __builtin_amdgcn_perm(0u, b01, hi_b));
                const half8 a1 = as_half8(__builtin_amdgcn_perm(0u, b23, lo_a), __builtin_amdgcn_perm(0u, b23, lo_b),
                                          __builtin_amdgcn_perm(0u, b23, hi_a), __builtin_amdgcn_perm(0u, b23, hi_b));
#pragma unroll
                for (int r = 0; r < NROUND_V; ++r) acc_o[r] = MFMA16(a0, vops[r], acc_o[r], 0, 0, 0);
#pragma unroll
                for (int r = 0; r < NROUND_V; ++r) acc_o[r] = MFMA16(a1, vops[NROUND_V + r], acc_o[r], 0, 0, 0);
            } else {
                const half8 a = as_half8(__builtin_amdgcn_perm(0u, b01, lo_a), __builtin_amdgcn_perm(0u, b01, hi_a),
                                         __builtin_amdgcn_perm(0u, b23, lo_a), __builtin_amdgcn_perm(0u, b23, hi_a));
#pragma unroll
                for (int r = 0; r < NROUND_V; ++r) acc_o[r] = MFMA16(a, vops[r], acc_o[r], 0, 0, 0);
            }
        };
        half8 oa[NR], ob[NR];
        unsigned consumed = 0;
        auto v_tile = [&](VCodes &cd, const VCodes &next, long long tb_refill) {
#pragma unroll
            for (int q = 0; q < NR; ++q) ob[q] = gather_v(cd, 1, q);
            // take the tile's probabilities and rescale factors from the ring
            flag_wait(&sm_head[pr], consumed + 1);
            const unsigned char *const slot = ring + (consumed % kRing) * SLOT;
            const uintx2 w = *reinterpret_cast<const uintx2 *>(slot + lane * 8);
            const float alpha = *reinterpret_cast<const float *>(slot + 512 + 4 * kg);   // rows 4 kg .. of D: head kg
            p01 = w[0];
            p23 = w[1];
            ++consumed;
            flag_store(&sm_tail[pr], consumed);         // (a release: the two reads above have returned)
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int r = 0; r < NACC; ++r) acc_o[r] *= alpha;
            }
            pv(std::integral_constant<int, 0>{}, oa);
#pragma unroll
            for (int q = 0; q < NR; ++q) oa[q] = gather_v(cd, 2, q);
            pv(std::integral_constant<int, 1>{}, ob);
#pragma unroll
            for (int q = 0; q < NR; ++q) ob[q] = gather_v(cd, 3, q);
            load_codes_v(cd, tb_refill);
            pv(std::integral_constant<int, 2>{}, oa);
#pragma unroll
            for (int q = 0; q < NR; ++q) oa[q] = gather_v(next, 0, q);
            pv(std::integral_constant<int, 3>{}, ob);
        };
        // The consumer of a pair runs at a raised priority: it can never starve the producer (it
        // sleeps while the ring is empty), and otherwise the wavefronts launched first - the score
        // wavefronts - win the issue arbitration, the value wavefronts fall kRing tiles behind and
        // finish the split alone, two to a SIMD.
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int q = 0; q < NR; ++q) oa[q] = gather_v(va_c, 0, q);
        long long ta = tile_base(0), tb = tile_base(1);
        for (int k = 2; ta < n1; k += 2) {
            const long long tc = tile_base(k), td = tile_base(k + 1);
            v_tile(va_c, vb_c, tc);
            if (tb < n1) v_tile(vb_c, va_c, td);
            ta = tc;
            tb = td;
        }
        // acc_o[r] register v of lane (col, kg): head kg, channel DV * (NACC * col + r) + v
#pragma unroll
        for (int r = 0; r < NACC; ++r)
#pragma unroll
            for (int v = 0; v < DV; ++v) pair_o[kg * kD + DV * (NACC * col + r) + v] = acc_o[r][v];
    }

    // ---- fused append: this workgroup's sub-spaces of the new token, dealt to the wavefronts as
    // (sub-space, key | value) items behind their tiles.  Eq. 2 by exhaustive search over the table in
    // LDS: a lane scans centroids lane, lane + 64, ..; squared distances summed in channel order in
    // fp32; the lowest index among the centroids at minimum distance wins.  The key item also
    // leaves the new token's score share of its sub-space for the heads, the value item the
    // dequantized channels, for the merge kernel.
    if (has_new) {
        const long long pos = len - 1;
        auto new_items = [&](auto kv_c, auto nb_c, int i0) {
            constexpr int kv = decltype(kv_c)::value;          // 0: key sub-spaces, 1: value sub-spaces
            constexpr int NB = decltype(nb_c)::value;          // items taken at a time
            constexpr int DS = kv == 0 ? DK : DV, EN = 2 * DS, MX = kv == 0 ? MK : MV;
            constexpr int stride = kv == 0 ? ENTRY_K : ROW_V;  // entry c of a sub-space sits at tab + c * stride
            int m[NB];
            bool ok[NB];
            const unsigned char *tab[NB];
            float best[NB];
            unsigned arg[NB];
#pragma unroll
            for (int b4 = 0; b4 < NB; ++b4) {
                const int mm = s + (i0 + NW * b4) * S_;
                ok[b4] = mm < MX;
                m[b4] = ok[b4] ? mm : 0;                        // a surplus slot redoes sub-space 0 and writes nothing
                tab[b4] = kv == 0 ? sm_k + m[b4] * SUB_K
                                  : sm_v + (m[b4] % NROUND_V) * PLANE_V + (m[b4] / NROUND_V) * ENTRY_V;
                best[b4] = INFINITY;
                arg[b4] = 0;
            }
#pragma unroll
            for (int b4 = 0; b4 < NB; ++b4) {
                float x[DS];
#pragma unroll
                for (int jj = 0; jj < DS; ++jj) x[jj] = sm_new[kv * kD + m[b4] * DS + jj];
#pragma unroll
                for (int i = 0; i < kCentroids / 64; ++i) {
                    const unsigned c = lane + 64 * i;
                    _Float16 cen[DS];
                    __builtin_memcpy(cen, tab[b4] + c * stride, EN);
                    float dist = 0.f;
#pragma unroll
                    for (int jj = 0; jj < DS; ++jj) {
                        const float tdiff = x[jj] - (float)cen[jj];
                        dist = fmaf(tdiff, tdiff, dist);
                    }
                    if (dist < best[b4]) {
                        best[b4] = dist;
                        arg[b4] = c;
                    }
                }
            }
            unsigned code[NB];
#pragma unroll
            for (int b4 = 0; b4 < NB; ++b4) {
                // a non-negative fp32 orders like its bit pattern
                const unsigned dmin = wave_umin(__float_as_uint(best[b4]));
                code[b4] = wave_umin(__float_as_uint(best[b4]) == dmin ? arg[b4] : 0xffffffffu);
            }
#pragma unroll
            for (int b4 = 0; b4 < NB; ++b4) {
                if (!ok[b4]) continue;                          // wave-uniform
                _Float16 win[DS];
                __builtin_memcpy(win, tab[b4] + code[b4] * stride, EN);
                if (kv == 0) {
                    if (lane == 0) p.k_idx_w[((size_t)bg * p.n_cap + pos) * MK + m[b4]] = (uint8_t)code[b4];
                    if (lane < G_) {
                        float sc = 0.f;
#pragma unroll
                        for (int jj = 0; jj < DS; ++jj)
                            sc = fmaf(sm_qt[lane * kD + m[b4] * DS + jj] * fold, (float)win[jj], sc);
                        p.new_sc[((size_t)bg * MK + m[b4]) * G_ + lane] = sc;
                        sm_nsc[m[b4] * KG + lane] = sc;
                    }
                } else {
                    if (lane == 0)
                        p.v_idx_w[(size_t)bg * p.n_cap * MV + (VT ? v_tiled_offset(pos, m[b4], MV) : (size_t)pos * MV + m[b4])] =
                            (uint8_t)code[b4];
                    float mine = (float)win[0];
#pragma unroll
                    for (int jj = 1; jj < DS; ++jj) mine = lane == jj ? (float)win[jj] : mine;
                    if (lane < DS) {
                        p.new_v[(size_t)bg * kD + m[b4] * DS + lane] = mine;
                        sm_nv[m[b4] * DS + lane] = mine;
                    }
                }
            }
        };
        // key item i (sub-space s + i S) goes to wavefront i % NW, value item i to wavefront
        // (i + 1) % NW; a wavefront with one item of a kind (the usual case: at least as many
        // splits as sub-spaces) takes it alone, otherwise four at a time
        auto items8 = [&](auto kv_c) {
            constexpr int kv = decltype(kv_c)::value, MX = kv == 0 ? MK : MV;
            const int first = kv == 0 ? wave_u : (wave_u + NW - 1) % NW;
            if (s + (first + NW) * S_ < MX) {
                for (int i0 = first; s + i0 * S_ < MX; i0 += 4 * NW) new_items(kv_c, std::integral_constant<int, 4>{}, i0);
            } else if (s + first * S_ < MX) {
                new_items(kv_c, std::integral_constant<int, 1>{}, first);
            }
        };
        items8(std::integral_constant<int, 0>{});
        items8(std::integral_constant<int, 1>{});
    }

    // ---- merge the pairs of this split: the score wavefront of a pair left (m, l), the value
    // wavefront the accumulators
    __syncthreads();
    if (tid < G_ * kD) {
        const int e = tid, hh = e / kD, c = e % kD;
        float mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < kPairs; ++w) mx = fmaxf(mx, sm_ml[(w * 2 + 0) * KG + hh]);
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kPairs; ++w) {
            const float mw = sm_ml[(w * 2 + 0) * KG + hh];
            const float f = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - mx) : 0.f;
            o += f * reinterpret_cast<const float *>(sm_ring + w * kRing * SLOT)[e];
            l += f * sm_ml[(w * 2 + 1) * KG + hh];
        }
        if (S_ == 1 && !p.k_res) {
            // the workgroup holds the whole answer (a single split also encoded every sub-space of
            // a fused new token): fold the new token in and write the output rows
            if (has_new) {
                float s_new = 0.f;
                for (int m = 0; m < MK; ++m) s_new += sm_nsc[m * KG + hh];
                const float mt = fmaxf(mx, s_new);
                const float f = __builtin_amdgcn_exp2f(mx - mt), wgt = __builtin_amdgcn_exp2f(s_new - mt);
                o = f * o + wgt * sm_nv[c];
                l = f * l + wgt;
                mx = mt;
            }
            const size_t row = ((size_t)b * Hkv_ + g) * G_ + hh;
            p.out[row * kD + c] = __float2half(l > 0.f ? o / l : 0.f);
            if (c == 0 && p.lse) p.lse[row] = l > 0.f ? (mx + log2f(l)) * kLn2 : -INFINITY;
        } else {
            const size_t pi = (bg * S_ + s) * G_;
            p.part_o[pi * kD + e] = o;
            if (c == 0) {
                p.part_m[pi + hh] = mx;
                p.part_l[pi + hh] = l;
            }
        }
    }
}

template <int kD, int DK, int DV, bool VT>
int launch_roles(const DecodeParams &p, hipStream_t stream)
{
    constexpr size_t tables = 2 * (size_t)kCentroids * kD * 2;
    constexpr size_t smem = tables + sizeof(float) * ((kG + 3) * kD + (kD / DK) * kG) + kPairs * kRing * (64 * 8 + 16) +
                            sizeof(unsigned) * 2 * kPairs + sizeof(float) * 2 * kPairs * kG + 16;
    static_assert(smem <= 160 * 1024, "one workgroup per CU: tables, scratch and rings within 160 KB of LDS");
    // once per process and instantiation (function-local static: initialised thread-safely)
    static const bool configured =
        hipFuncSetAttribute(reinterpret_cast<const void *>(decode_roles_kernel<kD, DK, DV, VT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    if (!configured) return -4;
    dim3 grid(p.S, p.Hkv, p.B);
    hipLaunchKernelGGL((decode_roles_kernel<kD, DK, DV, VT>), grid, dim3(2 * kPairs * 64), smem, stream, p.q, p.lam, p.cb_k,
                       p.cb_v, p.k_new, p.v_new, (unsigned)p.Hkv | (unsigned)p.G << 24, p.S, p);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

} // namespace

} // namespace vecinfer
