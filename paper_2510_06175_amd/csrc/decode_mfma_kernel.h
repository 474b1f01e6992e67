// Kernel template of the matrix-core decode attention; included by the translation units that
// instantiate it (8-bit codes: decode_mfma.hip; 8-bit codes with the value codes in the tiled
// layout: decode_mfma_tiled.hip; 10- and 12-bit codes: decode_mfma_wide.hip).
//
// Matrix-core decode attention for gfx950: head dim D = 128 or 64, G = 1 .. 8 query heads
// per KV head (more than 4: two passes of 4 over the same gathered operands), sub-vector dims d_k, d_v = 8,
// 4 or 2, chosen separately for keys and values (M = D / d = 8 .. 64 sub-spaces), 8-bit codes
// with one table per sub-space, or (D = 128, d = 8 or 4) 10- / 12-bit codes packed bit by bit,
// with one table of 2^b centroids shared by the sub-spaces of the head (the codebook of Sec. 2.2
// and Alg. 1: 2^b x d x 2 bytes; d8b12, d4b12, d4b10 of Sec. 4.1).
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
//   a P.V operand.  q~ is split into an fp16 high and low part so that the scores are
//   fp32-accurate: columns t0 < 2 carry the high part, columns t0 >= 2 the low part, and one
//   DPP add across the quad recombines them.  1/sqrt(D) and log2(e) are folded into q~.
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
#pragma once
#include "common.h"
#include "mfma_helpers.h"

namespace vecinfer {


namespace {

// DK, DV: sub-vector dims of the key and the value codebooks (keys and values may be quantized
// differently, Sec. 3.2).
// HG: head groups of 4 query heads that share the gathered key / value operands (G <= 4 HG).
// At D = 128 the codebooks fill LDS, so a CU holds one workgroup = NW / 4 wavefronts per SIMD: say
// so, or the compiler squeezes some instantiations under 168 registers for a third wavefront
// that can never come, and serialises gathers to do it (58 -> 43 us for d_k = 4, d_v = 8).
// BK, BV: code widths.  8: one byte per code, one table of 256 centroids per sub-space.  10 or 12:
// codes packed end to end in the token's row, one table of 2^b centroids for all sub-spaces.
// VT: 8-bit value codes stored in tiles of 64 tokens (v_tiled_offset): a lane's share of a tile is
// 16 NROUND_V bytes, fetched with NROUND_V 16-byte loads.
template <int kD, int DK, int DVR, int HG, int NW, bool SPLITQ, int BK = 8, int BV = 8, bool VT = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(NW / 4, kD == 128 ? NW / 4 : NW / 2)))
void decode_mfma_kernel(const __half *q_arg, const float *lam_arg, const __half *cb_k_arg, const __half *cb_v_arg,
                        const __half *k_new_arg, const __half *v_new_arg, unsigned hkv_g_arg, int S_, DecodeParams p)
{
    constexpr int KG = kG * HG;                        // head slots of the workgroup
    // d_v = 8 needs 16 value sub-spaces (one per MFMA column): D = 128.  At D = 64 each of the 8
    // sub-spaces is therefore handled as two of 4 channels that share the code byte (VSPLIT): the
    // gather, the P.V operands and the accumulators are those of d_v = 4 (DV below), only the
    // addressing of the code rows, the staging of the table and the search for a fused new token
    // know the real sub-vector (DVR).
    constexpr bool VSPLIT = kD == 64 && DVR == 8;
    constexpr int DV = VSPLIT ? 4 : DVR;
    static_assert((kD == 128 || kD == 64) && (DK == 8 || DK == 4 || DK == 2) && (DVR == 8 || DVR == 4 || DVR == 2),
                  "shapes this kernel is laid out for");
    static_assert(!VSPLIT || !VT, "split value sub-spaces: codes in rows");
    constexpr bool WK = BK > 8, WV = BV > 8;           // wide codes: shared table, packed rows
    static_assert(!VT || !WV, "tiled value codes are 8-bit codes");
    static_assert((BK == 8 || ((BK == 10 || BK == 12) && DK >= 4 && (kD / DK * BK) % 32 == 0)) &&
                      (BV == 8 || ((BV == 10 || BV == 12) && DVR >= 4 && (kD / DVR * BV) % 32 == 0)),
                  "wide codes: 10 or 12 bits, d = 4 or 8, rows of whole 32-bit words (not d = 8 with 10 bits at D = 64)");
    constexpr int BLOCK = NW * 64;
    constexpr int MK = kD / DK, MV = kD / DVR;         // sub-spaces: 8, 16, 32 or 64
    // bytes of the key / value tables of a KV head in LDS
    constexpr int CBK_BYTES = WK ? (1 << BK) * DK * 2 : kCentroids * kD * 2;
    constexpr int CBV_BYTES = WV ? (1 << BV) * DVR * 2 : kCentroids * kD * 2;
    constexpr int ROWB_K = MK * BK / 8, ROWB_V = MV * BV / 8;    // bytes of a token's code row
    constexpr int ENTRY_K = DK * 2, ENTRY_V = DV * 2;  // bytes per centroid: 8 or 4
    constexpr int SUB_K = kCentroids * ENTRY_K;        // one sub-space table: 2048 or 1024 bytes
    constexpr int SUB_V = kCentroids * ENTRY_V;
    constexpr int NR = kD / 32;                        // score MFMA rounds (32 channels each): 4 or 2;
                                                       // also the P.V operands (and MFMAs) per sub-tile
    constexpr int H = NR / 2;                          // rounds per pipeline stage
    constexpr int NROUND_V = (kD / DV) / 16;           // value sub-spaces per MFMA column: 1, 2 or 4
    // Wide codes.  A lane's key operand needs the MK / 4 consecutive codes of quarter kg of its
    // token's row; the four lanes of a quad (columns 4a .. 4a+3) need, of each of their four
    // tokens, the MV / 4 consecutive codes of quarter a of its row.  Either way that is a run of
    // (M / 4) b bits which starts on a byte: it is fetched as the 2 (d = 8) or 3 (d = 4) aligned
    // dwords that contain it, and a code is cut out of that window when its gather is issued.
    // For values quad lane t0 fetches the window of token t0 of the k-group, and the others read
    // it with DPP.
    constexpr int WIN_K = DK == 8 ? 2 : 3, WIN_V = DVR == 8 ? 2 : 3;
    constexpr int KW = WK ? WIN_K : (MK / 4 + 3) / 4;  // key-code dwords per lane per sub-tile (MK / 4 bytes)
    constexpr int VW = WV ? WIN_V : NROUND_V;          // value-code dwords per lane per sub-tile (4 tokens x NROUND_V bytes)
    // P.V accumulators per head group: one per value sub-space of the lane's column, except at
    // d_v = 8, where the one sub-space is covered in two halves of 4 channels (the four t0 rows of
    // a head serve channels t0 and t0 + 4 in turn).  Register v of accumulator a is channel
    // kChanBlock * (NACC * col + a) + v.
    constexpr int NACC = DV == 8 ? 2 : NROUND_V;
    constexpr int kChanBlock = DV == 8 ? 4 : DV;
    // LDS layout of the value codebook: [r][code][col] with sub-space m = NROUND_V * col + r.
    // LDS serves a gather 16 lanes at a time, and the 16 lanes of such a group read the same r
    // and 16 different col: with the 16 entries of a code in one ROW_V-byte row they fall on
    // disjoint banks whatever their codes are (4.4 instead of 6.7 cycles per gather).  The key
    // codebook keeps the [m][code] order: the 16 lanes of a group all read one sub-space there.
    constexpr int ROW_V = 16 * ENTRY_V;                // 128 or 64 bytes
    constexpr int PLANE_V = kCentroids * ROW_V;        // one r: 32768 or 16384 bytes

    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *const sm_k = smem;
    unsigned char *const sm_v = smem + CBK_BYTES;
    float *const sm_qt = reinterpret_cast<float *>(smem + CBK_BYTES + CBV_BYTES);   // [KG][D]
    float *const sm_new = sm_qt + KG * kD;                                 // [2][D]: k~ and v of the new token
    float *const sm_nsc = sm_new + 2 * kD;                                 // [MK][KG]: its score shares (log2 units)
    float *const sm_nv = sm_nsc + MK * KG;                                 // [D]:    its dequantized value
    unsigned long long *const sm_red = reinterpret_cast<unsigned long long *>(sm_nv + kD);   // [4][NW] (wide codes)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Hkv_ = (int)(hkv_g_arg & 0xffffffu), G_ = (int)(hkv_g_arg >> 24);   // = p.Hkv, p.G
    // Workgroups are dealt to the 8 XCDs round-robin in linear order, so the KV head varies
    // fastest: with 8 KV heads every XCD serves one head and its L2 fetches one codebook set
    // (128 KB) instead of all of them.  (The grid is (S, Hkv, B).)
    const int lin = blockIdx.x + S_ * blockIdx.y;
    const int g = lin % Hkv_, s = lin / Hkv_, b = blockIdx.z;
    const int col = lane & 15;       // MFMA row (A) / column (B, D) index of this lane
    const int kg = lane >> 4;        // k-group (A, B) / row group (D) of this lane
    const size_t bg = (size_t)b * Hkv_ + g;
    // ---- The kernel's first memory requests use nothing but the leading arguments, which the
    // command processor can place in scalar registers before the wavefront starts (kernel-argument
    // preloading); everything else of `p` takes a trip to the argument buffer, which now runs
    // beside these requests instead of ahead of them.
    // The wavefront's small input rows are requested first: loads come back in order, so the
    // query transform below runs while the codebooks and the first code tiles are still on their way
    // (wavefront hh < G: query head hh; the last two wavefronts: key and value row of a fused new
    // token).  Every wavefront issues the same six loads (a wavefront without a query head, or a
    // launch without a new token, reads a row that exists anyway and ignores it), and the fp16
    // rows are kept as raw bits until they are used: neither a branch nor a conversion makes the
    // wavefront wait here for data it has only just requested.
    auto raw16 = [](const __half *src) -> unsigned { return *reinterpret_cast<const unsigned short *>(src); };
    auto widen = [](unsigned bits) { return (float)__builtin_bit_cast(_Float16, (unsigned short)bits); };
    const bool q_role = wave < KG && wave < G_;
    const __half *const qsrc = q_arg + (((size_t)b * Hkv_ + g) * G_ + (q_role ? wave : 0)) * kD;
    const unsigned qh0 = raw16(qsrc + lane), qh1 = raw16(qsrc + (kD == 128 ? 64 : 0) + lane);
    const float ql0 = lam_arg[(size_t)g * kD + lane], ql1 = lam_arg[(size_t)g * kD + (kD == 128 ? 64 : 0) + lane];
    const __half *const nsrc = k_new_arg ? (wave == NW - 1 ? v_new_arg : k_new_arg) + bg * kD : qsrc;
    const unsigned nh0 = raw16(nsrc + lane), nh1 = raw16(nsrc + (kD == 128 ? 64 : 0) + lane);
    const float nl0 = ql0, nl1 = ql1;
    asm volatile("" ::: "memory");                 // keep these loads ahead of the big ones below
    constexpr int CPL = 16 / ENTRY_V;                  // codes per 16-byte load of the value codebook
    // each codebook is staged as items of 1 KB (one wavefront instruction each), dealt round-robin
    constexpr int kStageK = CBK_BYTES / 1024, kStageKPerWave = (kStageK + NW - 1) / NW;
    constexpr int kStageV = CBV_BYTES / 1024, kStageVPerWave = (kStageV + NW - 1) / NW;
    static_assert(WV || NROUND_V * (kCentroids / (4 * CPL)) == kStageV, "value items: (code group, r)");
    const int vq = lane >> 4, vcol = lane & 15;
    uintx4 vreg[kStageVPerWave];
    // ---- stage both codebooks of this KV head in LDS (Alg. 1 step 7, and C_k likewise), through
    // registers: all 16 loads of a wavefront (16 KB) are issued back to back right behind the query
    // rows; the LDS writes come after the q~ section.
    // (Direct global->LDS loads measured slower here: a wavefront got through its 8 of them at
    // about one L2 latency each.)
    uintx4 kreg[kStageKPerWave];
    {
        const unsigned char *srck = reinterpret_cast<const unsigned char *>(cb_k_arg) + (size_t)g * CBK_BYTES;
        const unsigned char *srcv = reinterpret_cast<const unsigned char *>(cb_v_arg) + (size_t)g * CBV_BYTES;
        // keys keep the [m][code] order (a shared table its one order): item = 1 KB chunk, 16 bytes per lane
#pragma unroll
        for (int j = 0; j < kStageKPerWave; ++j) {
            const int it = wave + NW * j;
            if (kStageK % NW == 0 || it < kStageK)
                kreg[j] = *reinterpret_cast<const uintx4 *>(srck + it * 1024 + lane * 16);
        }
        // The value codebook is transposed on the way, through registers: a lane loads 16 bytes
        // (CPL = 16 / ENTRY_V consecutive codes of one sub-space) and writes them entry by entry.
        // The 16 lanes of a quarter-wavefront hold 16 different col (distinct banks on the write);
        // the four quarters take adjacent 16-byte pieces, so an instruction reads 64 contiguous
        // bytes of 16 tables.  Item it serves r = it % NROUND_V and the 4 * CPL codes of code
        // group it / NROUND_V.
        // (VSPLIT: a lane's 16 bytes are the whole centroid `8 it + lane / 8` of sub-space lane % 8, i.e.
        // the entries of that code for columns 2 (lane % 8) and 2 (lane % 8) + 1: one 16-byte write.)
#pragma unroll
        for (int j = 0; j < kStageVPerWave; ++j) {
            const int it = wave + NW * j;
            const int r = it % NROUND_V, code = (it / NROUND_V) * 4 * CPL + vq * CPL;
            if (kStageV % NW == 0 || it < kStageV)
                vreg[j] = WV ? *reinterpret_cast<const uintx4 *>(srcv + it * 1024 + lane * 16)   // shared table: as is
                          : VSPLIT ? *reinterpret_cast<const uintx4 *>(srcv + (lane & 7) * (kCentroids * 16) + (8 * it + (lane >> 3)) * 16)
                             : *reinterpret_cast<const uintx4 *>(srcv + (NROUND_V * vcol + r) * SUB_V + code * ENTRY_V);
        }
    }
    // Every other argument the prologue uses is read here, in one batch of scalar loads: left to
    // itself the compiler fetches them where they are first needed, one cold trip to the argument
    // buffer after the other along the prologue.
#define VECINFER_PIN(x) asm volatile("" ::"s"(x))
    VECINFER_PIN(p.seq_lens); VECINFER_PIN(p.N); VECINFER_PIN(p.n_cap); VECINFER_PIN(p.k_idx); VECINFER_PIN(p.v_idx);
#undef VECINFER_PIN

    // With a fused append the new token is the sequence's last one: its codes are produced in
    // this launch (below), so the tile loop covers the len - 1 older tokens only.  Workgroup s
    // encodes sub-spaces s, s + S, ... of the new token's key and value.
    const long long len = seq_len_of(p, b);
    const bool fused = k_new_arg != nullptr && len > 0;
    // items of the new token that are shared out: sub-spaces (8-bit codes), or groups of four
    // sub-spaces whose codes fill a whole number of bytes (10- and 12-bit codes)
    constexpr int ITEMS_K = WK ? MK / 4 : MK, ITEMS_V = WV ? MV / 4 : MV;
    // workgroup s takes key items s, s + S, ...; value sub-spaces likewise, value groups (wide codes)
    // starting behind the key items: group j goes to workgroup (j + ITEMS_K) % S
    const int vgrp0 = (s + S_ - ITEMS_K % S_) % S_;        // first value group of this workgroup
    const bool has_new = fused && (s < ITEMS_K || (WV ? vgrp0 < ITEMS_V : s < ITEMS_V));
    long long n0, n1;
    split_range(fused ? len - 1 : len, S_, s, kTile, n0, n1);
    if constexpr (WK || WV) {
        // A group of the new token with 10- / 12-bit codes is a search through the whole shared
        // table: microseconds of work on the few workgroups that take one, which the others
        // would wait out.  Those workgroups therefore get that much shorter a token range
        // (wK, wV tokens; multiples of the tile), and all ranges shift accordingly: boundary(s) =
        // s * chunk - (weights of the workgroups before s).  Only when every workgroup has at
        // most one group of a kind and the ranges stay non-empty; the merge does not care how
        // the tokens are dealt.
        // (weights in tiles, from timing four configurations at 196608 tokens: 5 + 14 C / 4096 at
        // d = 8, 5 + 2 C / 4096 at d = 4; the step is within 0.3 us of its best over a wide range)
        constexpr long long wK = WK ? kTile * (((1 << BK) * (DK == 8 ? 14 : 2)) / 4096 + 5) : 0;
        constexpr long long wV = WV ? kTile * (((1 << BV) * (DVR == 8 ? 14 : 2)) / 4096 + 5) : 0;
        constexpr int IK = WK ? ITEMS_K : 0, IV = WV ? ITEMS_V : 0;
        if (fused && S_ >= IK && S_ >= IV) {
            const long long total = len - 1 + wK * IK + wV * IV;
            long long chunk = (total + S_ - 1) / S_;
            chunk = (chunk + kTile - 1) / kTile * kTile;
            if (chunk >= wK + wV) {
                const int a = ITEMS_K % S_;                    // first workgroup with a value group
                auto boundary = [&](int t) -> long long {
                    const long long before_k = t < IK ? t : IK;
                    const int hi = a + IV;
                    long long before_v = (t < hi ? t : hi) - a;
                    if (before_v < 0) before_v = 0;
                    if (hi > S_) before_v += t < hi - S_ ? t : hi - S_;
                    long long x = (long long)t * chunk - wK * before_k - wV * before_v;
                    return x < 0 ? 0 : (x > len - 1 ? len - 1 : x);
                };
                n0 = boundary(s);
                n1 = boundary(s + 1);
            }
        }
    }

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
    unsigned mask_a, mask_b;                             // select the fp16 slot(s) of (p, p)
    if (DV == 4 || DV == 8) {
        // d_v = 8: the same two masks pick channel t0 in the first dword pair of the operand
        // (channels 0-3) or channel t0 + 4 in the second pair (channels 4-7)
        mask_a = t0 == 0 ? 0x0000ffffu : (t0 == 1 ? 0xffff0000u : 0u);
        mask_b = t0 == 2 ? 0x0000ffffu : (t0 == 3 ? 0xffff0000u : 0u);
    } else {
        mask_a = t0 == 0 ? 0x0000ffffu : (t0 == 1 ? 0xffff0000u : 0u);
        mask_b = 0u;
    }
    unsigned sel[4];                                     // sel[i] = all ones iff t0 == i
#pragma unroll
    for (int i = 0; i < 4; ++i) sel[i] = t0 == i ? 0xffffffffu : 0u;
    // LDS byte offsets: keys  MK/4 sub-spaces per kg
    //                   values sub-space NROUND_V*col + r
    // LDS offset of the dynamic segment.  The kernel owns no static LDS, so the segment starts at
    // 0 (the launcher checks the kernel's static LDS size and refuses to launch otherwise); read
    // off the pointer, the compiler would learn that constant only after instruction selection
    // and keep an add of it in front of every gather of the shared tables of wide codes.
    const unsigned lds_base = 0u;
    const unsigned lds_k = lds_base + (WK ? 0u : (unsigned)(kg * (MK / 4) * SUB_K));
    // (wide codes with split value sub-spaces: column col reads half col & 1 of its 16-byte centroid)
    const unsigned lds_v = lds_base + (unsigned)CBK_BYTES +
                           (WV ? (VSPLIT ? (unsigned)((col & 1) * ENTRY_V) : 0u) : (unsigned)(col * ENTRY_V));
    // wide codes: first bit of the lane's run of codes inside its window, and of its own code(s)
    // inside the quad's window
    const unsigned pos_k = (unsigned)(kg * (MK / 4) * BK) & 31u;
    const unsigned pos_v = ((unsigned)((col >> 2) * (MV / 4) * BV) & 31u) +
                           (unsigned)((VSPLIT ? (col & 3) >> 1 : (col & 3) * NROUND_V) * BV);

    const uint8_t *krow = p.k_idx + bg * p.n_cap * ROWB_K;
    const uint8_t *vrow = p.v_idx + bg * p.n_cap * ROWB_V;
    const long long last = n1 - 1;

    // token owned by A-row i of sub-tile st: base + 16 st + 4 (i % 4) + i / 4, so that D-register v
    // of row group rg is token base + 16 st + 4 v + rg
    const int krow_tok = 4 * (col & 3) + (col >> 2);

    // Codes of one 64-token tile as this lane needs them: kc = the key-code bytes of the lane's
    // A row in each sub-tile, vc = the value-code bytes of the 4 tokens of its k-group.
    struct Codes {
        unsigned kc[4][KW];
        unsigned vc[4][VW];
    };
    // The code rows of (b, g) are read through buffer descriptors whose extent ends at the
    // split's last token: a lane's address is one loop-invariant VGPR offset plus the tile's
    // base plus an instruction immediate, and loads past the end of the split return 0 (a
    // valid code) instead of needing a clamp.  The host checks N * M < 2^31.
    const __amdgpu_buffer_rsrc_t rsrc_k =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(krow), 0, (int)((unsigned)n1 * ROWB_K), 0x00020000);
    // (tiled value codes: whole 64-token blocks; n_cap is a multiple of 64, so the last block exists)
    const __amdgpu_buffer_rsrc_t rsrc_v = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(vrow), 0, (int)((unsigned)(VT ? (n1 + 63) / 64 * 64 : n1) * ROWB_V), 0x00020000);
    const unsigned koff_lane = WK ? (unsigned)(krow_tok * ROWB_K + 4 * ((kg * (MK / 4) * BK) >> 5))
                                  : (unsigned)(krow_tok * MK + kg * (MK / 4));
    const unsigned voff_lane = WV ? (unsigned)((4 * (col & 3) + kg) * ROWB_V + 4 * (((col >> 2) * (MV / 4) * BV) >> 5))
                               : VT ? (unsigned)(lane * 16)
                               : VSPLIT ? (unsigned)(kg * MV + (col >> 1))
                                    : (unsigned)(kg * MV + col * NROUND_V);

    auto load_codes_k = [&](Codes &cd, long long tb) {
        const unsigned ko = (unsigned)tb * ROWB_K + koff_lane;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            // keys: the MK / 4 code bytes of the lane's k-slot range of its token
            if constexpr (WK) {
#pragma unroll
                for (int j = 0; j < WIN_K; ++j)
                    cd.kc[st][j] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_k, ko + 16 * st * ROWB_K + 4 * j, 0, kStreamPolicy);
            } else if constexpr (MK / 4 == 2) {
                cd.kc[st][0] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rsrc_k, ko + 16 * st * MK, 0, kStreamPolicy);
            } else if constexpr (MK / 4 == 4) {
                cd.kc[st][0] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_k, ko + 16 * st * MK, 0, kStreamPolicy);
            } else if constexpr (MK / 4 == 8) {
                const uintx2 w = __builtin_amdgcn_raw_buffer_load_b64(rsrc_k, ko + 16 * st * MK, 0, kStreamPolicy);
                cd.kc[st][0] = w[0]; cd.kc[st][1] = w[1];
            } else {
                const uintx4 w = __builtin_amdgcn_raw_buffer_load_b128(rsrc_k, ko + 16 * st * MK, 0, kStreamPolicy);
                cd.kc[st][0] = w[0]; cd.kc[st][1] = w[1]; cd.kc[st][2] = w[2]; cd.kc[st][3] = w[3];
            }
        }
    };
    auto load_codes_v = [&](Codes &cd, long long tb) {
        const unsigned vo = (unsigned)tb * ROWB_V + voff_lane;
        if constexpr (VT) {
            // the lane's 16 NROUND_V bytes of the tile, in the order (sub-tile, token v, round r), 16
            // from each of the block's NROUND_V slabs of 1 KB: dword j of them is cd.vc[j / NROUND_V][j % NROUND_V]
            unsigned w[4 * NROUND_V];
#pragma unroll
            for (int j = 0; j < NROUND_V; ++j) {
                const uintx4 x = __builtin_amdgcn_raw_buffer_load_b128(rsrc_v, vo + 1024 * j, 0, kStreamPolicy);
                w[4 * j] = x[0]; w[4 * j + 1] = x[1]; w[4 * j + 2] = x[2]; w[4 * j + 3] = x[3];
            }
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int j = 0; j < NROUND_V; ++j) cd.vc[st][j] = w[st * NROUND_V + j];
            return;
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            // values: NROUND_V bytes (sub-spaces NROUND_V col ..) of each of the tokens 4 v + kg,
            // packed token after token: byte v * NROUND_V + r
            if constexpr (WV) {
                // the window of token 4 (col & 3) + kg: quarter col / 4 of its row
#pragma unroll
                for (int j = 0; j < WIN_V; ++j)
                    cd.vc[st][j] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_v, vo + 16 * st * ROWB_V + 4 * j, 0, kStreamPolicy);
            } else if constexpr (NROUND_V == 1) {
                unsigned w = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    w |= (unsigned)__builtin_amdgcn_raw_buffer_load_b8(rsrc_v, vo + (16 * st + 4 * v) * MV, 0, kStreamPolicy) << (8 * v);
                cd.vc[st][0] = w;
            } else if constexpr (NROUND_V == 2) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    ushortx2 t;
                    t[0] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rsrc_v, vo + (16 * st + 8 * u) * MV, 0, kStreamPolicy);
                    t[1] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(rsrc_v, vo + (16 * st + 8 * u + 4) * MV, 0, kStreamPolicy);
                    cd.vc[st][u] = __builtin_bit_cast(unsigned, t);
                }
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    cd.vc[st][v] = __builtin_amdgcn_raw_buffer_load_b32(rsrc_v, vo + (16 * st + 4 * v) * MV, 0, kStreamPolicy);
            }
        }
    };
    auto load_codes = [&](Codes &cd, long long tb) {
        load_codes_k(cd, tb);
        load_codes_v(cd, tb);
    };

    // Which tiles a wavefront owns.  The two wavefronts of a SIMD do not run at the same speed:
    // the one launched first (wavefronts 0 .. NW/2-1) wins the issue arbitration and gets through
    // a tile about 13 % sooner, so an even deal leaves it idle at the end of a long split.  Tiles
    // are therefore dealt in periods of 12 rounds: 11 rounds to every wavefront in turn and one
    // round shared by the first half only, two tiles each (13 : 11).  Short splits (under 11
    // rounds) see the plain round-robin.  The deal is static, so results are reproducible.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto tile_base = [&](int k) -> long long {          // first token of this wavefront's k-th tile
        constexpr int kFull = 11, kPeriod = (kFull + 1) * NW;
        int per, off;
        if (NW != 8) {
            per = 0;
            off = k * NW + wave_u;                          // plain round-robin
        } else if (wave_u < NW / 2) {
            per = k / (kFull + 2);
            const int i = k % (kFull + 2);
            off = i < kFull ? i * NW + wave_u : kFull * NW + (i - kFull) * (NW / 2) + wave_u;
        } else {
            per = k / kFull;
            off = (k % kFull) * NW + wave_u;
        }
        return n0 + ((long long)per * kPeriod + off) * kTile;
    };
    Codes ca, cb;

    // The first two tiles' codes start their trip from HBM now, under the prologue.  They are
    // requested after the codebooks: loads return in order, and the first touch of the code stream
    // is the slowest load of the kernel, so the other way round the staging would wait behind it.
    load_codes(ca, tile_base(0));
    load_codes(cb, tile_base(1));
    // ---- q~ = (q * lambda) H_D for the 4 heads of the group (un-normalised butterflies):
    // wavefront hh transforms head hh in registers, a lane holding channels `lane` and
    // `lane + 64`: one in-lane butterfly (partner distance 64), six across lanes.
    static_assert(KG <= NW && NW >= 2, "one wavefront per head slot for the query transform");
    if (wave < KG && wave >= G_) {
        // spare head slot (G < 4): a zero query; its scores and outputs are never written out
        sm_qt[wave * kD + lane] = 0.f;
        if (kD == 128) sm_qt[wave * kD + 64 + lane] = 0.f;
    } else if (wave < KG && kD == 64) {
        // D = 64: one channel per lane, six butterfly stages across lanes
        float x0 = widen(qh0) * ql0;
#pragma unroll
        for (int st = 1; st < 64; st <<= 1) {
            const float o0 = __shfl_xor(x0, st);
            x0 = (lane & st) != 0 ? (o0 - x0) : (x0 + o0);
        }
        sm_qt[wave * kD + lane] = x0;
    } else if (wave < KG) {
        float x0 = widen(qh0) * ql0, x1 = widen(qh1) * ql1;
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
        sm_qt[wave * kD + lane] = x0;
        sm_qt[wave * kD + 64 + lane] = x1;
    }
    // the new token's key and value (fused append): the last two wavefronts
    if (has_new && wave == NW - 2 && kD == 64) {
        float x0 = widen(nh0) / nl0;
#pragma unroll
        for (int st = 1; st < 64; st <<= 1) {
            const float o0 = __shfl_xor(x0, st);
            x0 = (lane & st) != 0 ? (o0 - x0) : (x0 + o0);
        }
        sm_new[lane] = x0 * (1.0f / sqrtf((float)kD));
    } else if (has_new && wave == NW - 2) {
        // k~ = (k / lambda) H_D of the new token (Eq. 9), operation for operation what the
        // cache-fill kernels compute (true division, butterfly stages at distance 1, 2, .. 64,
        // then 1/sqrt D), so that the fused step writes the codes a separate append would
        float x0 = widen(nh0) / nl0, x1 = widen(nh1) / nl1;
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
    } else if (has_new && wave == NW - 1) {
        sm_new[kD + lane] = widen(nh0);
        if (kD == 128) sm_new[kD + 64 + lane] = widen(nh1);
    }
    // second half of the codebook staging: registers -> LDS
#pragma unroll
    for (int j = 0; j < kStageKPerWave; ++j) {
        const int it = wave + NW * j;
        if (kStageK % NW == 0 || it < kStageK)
            *reinterpret_cast<uintx4 *>(sm_k + it * 1024 + lane * 16) = kreg[j];
    }
#pragma unroll
    for (int j = 0; j < kStageVPerWave; ++j) {
        const int it = wave + NW * j;
        const int r = it % NROUND_V, code = (it / NROUND_V) * 4 * CPL + vq * CPL;
        if constexpr (WV) {
            if (kStageV % NW == 0 || it < kStageV)
                *reinterpret_cast<uintx4 *>(sm_v + it * 1024 + lane * 16) = vreg[j];
        } else if constexpr (VSPLIT) {
            if (kStageV % NW == 0 || it < kStageV)
                *reinterpret_cast<uintx4 *>(sm_v + (8 * it + (lane >> 3)) * ROW_V + (lane & 7) * 16) = vreg[j];
        } else if (kStageV % NW == 0 || it < kStageV) {
#pragma unroll
            for (int e = 0; e < CPL; ++e) {
                unsigned char *const d = sm_v + r * PLANE_V + (code + e) * ROW_V + vcol * ENTRY_V;
                if constexpr (DV == 8)
                    *reinterpret_cast<uintx4 *>(d) = vreg[j];
                else if constexpr (DV == 4)
                    *reinterpret_cast<uintx2 *>(d) = uintx2{vreg[j][2 * e], vreg[j][2 * e + 1]};
                else
                    *reinterpret_cast<unsigned *>(d) = vreg[j][e];
            }
        }
    }
    __syncthreads();

    // ---- B operands of the score MFMAs: q~_h[(D/4) kg + 8r .. +8); columns with t0 < 2 take the
    // fp16 high part, columns with t0 >= 2 the low part (x - float(hi)).
    // fold = (1/sqrt D of H_D) * (1/sqrt D of the score) * log2 e
    // With the split query a head has four columns but only two parts, so a column can serve two
    // sub-tiles: the operand exists in two copies, copy c zero outside the columns with t0 % 2 = c,
    // sub-tile st multiplies copy st % 2, and sub-tiles 0, 1 (2, 3) accumulate in one register
    // set.  Column t0 of that set then holds part t0 / 2 of sub-tile t0 % 2 (2 + t0 % 2) and nothing
    // else, which leaves the softmax a two-way pick instead of two four-way picks per score.
    // (One head group only: with two the copies cost 32 more registers than there are.)
    constexpr int NQ = SPLITQ && HG == 1 ? 2 : 1;    // operand copies;  score register sets = 4 / NQ
    half8 bq[HG][NQ][NR];
    {
        const float fold = kLog2e / (float)kD;
#pragma unroll
        for (int hg = 0; hg < HG; ++hg) {
            const int hh = kG * hg + (col >> 2);
#pragma unroll
            for (int r = 0; r < NR; ++r)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = sm_qt[hh * kD + (kD / 4) * kg + 8 * r + e] * fold;
                    const _Float16 hi = (_Float16)x;
                    const _Float16 lo = (_Float16)(x - (float)hi);
                    const _Float16 part = (SPLITQ && (col & 2)) ? lo : hi;
#pragma unroll
                    for (int c = 0; c < NQ; ++c) bq[hg][c][r][e] = (NQ == 1 || (col & 1) == c) ? part : (_Float16)0.f;
                }
        }
    }

    // ---- fused append: this workgroup's sub-spaces of the new token, dealt to the wavefronts as
    // (sub-space, key | value) items.  Eq. 2 by exhaustive search over the table already in LDS: a lane
    // scans centroids lane, lane + 64, ..; squared distances summed in channel order in fp32; the
    // lowest index among the centroids at minimum distance wins.  The key item
    // also leaves the new token's score share of its sub-space for the 4 heads, the value item
    // the dequantized channels, for the merge kernel.
    const long long pos = len - 1;
    const float fold = kLog2e / (float)kD;
    // A wavefront takes up to four items of one kind at a time (items i0, i0 + NW, ..): their
    // chains of LDS reads, distance arithmetic and cross-lane reductions are independent, so
    // they overlap instead of paying their latencies one after the other.
    auto new_items = [&](auto kv_c, auto nb_c, int i0) {
        constexpr int kv = decltype(kv_c)::value;          // 0: key sub-spaces, 1: value sub-spaces
        constexpr int NB = decltype(nb_c)::value;          // items taken at a time
        constexpr int DS = kv == 0 ? DK : DVR, EN = 2 * DS, MX = kv == 0 ? MK : MV;
        // entry c of a sub-space sits at tab + c * stride (value tables are transposed)
        constexpr int stride = kv == 0 ? ENTRY_K : ROW_V;
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
                      : VSPLIT ? sm_v + m[b4] * 2 * ENTRY_V        // columns 2 m and 2 m + 1 side by side
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
    // Wide codes: an item is a group of four sub-spaces (4 b bits = whole bytes of the packed
    // row) and the whole workgroup works on it: wavefront w scans centroids
    // [w C / NW, (w + 1) C / NW) of the one table for the four sub-vectors at once, a lane taking
    // every 64th of them in increasing order (strict "<": its lowest index wins); the
    // wavefronts' (distance bits, index) keys meet in LDS and the smallest key wins, which is the
    // lowest index at the minimum distance.  Same distance arithmetic as the append kernels.
    auto wide_item = [&](auto kv_c, int grp) {
        constexpr int kv = decltype(kv_c)::value;
        constexpr int DS = kv == 0 ? DK : DVR, BITS = kv == 0 ? BK : BV, MX = kv == 0 ? MK : MV;
        constexpr int C = 1 << BITS, PER_WAVE = C / NW, EN = 2 * DS;
        const unsigned char *const tab = kv == 0 ? sm_k : sm_v;
        float x[4][DS];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int jj = 0; jj < DS; ++jj) x[i][jj] = sm_new[kv * kD + (4 * grp + i) * DS + jj];
        unsigned best[4], arg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            best[i] = 0x7f800000u;                         // +inf
            arg[i] = 0;
        }
#pragma unroll 2
        for (int it = 0; it < PER_WAVE / 64; ++it) {
            const unsigned c = (unsigned)(wave_u * PER_WAVE + it * 64 + lane);
            _Float16 cen[DS];
            __builtin_memcpy(cen, tab + c * EN, EN);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float dist = 0.f;
#pragma unroll
                for (int jj = 0; jj < DS; ++jj) {
                    const float tdiff = x[i][jj] - (float)cen[jj];
                    dist = fmaf(tdiff, tdiff, dist);
                }
                const unsigned v = __float_as_uint(dist);  // a non-negative fp32 orders like its bit pattern
                if (v < best[i]) {
                    best[i] = v;
                    arg[i] = c;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned dmin = wave_umin(best[i]);
            const unsigned code = wave_umin(best[i] == dmin ? arg[i] : 0xffffffffu);
            if (lane == 0) sm_red[i * NW + wave_u] = ((unsigned long long)dmin << 32) | code;
        }
        __syncthreads();
        if (wave_u == 0) {
            // lanes 16 i .. 16 i + 15 look after sub-vector i of the group
            const int i = lane >> 4, l16 = lane & 15, m = 4 * grp + i;
            unsigned long long key = sm_red[i * NW];
#pragma unroll
            for (int w = 1; w < NW; ++w) key = sm_red[i * NW + w] < key ? sm_red[i * NW + w] : key;
            const unsigned code = (unsigned)key;
            _Float16 win[DS];
            __builtin_memcpy(win, tab + code * EN, EN);
            if (kv == 0) {
                if (l16 < G_) {
                    float sc = 0.f;
#pragma unroll
                    for (int jj = 0; jj < DS; ++jj)
                        sc = fmaf(sm_qt[l16 * kD + m * DS + jj] * fold, (float)win[jj], sc);
                    p.new_sc[((size_t)bg * MK + m) * G_ + l16] = sc;
                    sm_nsc[m * KG + l16] = sc;
                }
            } else {
                float mine = (float)win[0];
#pragma unroll
                for (int jj = 1; jj < DS; ++jj) mine = l16 == jj ? (float)win[jj] : mine;
                if (l16 < DS) {
                    p.new_v[(size_t)bg * kD + m * DS + l16] = mine;
                    sm_nv[m * DS + l16] = mine;
                }
            }
            // the group's four codes, end to end, are bytes [grp 4 b / 8, (grp + 1) 4 b / 8) of the row
            const unsigned c0 = (unsigned)__shfl(code, 0), c1 = (unsigned)__shfl(code, 16);
            const unsigned c2 = (unsigned)__shfl(code, 32), c3 = (unsigned)__shfl(code, 48);
            const unsigned long long bits = (unsigned long long)c0 | ((unsigned long long)c1 << BITS) |
                                            ((unsigned long long)c2 << (2 * BITS)) |
                                            ((unsigned long long)c3 << (3 * BITS));
            constexpr int GB = 4 * BITS / 8;
            uint8_t *const row = (kv == 0 ? p.k_idx_w : p.v_idx_w) + ((size_t)bg * p.n_cap + pos) * (MX * BITS / 8);
            if (lane < GB) row[grp * GB + lane] = (uint8_t)(bits >> (8 * lane));
        }
        __syncthreads();                                   // sm_red is free for the next item
    };
    if constexpr (WK) {
        if (has_new)
            for (int grp = s; grp < ITEMS_K; grp += S_) wide_item(std::integral_constant<int, 0>{}, grp);
    }
    if constexpr (WV) {
        // value groups start where the key items end, so that other workgroups take them
        if (has_new)
            for (int grp = vgrp0; grp < ITEMS_V; grp += S_) wide_item(std::integral_constant<int, 1>{}, grp);
    }
    // 8-bit codes: key item i (sub-space s + i S) goes to wavefront i % NW, value item i to
    // wavefront (i + 1) % NW; a wavefront with one item of a kind (the usual case: at least as
    // many splits as sub-spaces) takes it alone, otherwise four at a time
    auto items8 = [&](auto kv_c) {
        constexpr int kv = decltype(kv_c)::value, MX = kv == 0 ? MK : MV;
        const int first = kv == 0 ? wave_u : (wave_u + NW - 1) % NW;
        if (s + (first + NW) * S_ < MX) {
            for (int i0 = first; s + i0 * S_ < MX; i0 += 4 * NW) new_items(kv_c, std::integral_constant<int, 4>{}, i0);
        } else if (s + first * S_ < MX) {
            new_items(kv_c, std::integral_constant<int, 1>{}, first);
        }
    };
    float m_run[HG];                  // running max of head 4 hg + col/4 (log2 units), same in all its lanes
    float l_part[HG];                 // this lane's share of the running sum
    floatx4 acc_o[HG][NACC];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
        m_run[hg] = -INFINITY;
        l_part[hg] = 0.f;
#pragma unroll
        for (int r = 0; r < NACC; ++r) acc_o[hg][r] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // LDS byte address of centroid `code byte k of w` in the sub-space table at `base`:
    // one v_dot4_u32_u8 (w . (ENTRY_K << 8k) + base) instead of a bit-field extract and a shift-add.
    auto lds_addr = [&](unsigned w, int k, unsigned base) -> unsigned {
        return __builtin_amdgcn_udot4(w, (unsigned)ENTRY_K << (8 * k), base, false);
    };
    auto lds_addr_v = [&](unsigned w, int k, unsigned base) -> unsigned {   // code * ROW_V + base
        if constexpr (ROW_V > 255)                  // the multiplier of v_dot4 is one byte: halve, then double
            return __builtin_amdgcn_udot4(w, (unsigned)(ROW_V / 2) << (8 * k), base >> 1, false) << 1;
        else
            return __builtin_amdgcn_udot4(w, (unsigned)ROW_V << (8 * k), base, false);
    };
    // Wide codes: the B-bit field at bit `pos` (a lane constant, below 32 W - B) of a window of W
    // dwords, as the byte offset of its centroid in the shared table (entry = 1 << LOG2E bytes).
    auto field2 = [](unsigned w0, unsigned w1, unsigned pos, auto bits_c, auto log2e_c) -> unsigned {
        constexpr int B = decltype(bits_c)::value, LOG2E = decltype(log2e_c)::value;
        const unsigned long long w = ((unsigned long long)w1 << 32) | w0;
        return ((unsigned)(w >> pos) & ((1u << B) - 1u)) << LOG2E;
    };
    // A window of three dwords moved down by the lane constant `pos`, so that the fields of the
    // lane's run sit at the same bit positions in every lane (one funnel shift per dword and
    // window instead of a dword select and a 64-bit shift per code).  `nd` = dwords of the result
    // that are used.
    auto align3 = [](unsigned w0, unsigned w1, unsigned w2, unsigned pos, unsigned (&o)[3], auto nd_c) {
        constexpr int ND = decltype(nd_c)::value;
        const unsigned j = pos >> 5, sh = pos & 31u;
        const unsigned t0 = j == 0 ? w0 : (j == 1 ? w1 : w2), t1 = j == 0 ? w1 : (j == 1 ? w2 : 0u);
        o[0] = __builtin_amdgcn_alignbit(t1, t0, sh);
        if constexpr (ND > 1) {
            const unsigned t2 = j == 0 ? w2 : 0u;
            o[1] = __builtin_amdgcn_alignbit(t2, t1, sh);
            o[2] = t2 >> sh;
        } else {
            o[1] = o[2] = 0u;
        }
    };
    // the B-bit field at the constant bit `at` of an aligned window, as a table offset
    auto const_field = [](const unsigned (&o)[3], int at, auto bits_c, auto log2e_c) -> unsigned {
        constexpr int B = decltype(bits_c)::value, LOG2E = decltype(log2e_c)::value;
        const int j = at >> 5, sh = at & 31;
        const unsigned x = sh + B <= 32 ? o[j] >> sh : __builtin_amdgcn_alignbit(o[j + 1 < 3 ? j + 1 : 2], o[j], (unsigned)sh);
        return (x & ((1u << B) - 1u)) << LOG2E;
    };
    // key code i of the lane's run in the window w
    auto win_field_k = [&](const unsigned (&w)[KW], int i) -> unsigned {
        constexpr auto bits_c = std::integral_constant<int, BK>{};
        constexpr auto log2e_c = std::integral_constant<int, DK == 8 ? 4 : 3>{};
        if constexpr (!WK) return 0u;
        else if constexpr (WIN_K == 2) return field2(w[0], w[1], pos_k + BK * i, bits_c, log2e_c);
        else {
            unsigned o[3];
            align3(w[0], w[1], w[2], pos_k, o, std::integral_constant<int, 3>{});
            return const_field(o, BK * i, bits_c, log2e_c);
        }
    };
    // A operand of the score MFMA for sub-tile st, round r: the centroids of 8/d consecutive
    // key sub-spaces of the lane's token (pure LDS gathers, no arithmetic on the values).
    auto gather_k = [&](const Codes &cd, int st, int r) -> half8 {
        if constexpr (WK && DK == 8) {
            // code r of the lane's four
            return __builtin_bit_cast(half8, lds_load_b128(lds_k + win_field_k(cd.kc[st], r)));
        } else if constexpr (WK) {
            // codes 2r, 2r + 1 of the lane's eight
            const uint2 x0 = lds_load_b64(lds_k + win_field_k(cd.kc[st], 2 * r));
            const uint2 x1 = lds_load_b64(lds_k + win_field_k(cd.kc[st], 2 * r + 1));
            return as_half8(x0.x, x0.y, x1.x, x1.y);
        } else if constexpr (DK == 8) {
            // sub-space (MK/4) kg + r: one 16-byte entry is the whole operand
            return __builtin_bit_cast(half8, lds_load_b128(lds_addr(cd.kc[st][0], r, lds_k) + r * SUB_K));
        } else if (DK == 4) {
            // sub-spaces (MK/4) kg + 2r, + 2r + 1: code bytes 2r, 2r+1 of the lane's MK / 4
            const unsigned w = cd.kc[st][r >> 1];
            const int k0 = 2 * (r & 1);
            const uint2 x0 = lds_load_b64(lds_addr(w, k0, lds_k) + (2 * r) * SUB_K);
            const uint2 x1 = lds_load_b64(lds_addr(w, k0 + 1, lds_k) + (2 * r + 1) * SUB_K);
            return as_half8(x0.x, x0.y, x1.x, x1.y);
        } else {
            // sub-spaces (MK/4) kg + 4r .. +3: the 4 code bytes of dword r
            const unsigned w = cd.kc[st][r];
            unsigned x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                x[q] = lds_load_b32(lds_addr(w, q, lds_k) + (4 * r + q) * SUB_K);
            return as_half8(x[0], x[1], x[2], x[3]);
        }
    };
    // B operand q (0 .. NR-1) of the P.V MFMAs of sub-tile st; the code of (token v of the
    // k-group, round r) is byte v * NROUND_V + r of the packed value codes.  d = 4:
    // q = u * NROUND_V + r (step u, round r): centroids of sub-space NROUND_V col + r for tokens
    // 2u, 2u+1.  d = 2: q = r: centroids of sub-space NROUND_V col + r for the 4 tokens.
    // wide value codes: the window that quad lane v fetched (token v of the k-group)
    auto quad_get = [](unsigned x, int v) -> unsigned {
        switch (v) {                                    // v is a constant after unrolling
        case 0: return quad_bcast<0>(x);
        case 1: return quad_bcast<1>(x);
        case 2: return quad_bcast<2>(x);
        default: return quad_bcast<3>(x);
        }
    };
    // value code r (of the lane's NROUND_V) of token v of the k-group
    auto win_field_v = [&](const unsigned (&w)[VW], int v, int r) -> unsigned {
        constexpr auto bits_c = std::integral_constant<int, BV>{};
        constexpr auto log2e_c = std::integral_constant<int, DVR == 8 ? 4 : 3>{};   // bytes of a table entry
        if constexpr (!WV) return 0u;
        else if constexpr (WIN_V == 2) return field2(quad_get(w[0], v), quad_get(w[1], v), pos_v + BV * r, bits_c, log2e_c);
        else {
            // (the lane's run, NROUND_V codes, fits one dword)
            unsigned o[3];
            align3(quad_get(w[0], v), quad_get(w[1], v), quad_get(w[2], v), pos_v, o, std::integral_constant<int, 1>{});
            return const_field(o, BV * r, bits_c, log2e_c);
        }
    };
    auto gather_v = [&](const Codes &cd, int st, int q) -> half8 {
        if constexpr (WV && DV == 8) {
            // q = token v of the k-group: the 8 channels of sub-space col of that token
            return __builtin_bit_cast(half8, lds_load_b128(lds_v + win_field_v(cd.vc[st], q, 0)));
        } else if constexpr (WV) {
            // q = 2 u + r: sub-space 2 col + r of tokens 2u, 2u + 1
            const int u = q / NROUND_V, r = q % NROUND_V;
            const uint2 x0 = lds_load_b64(lds_v + win_field_v(cd.vc[st], 2 * u, r));
            const uint2 x1 = lds_load_b64(lds_v + win_field_v(cd.vc[st], 2 * u + 1, r));
            return as_half8(x0.x, x0.y, x1.x, x1.y);
        } else if constexpr (DV == 8) {
            // q = token v of the k-group: the 8 channels of sub-space col of that token
            return __builtin_bit_cast(half8, lds_load_b128(lds_addr_v(cd.vc[st][0], q, lds_v)));
        } else if (DV == 4) {
            const int u = q / NROUND_V, r = q % NROUND_V;
            const int b0 = 2 * u * NROUND_V + r, b1 = (2 * u + 1) * NROUND_V + r;
            const uint2 x0 = lds_load_b64(lds_addr_v(cd.vc[st][b0 >> 2], b0 & 3, lds_v) + r * PLANE_V);
            const uint2 x1 = lds_load_b64(lds_addr_v(cd.vc[st][b1 >> 2], b1 & 3, lds_v) + r * PLANE_V);
            return as_half8(x0.x, x0.y, x1.x, x1.y);
        } else {
            unsigned x[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int bi = v * NROUND_V + q;
                x[v] = lds_load_b32(lds_addr_v(cd.vc[st][bi >> 2], bi & 3, lds_v) + q * PLANE_V);
            }
            return as_half8(x[0], x[1], x[2], x[3]);
        }
    };

    half8 ka[4 * H];                 // score operands of the first H rounds of the tile about to be processed
    // One tile, as five stages.  In every stage but the softmax the matrix cores work on
    // operands gathered in the previous stage while the vector ALU forms the addresses of, and
    // LDS serves, the gathers of the next one; the scheduling hints interleave the three
    // instruction kinds so that each MFMA's 16 busy cycles are filled:
    //   1  MFMA K first H rounds  | gather K last H rounds          (H = 2 at D = 128, 1 at D = 64)
    //   2  MFMA K last H rounds   | gather V sub-tiles 0-1
    //   3  online softmax         | gather V sub-tiles 2-3 (issued first, lands under the softmax)
    //   4  MFMA P.V sub-tiles 0-1 | gather K first H rounds of the NEXT tile
    //   5  MFMA P.V sub-tiles 2-3
    // A tile's key-code registers are refilled from HBM (with the codes of the tile two ahead) at the
    // end of stage 1, its value-code registers at the start of stage 3: right after their last use,
    // which gives the loads the longest run-up the two register sets allow (1.1 - 1.6 us less per
    // call at 196608 tokens than refilling both in stage 5; a third register set measured slower).
    // Every stage pairs 4 H MFMAs with 4 H operand gathers.
    constexpr int kReadsK = 8 / DK;                   // ds_reads (and address ops) per gathered half8
    constexpr int kReadsV = 8 / DV;
    // H groups of: the address (and other vector-ALU) ops of four operand gathers, then four
    // rounds of MFMAs, then the four gathers' LDS reads.  The address op (v_dot4) needs a few wait
    // states before an LDS instruction may read its result: with the MFMAs in between they are
    // free, and groups of four measured 1 us per call faster than alternating one by one.
#define VI_GROUPS8(MF, RD, XV)                                                             \
    _Pragma("unroll") for (int gi = 0; gi < H; ++gi) {                                        \
        __builtin_amdgcn_sched_group_barrier(0x002, 4 * ((RD) + (XV)), 0);                  \
        __builtin_amdgcn_sched_group_barrier(0x008, 4 * (MF), 0);                           \
        __builtin_amdgcn_sched_group_barrier(0x100, 4 * (RD), 0);                           \
    }
    auto process_tile = [&](Codes &cd, const Codes &next, long long tb, long long tb_refill) {
        half8 kb[4 * H], va[2 * NR], vb[2 * NR];
        const floatx4 kZero4 = {0.f, 0.f, 0.f, 0.f};
        floatx4 sacc[HG][4 / NQ];              // split query: set a holds sub-tiles 2a, 2a + 1
        // (sub-tiles in the order 0, 2, 1, 3: consecutive MFMAs accumulate in different sets)
        auto st_of = [](int i) { return NQ == 2 ? (i & 1) * 2 + (i >> 1) : i; };

        // ---- stage 1
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int hr = 0; hr < H; ++hr)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int st = st_of(i), a = st / NQ, c = st % NQ;
#pragma unroll
                for (int hg = 0; hg < HG; ++hg)
                    sacc[hg][a] = MFMA16(ka[H * st + hr], bq[hg][c][hr], hr == 0 && c == 0 ? kZero4 : sacc[hg][a], 0, 0, 0);
                kb[H * st + hr] = gather_k(cd, st, H + hr);
            }
        VI_GROUPS8(HG, kReadsK, 0)
        load_codes_k(cd, tb_refill);              // this tile's key codes are consumed: refill them (two tiles ahead)
        __builtin_amdgcn_sched_barrier(0);

        // ---- stage 2
#pragma unroll
        for (int hr = 0; hr < H; ++hr)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int st = st_of(i), a = st / NQ, c = st % NQ;
#pragma unroll
                for (int hg = 0; hg < HG; ++hg)
                    sacc[hg][a] = MFMA16(kb[H * st + hr], bq[hg][c][H + hr], sacc[hg][a], 0, 0, 0);
                va[4 * hr + i] = gather_v(cd, (4 * hr + i) / NR, (4 * hr + i) % NR);   // sub-tiles 0, 1
            }
        VI_GROUPS8(HG, kReadsV, 0)
        __builtin_amdgcn_sched_barrier(0);

        // ---- stage 3: online softmax of this wavefront (Alg. 1 steps 12-13).
        // The four lanes of a quad (same head, t0 = 0..3) hold identical copies of all 16 scores
        // of their row group.  Lane t0 keeps only sub-tile t0's four, so the quad does each
        // exp once; the P.V operand build below fetches them back across the quad with DPP.
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            vb[q] = gather_v(cd, 2, q);
            vb[NR + q] = gather_v(cd, 3, q);
        }
        load_codes_v(cd, tb_refill);              // this tile's value codes are consumed
        __builtin_amdgcn_sched_barrier(0);
        unsigned pp[HG][4];                      // (p, p) as fp16 pairs, tokens 4v + kg of sub-tile t0
#pragma unroll
        for (int hg = 0; hg < HG; ++hg) {
            // Branch-free per-lane pick with bit masks (v_bfi_b32 / v_cndmask).  With the split query,
            // columns t0 < 2 carry q~_hi . k and columns t0 >= 2 carry q~_lo . k, and a lane's two
            // register sets hold its part of sub-tiles t0 % 2 and 2 + t0 % 2: it keeps the one of
            // sub-tile t0 (`mine`) and hands the other - its part of sub-tile t0 ^ 2, which the lane
            // two further on keeps - across the quad (`theirs`), so that one DPP add per score
            // restores the full precision: 3 operations per score.  (Two head groups: one register
            // set per sub-tile, `mine` and `theirs` picked among four.)
            auto bfi = [](unsigned m, unsigned a, unsigned b) -> unsigned { return (m & a) | (~m & b); };
            float sc[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if constexpr (NQ == 2) {
                    const unsigned lower = __float_as_uint(sacc[hg][0][v]), upper = __float_as_uint(sacc[hg][1][v]);
                    const unsigned up = sel[2] | sel[3];                   // all ones iff t0 >= 2
                    const unsigned mine = bfi(up, upper, lower), theirs = bfi(up, lower, upper);
                    sc[v] = __uint_as_float(mine) + quad_xor<2>(__uint_as_float(theirs));
                } else {
                    const unsigned s0 = __float_as_uint(sacc[hg][0][v]), s1 = __float_as_uint(sacc[hg][1][v]);
                    const unsigned s2 = __float_as_uint(sacc[hg][2 % (4 / NQ)][v]), s3 = __float_as_uint(sacc[hg][3 % (4 / NQ)][v]);
                    const unsigned mine = bfi(sel[3], s3, bfi(sel[2], s2, bfi(sel[1], s1, s0)));
                    if (SPLITQ) {
                        const unsigned theirs = bfi(sel[1], s3, bfi(sel[0], s2, bfi(sel[3], s1, s0)));
                        sc[v] = __uint_as_float(mine) + quad_xor<2>(__uint_as_float(theirs));
                    } else {
                        sc[v] = __uint_as_float(mine);
                    }
                }
            }
            if (tb + kTile > n1) {                  // tail tile: tokens past the end get p = 0
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (tb + 16 * t0 + 4 * v + kg > last) sc[v] = -INFINITY;
            }
            float tmax = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
            tmax = fmaxf(tmax, quad_xor<1>(tmax));
            tmax = fmaxf(tmax, quad_xor<2>(tmax));
            tmax = rows_max(tmax);
            const float m_new = fmaxf(m_run[hg], tmax);
            if (__any(m_new > m_run[hg])) {
                const float alpha = __builtin_amdgcn_exp2f(m_run[hg] - m_new);   // 0 on the first tile
                l_part[hg] *= alpha;
                const float alpha_o = __shfl(alpha, 4 * kg);                     // lane 4kg serves head kg
#pragma unroll
                for (int r = 0; r < NACC; ++r) acc_o[hg][r] *= alpha_o;
                m_run[hg] = m_new;
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float pr = __builtin_amdgcn_exp2f(sc[v] - m_run[hg]);
                l_part[hg] += pr;
                pp[hg][v] = pack_dup_f16(pr);          // (p, p) as two fp16, round-to-nearest-even: one v_cvt_pk_f16_f32
            }
        }

        // ---- o += P . VQ^-1(V_q)  (step 16)
        auto pv = [&](auto st_c, const half8 *vops) {
            constexpr int st = decltype(st_c)::value;
#pragma unroll
            for (int hg = 0; hg < HG; ++hg) {
                // p of sub-tile st lives in quad lane st
                const unsigned p0 = quad_bcast<st>(pp[hg][0]), p1 = quad_bcast<st>(pp[hg][1]);
                const unsigned p2 = quad_bcast<st>(pp[hg][2]), p3 = quad_bcast<st>(pp[hg][3]);
                if constexpr (DV == 8) {
                    // one token per step; channels t0 (first accumulator) and t0 + 4 (second).
                    // (Two tokens per MFMA as at d = 4, with the halves of a centroid gathered apart,
                    // halve the MFMAs but double the LDS reads: 1.5 us slower per call with 8-bit
                    // codes, 6 us with a shared table, whose reads meet at random banks.)
                    const unsigned pt[4] = {p0, p1, p2, p3};
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const half8 alo = as_half8(pt[v] & mask_a, pt[v] & mask_b, 0u, 0u);
                        const half8 ahi = as_half8(0u, 0u, pt[v] & mask_a, pt[v] & mask_b);
                        acc_o[hg][0] = MFMA16(alo, vops[v], acc_o[hg][0], 0, 0, 0);
                        acc_o[hg][1] = MFMA16(ahi, vops[v], acc_o[hg][1], 0, 0, 0);
                    }
                } else if (DV == 4) {
                    const half8 a0 = as_half8(p0 & mask_a, p0 & mask_b, p1 & mask_a, p1 & mask_b);
                    const half8 a1 = as_half8(p2 & mask_a, p2 & mask_b, p3 & mask_a, p3 & mask_b);
#pragma unroll
                    for (int r = 0; r < NROUND_V; ++r) acc_o[hg][r] = MFMA16(a0, vops[r], acc_o[hg][r], 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < NROUND_V; ++r)
                        acc_o[hg][r] = MFMA16(a1, vops[NROUND_V + r], acc_o[hg][r], 0, 0, 0);
                } else {
                    const half8 a = as_half8(p0 & mask_a, p1 & mask_a, p2 & mask_a, p3 & mask_a);
#pragma unroll
                    for (int r = 0; r < NROUND_V; ++r)
                        acc_o[hg][r] = MFMA16(a, vops[r], acc_o[hg][r], 0, 0, 0);
                }
            }
        };
        // ---- stage 4
        __builtin_amdgcn_sched_barrier(0);
        pv(std::integral_constant<int, 0>{}, va);
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int hr = 0; hr < H; ++hr) ka[H * st + hr] = gather_k(next, st, hr);
        pv(std::integral_constant<int, 1>{}, va + NR);
#pragma unroll
        for (int st = 2; st < 4; ++st)
#pragma unroll
            for (int hr = 0; hr < H; ++hr) ka[H * st + hr] = gather_k(next, st, hr);
        VI_GROUPS8(HG * (DV == 8 ? 2 : 1), kReadsK, 3 * HG)
        __builtin_amdgcn_sched_barrier(0);

        // ---- stage 5
        pv(std::integral_constant<int, 2>{}, vb);
        pv(std::integral_constant<int, 3>{}, vb + NR);
        __builtin_amdgcn_sched_barrier(0);
    };
#undef VI_GROUPS8

    // Two tiles of codes in flight: a tile's registers are refilled (two tiles ahead) as soon as
    // the last gather that uses them has been issued.  Loads past the end of the split return code 0 (buffer
    // range check), so the refill and the look-ahead gathers need no bounds branch.
    {
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int hr = 0; hr < H; ++hr) ka[H * st + hr] = gather_k(ca, st, hr);
        // a wavefront's tile bases increase with k: once one is past the end, all later ones are
        long long ta = tile_base(0), tb = tile_base(1);
        for (int k = 2; ta < n1; k += 2) {
            const long long tc = tile_base(k), td = tile_base(k + 1);
            process_tile(ca, cb, ta, tc);
            if (tb < n1) process_tile(cb, ca, tb, td);
            ta = tc;
            tb = td;
        }
    }

    // 8-bit codes: the new token's items come after the wavefront's tiles.  The wavefronts that take
    // them (the first ones of the workgroup) are the ones that finish their tiles first, so the
    // items fill time in which the workgroup waits for its slower wavefronts anyway; the tables are
    // still in LDS until the barrier below.
    if (has_new) {
        if constexpr (!WK) items8(std::integral_constant<int, 0>{});
        if constexpr (!WV) items8(std::integral_constant<int, 1>{});
    }
    // ---- merge the wavefronts of this split through LDS (the codebooks are no longer needed)
    float l_head[HG];
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
        l_head[hg] = l_part[hg] + quad_xor<1>(l_part[hg]);
        l_head[hg] += quad_xor<2>(l_head[hg]);
        l_head[hg] += __shfl_xor(l_head[hg], 16);
        l_head[hg] += __shfl_xor(l_head[hg], 32);
    }
    // A single split folds the fused new token in below.  Its score shares and dequantized value
    // sit in the scratch behind the tables, and with small shared tables (10-bit codes on both
    // sides, two head groups) the wavefronts' partials written next reach into that scratch:
    // every thread takes what it will need into registers first.
    constexpr int kMergeIters = (KG * kD + BLOCK - 1) / BLOCK;
    const bool fold_new = S_ == 1 && !p.k_res && has_new;
    float new_s[kMergeIters], new_val[kMergeIters];
    if (fold_new) {
        __syncthreads();                                   // the items' scratch writes
#pragma unroll
        for (int i = 0; i < kMergeIters; ++i) {
            const int e = tid + i * BLOCK, hh = e / kD, c = e % kD;
            new_s[i] = 0.f;
            new_val[i] = 0.f;
            if (e < G_ * kD) {
                for (int m = 0; m < MK; ++m) new_s[i] += sm_nsc[m * KG + hh];
                new_val[i] = sm_nv[c];
            }
        }
    }
    __syncthreads();
    float *const sm_o = reinterpret_cast<float *>(smem);                  // [NW][KG][D]
    float *const sm_m = sm_o + NW * KG * kD;                              // [NW][KG]
    float *const sm_l = sm_m + NW * KG;                                   // [NW][KG]
#pragma unroll
    for (int hg = 0; hg < HG; ++hg) {
        // acc_o[hg][r] register v of lane (col, kg): head 4 hg + kg, channel kChanBlock * (NACC * col + r) + v
#pragma unroll
        for (int r = 0; r < NACC; ++r)
#pragma unroll
            for (int v = 0; v < kChanBlock; ++v)
                sm_o[(wave * KG + kG * hg + kg) * kD + kChanBlock * (NACC * col + r) + v] = acc_o[hg][r][v];
        if (kg == 0 && (col & 3) == 0) {
            sm_m[wave * KG + kG * hg + (col >> 2)] = m_run[hg];
            sm_l[wave * KG + kG * hg + (col >> 2)] = l_head[hg];
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kMergeIters; ++it) {
        const int e = tid + it * BLOCK;
        if (e >= G_ * kD) break;
        const int hh = e / kD, c = e % kD;
        float mx = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) mx = fmaxf(mx, sm_m[w * KG + hh]);
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = sm_m[w * KG + hh];
            const float f = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - mx) : 0.f;
            o += f * sm_o[w * KG * kD + e];
            l += f * sm_l[w * KG + hh];
        }
        if (S_ == 1 && !p.k_res) {
            // the workgroup holds the whole answer (a single split also encoded every sub-space of
            // a fused new token): fold the new token in and write the output rows
            if (has_new) {
                const float s_new = new_s[it];
                const float mt = fmaxf(mx, s_new);
                const float f = __builtin_amdgcn_exp2f(mx - mt), wgt = __builtin_amdgcn_exp2f(s_new - mt);
                o = f * o + wgt * new_val[it];
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

template <int kD, int DK, int DV, int HG, int NW, bool SPLITQ, int BK, int BV, bool VT>
int launch_hg(const DecodeParams &p, hipStream_t stream)
{
    constexpr int KG = kG * HG;
    constexpr size_t cbk = BK > 8 ? ((size_t)1 << BK) * DK * 2 : (size_t)kCentroids * kD * 2;
    constexpr size_t cbv = BV > 8 ? ((size_t)1 << BV) * DV * 2 : (size_t)kCentroids * kD * 2;
    // the tables, q~ and the new token's scratch during the tile loop; the wavefronts' partials after it
    constexpr size_t loop_bytes = cbk + cbv + sizeof(float) * ((KG + 3) * kD + (kD / DK) * KG) + 8 * 4 * NW + 16;
    constexpr size_t merge_bytes = sizeof(float) * (NW * KG * kD + 2 * NW * KG);
    constexpr size_t smem = loop_bytes > merge_bytes ? loop_bytes : merge_bytes;
    // once per process and instantiation (function-local static: initialised thread-safely)
    static const bool configured = [] {
        const void *fn = reinterpret_cast<const void *>(decode_mfma_kernel<kD, DK, DV, HG, NW, SPLITQ, BK, BV, VT>);
        // (the kernel takes the dynamic segment to start at LDS offset 0: no static LDS in front of it)
        hipFuncAttributes attr;
        if (hipFuncGetAttributes(&attr, fn) != hipSuccess || attr.sharedSizeBytes != 0) return false;
        return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    }();
    if (!configured) return -4;
    dim3 grid(p.S, p.Hkv, p.B);
    hipLaunchKernelGGL((decode_mfma_kernel<kD, DK, DV, HG, NW, SPLITQ, BK, BV, VT>), grid, dim3(NW * 64), smem, stream,
                       p.q, p.lam, p.cb_k, p.cb_v, p.k_new, p.v_new, (unsigned)p.Hkv | (unsigned)p.G << 24, p.S, p);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

template <int kD, int DK, int DV, int NW, bool SPLITQ, int BK = 8, int BV = 8, bool VT = false>
int launch_typed(const DecodeParams &p, hipStream_t stream)
{
    return p.G <= kG ? launch_hg<kD, DK, DV, 1, NW, SPLITQ, BK, BV, VT>(p, stream)
                     : launch_hg<kD, DK, DV, 2, NW, SPLITQ, BK, BV, VT>(p, stream);
}

} // namespace

} // namespace vecinfer
