// Nearest-centroid search (Eq. 2) of the tiled cache-fill and K-Means kernels: a matrix-core screen
// followed by the exact comparison.
//
// What is written is, bit for bit, what the plain search writes: the centroid with the smallest
// squared distance, summed directly in fp32 in channel order, lowest index among equals.  The
// matrix cores only tell which centroids can possibly be that one:
//   score(c) = sigma (x . c - |c|^2 / 2)      (largest score <=> smallest distance)
// for the 64 tokens of a tile against the 256 centroids of a sub-space, as
// v_mfma_f32_32x32x16_f16 products: rows = 32 centroids, columns = 32 tokens, and along k
//   [ c          | c          | -sigma |c|^2 / 2 as two fp16 parts ]   (A)
//   [ hi(sigma x)| lo(sigma x)| 1 1                               ]   (B)
// (hi + lo: sigma x to 22 bits; the centroids are fp16 already; sigma, a power of two per
// sub-space, keeps the low parts out of the fp16 denormal range).  The screen's error is bounded
// (below), so every centroid that can win or tie has a score within `margin` of the best one.
// A lane keeps, of the 128 scores it sees per token, only their maxima over the 16 registers of
// each MFMA (8 "blocks") and over the 8 MFMAs for each register (16 "groups"): a score within the
// margin marks its block and its group, so the (few, normally one) marked pairs are a superset
// of the centroids that matter, and only those get the exact distance.
//
// Error bound, in score units (T = sum_j |x_j| max|c_j| + max|c|^2 / 2 bounds the sum of the
// magnitudes of a score's terms):
//   split of sigma x          <= 2^-22 sigma T        fp32 |c|^2 and its two parts   <= 2^-20.2 sigma T
//   fp32 accumulation of <= 18 products, every addition taken as truncating (2^-23): <= 2^-18.8 sigma T
//   (10 products and 2^-19.7 at d = 4; a matrix core that rounds once per instruction is far below this)
//   fp16 parts below 2^-14 taken as flushed to zero: <= 2^-14 (d max|c_j| + 3), whatever sigma
//   two scores compared: twice the sum, 2^-17.25 sigma T + 2^-13 (d max|c_j| + 3) < the margin's first terms
//   the exact distances themselves carry (d + 2) 2^-24 relative rounding each; a centroid is
//   safely worse when its true distance exceeds the best's by 2^-18.9 times the best distance
//   (<= 2 (|x|^2 + max|c|^2)), i.e. by 2^-18 sigma (|x|^2 + max|c|^2) in score units.
// margin = sigma (2^-17 T + 2^-18 (|x|^2 + max|c|^2)) + 2^-13 (d max|c_j| + 3).
// A token whose scaled sub-vector leaves the fp16 range (or holds an infinity or a NaN) has no
// finite best score, a sub-space whose |c|^2 does not fit gets a NaN sigma: either way the
// wavefront falls back to the plain search for that tile.
#pragma once
#include "common.h"

namespace vecinfer {

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// LDS tables of one codebook of C centroids: plane 0 = the fp16 centroids as MFMA A operands want
// them (d = 2: each twice, d = 4: 8 bytes, d = 8: 16 bytes), plane 1 = -sigma |c|^2 / 2 as {hi, lo};
// 16 spare bytes, so that an 8-byte read of the last plane-1 entry stays inside.
// C = 256: the codebook of one sub-space (8-bit codes); C = 2^b: the one codebook a KV head's
// sub-spaces share (10- / 12-bit codes), searched 256 centroids ("chunk") at a time.
template <int d, int C = kCentroids>
struct ScreenTab {
    static constexpr int kCenBytes = d == 8 ? 16 : 8;
    static constexpr int kPlane0 = C * kCenBytes;
    static constexpr int kBytes = kPlane0 + C * 4 + 16;
};

struct ScreenConsts {
    float sigma, cmax, nmax;
};

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// sigma: the power of two that brings max |c|^2 / 2 to about 2^10 (within 2^-14 .. 2^14).
// Centroids too large for the fp16 parts of -sigma |c|^2 / 2 (or not finite): no screen for this
// codebook; a NaN sigma makes every margin NaN, which sends every tile to the plain search.
__device__ __forceinline__ float screen_sigma(float nm)
{
    int e = 9 - ilogbf(fmaxf(0.5f * nm, 1e-30f));
    e = e < -14 ? -14 : (e > 14 ? 14 : e);
    const float sigma = ldexpf(1.0f, e);
    return 0.5f * sigma * nm < 60000.0f ? sigma : __builtin_nanf("");
}

template <int d>
__device__ __forceinline__ void screen_store_norm(unsigned char *plane1, int c, float sigma, float n)
{
    const float v = -0.5f * sigma * n;
    const _Float16 hi = (_Float16)v;
    const f16x2 h = {hi, (_Float16)(v - (float)hi)};
    *reinterpret_cast<f16x2 *>(plane1 + c * 4) = h;
}

// Plane-0 entry of centroid c from its fp16 values; returns |c|^2 (fp32) and folds max |c_j| into cm.
template <int d>
__device__ __forceinline__ float screen_store_centroid(const __half *src, unsigned char *tab, int c, float &cm)
{
    typedef _Float16 f16xd __attribute__((ext_vector_type(d)));
    const f16xd raw = *reinterpret_cast<const f16xd *>(src + (size_t)c * d);
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < d; ++j) {
        const float v = (float)raw[j];
        s = fmaf(v, v, s);
        cm = fmaxf(cm, fabsf(v));
    }
    if constexpr (d == 2) {
        const f16x4 h = {raw[0], raw[1], raw[0], raw[1]};
        *reinterpret_cast<f16x4 *>(tab + c * 8) = h;
    } else {
        *reinterpret_cast<f16xd *>(tab + c * (2 * d)) = raw;
    }
    return s;
}

// Tables of one sub-space's codebook `src` [256][d] fp16 (in memory), built by one wavefront: the
// one that searches the sub-space.
template <int d>
__device__ __forceinline__ ScreenConsts screen_prepare(const __half *src, unsigned char *tab, int lane)
{
    float n[4], cm = 0.f, nm = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        n[i] = screen_store_centroid<d>(src, tab, lane + 64 * i, cm);
        nm = fmaxf(nm, n[i]);
    }
    cm = wave_max(cm);
    nm = wave_max(nm);
    const float sigma = screen_sigma(nm);
#pragma unroll
    for (int i = 0; i < 4; ++i) screen_store_norm<d>(tab + ScreenTab<d>::kPlane0, lane + 64 * i, sigma, n[i]);
    if (lane < 4) *reinterpret_cast<unsigned *>(tab + ScreenTab<d>::kBytes - 16 + 4 * lane) = 0u;   // the spare bytes
    return ScreenConsts{sigma, cm, nm};
}

// Tables of a shared codebook `src` [C][d] fp16, built by the whole workgroup of BLOCK threads
// (`red_s`: 2 BLOCK / 64 floats of LDS scratch).  Ends with a barrier: the tables are complete.
template <int d, int C, int BLOCK>
__device__ __forceinline__ ScreenConsts screen_prepare_shared(const __half *src, unsigned char *tab, float *red_s)
{
    constexpr int PER = C / BLOCK, NW = BLOCK / 64;
    static_assert(C % BLOCK == 0, "whole rounds");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float n[PER], cm = 0.f, nm = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        n[i] = screen_store_centroid<d>(src, tab, tid + BLOCK * i, cm);
        nm = fmaxf(nm, n[i]);
    }
    cm = wave_max(cm);
    nm = wave_max(nm);
    if (lane == 0) {
        red_s[wave] = cm;
        red_s[NW + wave] = nm;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        cm = fmaxf(cm, red_s[w]);
        nm = fmaxf(nm, red_s[NW + w]);
    }
    const float sigma = screen_sigma(nm);
#pragma unroll
    for (int i = 0; i < PER; ++i) screen_store_norm<d>(tab + ScreenTab<d, C>::kPlane0, tid + BLOCK * i, sigma, n[i]);
    if (tid < 4) *reinterpret_cast<unsigned *>(tab + ScreenTab<d, C>::kBytes - 16 + 4 * tid) = 0u;        // the spare bytes
    __syncthreads();
    return ScreenConsts{sigma, cm, nm};
}

// Bits of the squared distance of x to centroid c of the codebook whose tables are `tab`: the
// fp16 centroid widened (exact), differences squared and summed in channel order in fp32.
template <int d>
__device__ __forceinline__ unsigned screen_dist_bits(const float (&x)[d], const unsigned char *tab, int c)
{
    typedef _Float16 f16xd __attribute__((ext_vector_type(d)));
    const f16xd cen = *reinterpret_cast<const f16xd *>(tab + c * ScreenTab<d>::kCenBytes);
    float dist = 0.f;
#pragma unroll
    for (int j = 0; j < d; ++j) {
        const float t = x[j] - (float)cen[j];
        dist = fmaf(t, t, dist);
    }
    return __float_as_uint(dist);
}

// The plain search of one token's sub-vector x over the C centroids (the same address in every
// lane: broadcast reads): groups of 8, the group minimum against the running best (strict "<":
// the earliest group wins), the winning group re-evaluated for the lowest index at the minimum.
template <int d, int C = kCentroids>
__device__ __forceinline__ void plain_search(const float (&x)[d], const unsigned char *tab, int &arg_out,
                                             unsigned &best_out)
{
    unsigned best = 0x7f800000u;            // +inf
    int best_group = 0;
#pragma unroll 2
    for (int c0 = 0; c0 < C; c0 += 8) {
        unsigned gmin = screen_dist_bits<d>(x, tab, c0);
#pragma unroll
        for (int k = 1; k < 8; ++k) {
            const unsigned v = screen_dist_bits<d>(x, tab, c0 + k);
            gmin = v < gmin ? v : gmin;
        }
        if (gmin < best) {
            best = gmin;
            best_group = c0;
        }
    }
    int arg = best_group;
#pragma unroll
    for (int k = 7; k >= 0; --k)
        if (screen_dist_bits<d>(x, tab, best_group + k) == best) arg = best_group + k;
    arg_out = arg;
    best_out = best;
}

// B operands and margins of tokens col (cb = 0) and 32 + col (cb = 1) of the tile.
template <int d>
struct ScreenOperands {
    f16x8 b1[2], b2[2];
    float mg[2];
};

template <int d>
__device__ __forceinline__ ScreenOperands<d> screen_operands(const float *x_s, int XS, int ch0, const ScreenConsts &k,
                                                             int h, int col)
{
    const _Float16 one = (_Float16)1.0f, zero = (_Float16)0.0f;
    const f16x8 ones = {one, one, zero, zero, zero, zero, zero, zero};
    const f16x8 zeros = {zero, zero, zero, zero, zero, zero, zero, zero};
    ScreenOperands<d> o;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        float x[d], l1 = 0.f, l2 = 0.f;
        _Float16 hi[d], lo[d];
#pragma unroll
        for (int j = 0; j < d; ++j) {
            x[j] = x_s[(32 * cb + col) * XS + ch0 + j];
            l1 += fabsf(x[j]);
            l2 = fmaf(x[j], x[j], l2);
            const float xs = x[j] * k.sigma;
            hi[j] = (_Float16)xs;
            lo[j] = (_Float16)(xs - (float)hi[j]);
        }
        o.mg[cb] = k.sigma * (0x1p-17f * (l1 * k.cmax + 0.5f * k.nmax) + 0x1p-18f * (l2 + k.nmax)) +
                   0x1p-13f * ((float)d * k.cmax + 3.0f);
        f16x8 v;
        o.b2[cb] = zeros;
        if constexpr (d == 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = h ? lo[j] : hi[j];
            o.b2[cb] = h ? zeros : ones;
        } else if constexpr (d == 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[j] = h ? ones[j] : hi[j];
                v[4 + j] = h ? zero : lo[j];
            }
        } else {
            v = zeros;
            v[0] = h ? one : hi[0];
            v[1] = h ? one : hi[1];
            v[2] = h ? zero : lo[0];
            v[3] = h ? zero : lo[1];
        }
        o.b1[cb] = v;
    }
    return o;
}

// Scores of the tile's 64 tokens against the 256 centroids row0 .. row0 + 255 of the codebook at
// `tab` (plane 1 at tab + plane1), 2 x 32 centroids at a time; out: their maxima per block (MFMA)
// and per group (accumulator register), for cb = 0, 1.
// kRolled: the four pairs of blocks as iterations of a real loop (the block maxima move up two
// places per iteration, so that no register is indexed by the loop counter).  Unrolled, the
// compiler is free to issue all 16 MFMAs first; inside the chunk loop of a shared codebook it does,
// and their 256 result registers spill (d8b12 cache fill 7.0 ms against 3.4 ms rolled); for a single
// chunk (8-bit codes) the unrolled form is 2 - 5 % faster.
template <int d, bool kRolled = false>
__device__ __forceinline__ void screen_chunk(const unsigned char *tab, int plane1, int row0, int h, int col,
                                             const ScreenOperands<d> &o, float (&bm)[2][8], float (&gm)[2][16])
{
    const _Float16 zero = (_Float16)0.0f;
    const f16x8 zeros = {zero, zero, zero, zero, zero, zero, zero, zero};
    const f32x16 z16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) gm[cb][r] = -INFINITY;
    if constexpr (kRolled) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 8; ++r) bm[cb][r] = -INFINITY;
    }
    constexpr int kUnroll = kRolled ? 1 : 4;
#pragma unroll kUnroll
    for (int rp = 0; rp < 4; ++rp) {
        f16x8 a1[2], a2[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int row = row0 + 32 * (2 * rp + u) + col;
            a2[u] = zeros;
            if constexpr (d == 8) {
                a1[u] = *reinterpret_cast<const f16x8 *>(tab + row * 16);
                const f16x2 nn = *reinterpret_cast<const f16x2 *>(tab + plane1 + row * 4);
                a2[u][0] = nn[0];
                a2[u][1] = nn[1];
            } else {
                // lanes 0-31: the centroid (8 bytes); lanes 32-63: the 4 bytes of plane 1, read as 8.
                // What lanes 32-63 get beyond their two halves meets zeros in the B operand, and it
                // is finite (entries of plane 1, or its zeroed spare bytes), so it adds nothing.
                const f16x4 rd = *reinterpret_cast<const f16x4 *>(tab + (h ? plane1 + row * 4 : row * 8));
                a1[u] = zeros;
#pragma unroll
                for (int j = 0; j < 4; ++j) a1[u][j] = rd[j];
                if constexpr (d == 4) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) a1[u][4 + j] = rd[j];
                }
            }
        }
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            f32x16 v[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                v[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[u], o.b1[cb], z16, 0, 0, 0);
                if constexpr (d == 8) v[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2[u], o.b2[cb], v[u], 0, 0, 0);
                float m = fmaxf(v[u][0], v[u][1]);
#pragma unroll
                for (int r = 2; r < 16; r += 2) m = fmaxf(fmaxf(m, v[u][r]), v[u][r + 1]);
                if constexpr (kRolled) {
                    if (u == 0) {
#pragma unroll
                        for (int r = 0; r < 6; ++r) bm[cb][r] = bm[cb][r + 2];
                    }
                    bm[cb][6 + u] = m;
                } else {
                    bm[cb][2 * rp + u] = m;
                }
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) gm[cb][r] = fmaxf(fmaxf(gm[cb][r], v[0][r]), v[1][r]);
        }
    }
}

__device__ __forceinline__ float screen_max8(const float (&bm)[8])
{
    float best = fmaxf(bm[0], bm[1]);
#pragma unroll
    for (int r = 2; r < 8; r += 2) best = fmaxf(fmaxf(best, bm[r]), bm[r + 1]);
    return best;
}

// A maximum above thr marks its block / group: the sign bit of thr - maximum, shifted into the
// mask (one subtraction and one v_alignbit each).  Bits 0-7: blocks, bits 8-23: groups.
__device__ __forceinline__ unsigned screen_marks(const float (&bm)[8], const float (&gm)[16], float thr)
{
    unsigned m = 0;
#pragma unroll
    for (int r = 15; r >= 0; --r) m = __builtin_amdgcn_alignbit(m, __float_as_uint(thr - gm[r]), 31);
#pragma unroll
    for (int r = 7; r >= 0; --r) m = __builtin_amdgcn_alignbit(m, __float_as_uint(thr - bm[r]), 31);
    return m;
}

// Exact distances of the centroids that `marks` (of the half hh of the wavefront, for the 256
// centroids from row0) points at; (best, arg) keeps the smallest (distance bits, index).
template <int d>
__device__ __forceinline__ void screen_eval(const float (&x)[d], const unsigned char *tab, int row0, unsigned marks,
                                            int hh, unsigned &best, int &arg)
{
    unsigned mb = marks & 0xffu;
    const unsigned mgp = (marks >> 8) & 0xffffu;
    while (mb) {
        const int rb = __builtin_ctz(mb);
        mb &= mb - 1;
        unsigned gg = mgp;
        while (gg) {
            const int r = __builtin_ctz(gg);
            gg &= gg - 1;
            const int c = row0 + 32 * rb + 8 * (r >> 2) + 4 * hh + (r & 3);   // row of register r of block rb
            const unsigned dist = screen_dist_bits<d>(x, tab, c);
            if (dist < best || (dist == best && c < arg)) {
                best = dist;
                arg = c;
            }
        }
    }
}

// The wavefront's 64 tokens (rows of x_s, channels ch0 .. ch0 + d) against the sub-space whose
// tables are `tab`.  Returns the code of token `lane` and the bits of its squared distance; false
// if the screen marked nothing for some token of the wavefront (the caller then runs the plain
// search; same for every lane).
template <int d>
__device__ __forceinline__ bool screen_search(const float *x_s, int XS, int ch0, const unsigned char *tab,
                                              const ScreenConsts &k, int lane, int &arg_out, unsigned &best_out)
{
    const int h = lane >> 5, col = lane & 31;
    const ScreenOperands<d> o = screen_operands<d>(x_s, XS, ch0, k, h, col);
    float bm[2][8], gm[2][16];
    screen_chunk<d>(tab, ScreenTab<d>::kPlane0, 0, h, col, o, bm, gm);
    // ---- blocks and groups within the margin of the token's best score (both halves of the wavefront)
    unsigned mask[2];
    bool finite[2];                        // the token's scores are numbers: the marks mean something
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        float best = screen_max8(bm[cb]);
        best = fmaxf(best, __shfl_xor(best, 32));
        const float thr = best - o.mg[cb];
        finite[cb] = fabsf(thr) < INFINITY;
        mask[cb] = screen_marks(bm[cb], gm[cb], thr);
    }
    // token `lane`: the marks of its own half of the rows, and those of the other half
    const unsigned mine = h ? mask[1] : mask[0];
    const unsigned other = __shfl_xor(h ? mask[0] : mask[1], 32);
    // ---- exact distances of the marked centroids
    float x[d];
#pragma unroll
    for (int j = 0; j < d; ++j) x[j] = x_s[lane * XS + ch0 + j];
    unsigned best = 0x7f800000u;
    int arg = 0;
    screen_eval<d>(x, tab, 0, mine, h, best, arg);
    screen_eval<d>(x, tab, 0, other, h ^ 1, best, arg);
    arg_out = arg;
    best_out = best;
    // no screen result for a token whose scaled operands left the fp16 range (infinite or NaN
    // scores), and none where nothing finite was found
    const bool mine_ok = h ? finite[1] : finite[0];
    return !__any(best == 0x7f800000u || !mine_ok);
}

// The same for a codebook of C = 2^b centroids shared by the sub-spaces, 256 centroids (a chunk)
// at a time.  Each half of the wavefront keeps, per token, the best score it has seen so far and
// the marks of at most two chunks: a chunk whose best score beats the running best by more than
// the margin replaces what was kept (nothing kept can still win), one within the margin of it is
// kept beside it (its marks taken against the better of the two), a third such chunk gives up
// (plain search for the tile; this needs three chunks within 2^-17 of each other).  Marks are
// taken against a threshold that only rises, so what is kept is a superset of the centroids
// within the margin of the final best; at the end a half whose best lies below the other
// half's threshold drops out.
template <int d, int C>
__device__ __forceinline__ bool screen_search_shared(const float *x_s, int XS, int ch0, const unsigned char *tab,
                                                     const ScreenConsts &k, int lane, int &arg_out,
                                                     unsigned &best_out)
{
    constexpr int NCH = C / kCentroids;
    static_assert(NCH >= 1 && NCH <= 64, "chunk index in 7 bits of a mark word");
    const int h = lane >> 5, col = lane & 31;
    const ScreenOperands<d> o = screen_operands<d>(x_s, XS, ch0, k, h, col);
    float run[2] = {-INFINITY, -INFINITY};
    unsigned s0[2] = {0u, 0u}, s1[2] = {0u, 0u};       // marks | chunk << 24; s1 bit 31: gave up
#pragma unroll 1
    for (int ch = 0; ch < NCH; ++ch) {
        float bm[2][8], gm[2][16];
        screen_chunk<d, true>(tab, ScreenTab<d, C>::kPlane0, ch * kCentroids, h, col, o, bm, gm);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            // (the marks are taken for every chunk: in a wavefront of 64 lanes some lane's running
            // best nearly always moves, and a branch here makes the compiler sink the group maxima
            // into it, with all 16 MFMA results live until then)
            const float cbst = screen_max8(bm[cb]);
            const bool matters = cbst >= run[cb] - o.mg[cb];
            const float nr = fmaxf(run[cb], cbst);
            const unsigned m = screen_marks(bm[cb], gm[cb], nr - o.mg[cb]) | ((unsigned)ch << 24);
            const bool replace = cbst > run[cb] + o.mg[cb];
            if (matters) {
                if (replace) {
                    s0[cb] = m;
                    s1[cb] = 0u;
                } else if (s0[cb] == 0u) {
                    s0[cb] = m;
                } else if (s1[cb] == 0u) {
                    s1[cb] = m;
                } else {
                    s1[cb] |= 0x80000000u;
                }
                run[cb] = nr;
            }
        }
    }
    bool ok[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const float thr = fmaxf(run[cb], __shfl_xor(run[cb], 32)) - o.mg[cb];
        ok[cb] = fabsf(thr) < INFINITY;
        if (run[cb] < thr) s0[cb] = s1[cb] = 0u;      // nothing in this half's rows reaches the threshold
    }
    // token `lane`: what its own half of the rows kept, and what the other half kept
    const unsigned mine0 = h ? s0[1] : s0[0], mine1 = h ? s1[1] : s1[0];
    const unsigned other0 = __shfl_xor(h ? s0[0] : s0[1], 32), other1 = __shfl_xor(h ? s1[0] : s1[1], 32);
    float x[d];
#pragma unroll
    for (int j = 0; j < d; ++j) x[j] = x_s[lane * XS + ch0 + j];
    unsigned best = 0x7f800000u;
    int arg = 0;
    screen_eval<d>(x, tab, (int)((mine0 >> 24) & 0x7fu) * kCentroids, mine0, h, best, arg);
    screen_eval<d>(x, tab, (int)((mine1 >> 24) & 0x7fu) * kCentroids, mine1, h, best, arg);
    screen_eval<d>(x, tab, (int)((other0 >> 24) & 0x7fu) * kCentroids, other0, h ^ 1, best, arg);
    screen_eval<d>(x, tab, (int)((other1 >> 24) & 0x7fu) * kCentroids, other1, h ^ 1, best, arg);
    arg_out = arg;
    best_out = best;
    const bool mine_ok = (h ? ok[1] : ok[0]) && ((mine1 | other1) & 0x80000000u) == 0u;
    return !__any(best == 0x7f800000u || !mine_ok);
}

// One wavefront, one sub-space, the 64 tokens of the tile in x_s: the screen and the exact
// distances of what it marks; the plain search when the screen gives no answer.
template <int d, int C = kCentroids>
__device__ __forceinline__ void search_tile(const float *x_s, int XS, int ch0, const unsigned char *tab,
                                            const ScreenConsts &k, int lane, int &arg, unsigned &best)
{
    if constexpr (C == kCentroids) {
        if (screen_search<d>(x_s, XS, ch0, tab, k, lane, arg, best)) return;
    } else {
        if (screen_search_shared<d, C>(x_s, XS, ch0, tab, k, lane, arg, best)) return;
    }
    float x[d];
#pragma unroll
    for (int j = 0; j < d; ++j) x[j] = x_s[lane * XS + ch0 + j];
    plain_search<d, C>(x, tab, arg, best);
}

} // namespace

} // namespace vecinfer
