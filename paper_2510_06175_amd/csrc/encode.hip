// Cache-fill kernels: key-side dual transform (Eq. 3, Eq. 6) and exhaustive nearest-centroid
// vector quantization (Eq. 2, Eq. 8).
//
// One workgroup (4 wavefronts) handles 64 tokens of one (batch, KV head).  The sub-spaces are
// searched four at a time (one per wavefront); the four codebooks are staged in LDS widened
// to fp32, one group after the other.
//   phase 1  transform: a lane owns 4 consecutive channels of one token; the first two
//            butterfly stages run inside the lane, the others across lanes with wavefront
//            shuffles.  The transformed tile is kept, as fp32, in LDS.
//            (Values skip the transform: the lane just widens its fp16 inputs.)
//   phase 2  search: a lane owns one token, a wavefront owns one sub-space at a time, so the
//            centroid under test is the same for all 64 lanes and is read from LDS as a
//            broadcast.  Squared distances are summed directly, in channel order, in fp32.
//            Centroids are scanned in groups of 8: only the group minimum is compared with
//            the running best (strict "<": the earliest group wins ties), and the winning
//            group is re-evaluated at the end to find the lowest index that attains the
//            minimum.  A non-negative fp32 orders like its bit pattern, so the minima are
//            taken on the bits (integer min: no NaN canonicalisation on the way).
//   phase 3  the 64 x M code bytes go out through LDS as whole 32-bit words.
#include "common.h"
#include "encode_screen.h"

namespace vecinfer {

namespace {

constexpr int kEncBlock = 256;
constexpr int kEncTokens = 64;     // tokens per workgroup = lanes per wavefront

// Phase 1 of the tiled kernels: the 64 tokens of the tile, smoothed and Hadamard-transformed
// (kTransform) or just widened (values), as fp32 rows of x_s (row stride D + 4 floats).  A lane
// owns 4 consecutive channels of one token; the first two butterfly stages run inside the lane,
// the others across lanes with wavefront shuffles.
// NCH < D: only channels ch0 .. ch0 + NCH - 1 are kept (row stride NCH + 4), for a workgroup that
// searches a group of sub-spaces; values outside the window are then not even loaded.
// The two halves are separate so that a kernel can request the next tile's rows before it searches
// the present one (the workgroups of the tile kernels fill a compute unit's LDS alone, so nothing
// else would cover the trip to memory): tile_request leaves the raw fp16 rows in registers
// (2 dwords per pass and lane), tile_finish converts, transforms and writes x_s.
template <int D, int BLOCK>
struct TileRows {
    static constexpr int LPT = D / 4;                           // lanes per token
    static constexpr int TPW = 64 / LPT;                        // tokens per wavefront pass
    static constexpr int NP = kEncTokens / TPW / (BLOCK / 64);  // passes per wavefront
    uint2 raw[NP];
};

template <int D, bool kTransform, int BLOCK = kEncBlock, int NCH = D>
__device__ __forceinline__ void tile_request(const EncodeParams &p, TileRows<D, BLOCK> &rows, long long t0, int bg,
                                             int ch0 = 0)
{
    constexpr int LPT = TileRows<D, BLOCK>::LPT, TPW = TileRows<D, BLOCK>::TPW, NP = TileRows<D, BLOCK>::NP;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c0 = 4 * (lane % LPT), tw = lane / LPT;
    const bool kept = NCH == D || (c0 >= ch0 && c0 < ch0 + NCH);
#pragma unroll
    for (int pi = 0; pi < NP; ++pi) {
        const int tl = (wave + pi * (BLOCK / 64)) * TPW + tw;   // token within the tile
        long long t = t0 + tl;
        if (t >= p.T) t = p.T - 1;                                  // tail: harmless duplicate
        rows.raw[pi] = make_uint2(0u, 0u);
        if (kTransform || kept) rows.raw[pi] = *reinterpret_cast<const uint2 *>(p.x + ((size_t)bg * p.T + t) * D + c0);
    }
}

template <int D, bool kTransform, int BLOCK = kEncBlock, int NCH = D>
__device__ __forceinline__ void tile_finish(const EncodeParams &p, const TileRows<D, BLOCK> &rows, float *x_s, int g,
                                            int ch0 = 0)
{
    constexpr int LPT = TileRows<D, BLOCK>::LPT, TPW = TileRows<D, BLOCK>::TPW, NP = TileRows<D, BLOCK>::NP;
    constexpr int XS = NCH + 4;                // padded row stride of the LDS tile (floats)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane % LPT;                // which 4 channels of the token
    const int tw = lane / LPT;                 // which token of this pass
    const int c0 = 4 * sub;
    const bool kept = NCH == D || (c0 >= ch0 && c0 < ch0 + NCH);
    float rl[4] = {1.f, 1.f, 1.f, 1.f};
    if (kTransform) {
        const float4 l4 = *reinterpret_cast<const float4 *>(p.lam + (size_t)g * D + c0);
        rl[0] = l4.x; rl[1] = l4.y; rl[2] = l4.z; rl[3] = l4.w;
    }
    const float hs = 1.0f / sqrtf((float)D);
    // All passes of the wavefront advance stage by stage, so that a stage's shuffles (NP x 4
    // independent ones) are in flight together instead of one LDS round trip at a time.
    float v[NP][4];
#pragma unroll
    for (int pi = 0; pi < NP; ++pi) {
        const __half2 h01 = *reinterpret_cast<const __half2 *>(&rows.raw[pi].x);
        const __half2 h23 = *reinterpret_cast<const __half2 *>(&rows.raw[pi].y);
        v[pi][0] = __low2float(h01); v[pi][1] = __high2float(h01);
        v[pi][2] = __low2float(h23); v[pi][3] = __high2float(h23);
    }
    if (kTransform) {
#pragma unroll
        for (int pi = 0; pi < NP; ++pi) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[pi][j] = v[pi][j] / rl[j];
            // butterflies with partner distance 1 and 2 (inside the lane)
            const float a0 = v[pi][0] + v[pi][1], a1 = v[pi][0] - v[pi][1];
            const float a2 = v[pi][2] + v[pi][3], a3 = v[pi][2] - v[pi][3];
            v[pi][0] = a0 + a2; v[pi][1] = a1 + a3; v[pi][2] = a0 - a2; v[pi][3] = a1 - a3;
        }
        // partner distance 4 .. D/2 (across lanes)
#pragma unroll
        for (int x = 1; x < LPT; x <<= 1) {
            float o[NP][4];
#pragma unroll
            for (int pi = 0; pi < NP; ++pi)
#pragma unroll
                for (int j = 0; j < 4; ++j) o[pi][j] = __shfl_xor(v[pi][j], x);
            const bool up = (sub & x) != 0;
#pragma unroll
            for (int pi = 0; pi < NP; ++pi)
#pragma unroll
                for (int j = 0; j < 4; ++j) v[pi][j] = up ? (o[pi][j] - v[pi][j]) : (v[pi][j] + o[pi][j]);
        }
#pragma unroll
        for (int pi = 0; pi < NP; ++pi)
#pragma unroll
            for (int j = 0; j < 4; ++j) v[pi][j] *= hs;
    }
#pragma unroll
    for (int pi = 0; pi < NP; ++pi) {
        const int tl = (wave + pi * (BLOCK / 64)) * TPW + tw;
        float4 w; w.x = v[pi][0]; w.y = v[pi][1]; w.z = v[pi][2]; w.w = v[pi][3];
        if (kept) *reinterpret_cast<float4 *>(&x_s[tl * XS + c0 - ch0]) = w;
    }
}

// Cache fill (Eq. 2, 3, 6, 8) and K-Means assignment (Sec. 2.2), 8-bit codes: one kernel.
//
// A workgroup (8 wavefronts) takes a group of MSW sub-spaces of one (sequence, KV head) and walks
// over a run of `tiles_per_wg` 64-token tiles, so that the group's search tables are built once
// per run: per sub-space the fp16 centroids and -sigma |c|^2 / 2 (encode_screen.h), 3 to 5 KB.
// Per tile: the rows are transformed into LDS (phase 1 above; once per group of sub-spaces, so
// M / MSW times in all), every wavefront searches MSW / 8 sub-spaces for the 64 tokens (a lane
// owns a token at the end), and the group's MSW code bytes per token go out as 8- or 16-byte
// stores (tiled value codes: byte by byte, each to its place in the token's 64-token block).
// kAccumulate (K-Means): every sub-vector is also added to the sum of its centroid in LDS
// (ds_add_f32; a run meets each centroid many times) and its squared distance to the run's error;
// at the end of the run the partial sums go to memory, one atomic per non-empty centroid, and the
// error to the training state.
constexpr int kVqBlock = 512;

// Sub-spaces per workgroup: all of them for the cache fill (32 at most: d = 2 at D = 128 takes two
// workgroups per tile), 16 (d = 8: 8) for K-Means, whose sums need 256 (d + 1) floats per sub-space.
template <int d, bool kAccumulate>
constexpr int vq_group(int M)
{
    const int most = !kAccumulate ? 32 : (d == 8 ? 8 : 16);
    return M < most ? M : most;
}

template <int D, int d, bool kAccumulate>
constexpr size_t vq_smem_bytes()
{
    constexpr int MSW = vq_group<d, kAccumulate>(D / d);
    constexpr int NCH = kAccumulate ? MSW * d : D;         // channels of the tile kept in LDS
    return (size_t)MSW * ScreenTab<d>::kBytes + sizeof(float) * kEncTokens * (NCH + 4) + (size_t)kEncTokens * MSW +
           (kAccumulate ? (sizeof(float) * (d + 1) + 1) * MSW * kCentroids : 0);
}

struct KmeansState {
    double err_cur;       // quantization error of the assignment being accumulated
    double err_prev;      // .. of the iteration before
    int32_t stop_at;      // iteration after whose update the training stopped (INT32_MAX: not yet)
    int32_t pad;
};

template <int D, int d, bool kTransform, bool kAccumulate>
__global__ __launch_bounds__(kVqBlock) void vq_tile_kernel(EncodeParams p, int tiles_per_wg, int iter, KmeansState *state)
{
    constexpr int M = D / d;
    constexpr int MSW = vq_group<d, kAccumulate>(M);       // sub-spaces of the workgroup
    constexpr int NW = kVqBlock / 64;
    constexpr int SPW = (MSW + NW - 1) / NW;               // sub-spaces per wavefront: 1, 2 or 4
    static_assert(MSW % NW == 0 && M % MSW == 0, "whole groups, dealt evenly to the wavefronts");
    // K-Means keeps only its group's channels of the tile (the sums need the room)
    constexpr int NCH = kAccumulate ? MSW * d : D;
    constexpr int XS = NCH + 4;                            // row stride of the transformed tile
    constexpr int TB = ScreenTab<d>::kBytes;
    extern __shared__ __align__(16) unsigned char vq_smem[];
    unsigned char *const tab_s = vq_smem;                                          // [MSW] search tables
    float *const x_s = reinterpret_cast<float *>(tab_s + MSW * TB);                // [64][XS] transformed tile
    uint8_t *const idx_s = reinterpret_cast<uint8_t *>(x_s + kEncTokens * XS);     // [64][MSW] codes of the tile
    float *const acc_s = reinterpret_cast<float *>(idx_s + kEncTokens * MSW);      // [MSW][256][d + 1] sums, counts
    volatile uint8_t *const tag_s = reinterpret_cast<volatile uint8_t *>(acc_s + MSW * kCentroids * (d + 1));   // [MSW][256]

    if (kAccumulate && iter > 0 && iter > state->stop_at) return;     // training already stopped (every thread alike)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = blockIdx.y;
    const int bg = blockIdx.z, g = bg % p.Hkv;
    const long long tile0 = (long long)blockIdx.x * tiles_per_wg;

    // ---- the search tables of this wavefront's sub-spaces (nobody else reads them)
    ScreenConsts sc[SPW];
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        const int ms = wave + NW * i;
        sc[i] = screen_prepare<d>(p.cb + ((size_t)g * M + (size_t)grp * MSW + ms) * kCentroids * d, tab_s + ms * TB, lane);
    }
    if (kAccumulate)
        for (int e = tid; e < MSW * kCentroids * (d + 1); e += kVqBlock) acc_s[e] = 0.f;

    float err = 0.f;
    const int win0 = NCH == D ? 0 : grp * MSW * d;         // first channel of the tile that is kept
    TileRows<D, kVqBlock> rows;
    if (tile0 * kEncTokens < p.T) tile_request<D, kTransform, kVqBlock, NCH>(p, rows, tile0 * kEncTokens, bg, win0);
    for (int ti = 0; ti < tiles_per_wg; ++ti) {
        const long long t0 = (tile0 + ti) * kEncTokens;
        if (t0 >= p.T) break;
        __syncthreads();                       // previous tile's x_s and idx_s consumed (first tile: accumulators cleared)
        tile_finish<D, kTransform, kVqBlock, NCH>(p, rows, x_s, g, win0);
        __syncthreads();
        // the next tile's rows travel while this one is searched
        if (ti + 1 < tiles_per_wg && t0 + kEncTokens < p.T)
            tile_request<D, kTransform, kVqBlock, NCH>(p, rows, t0 + kEncTokens, bg, win0);
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int ms = wave + NW * i;
            const int ch0 = (NCH == D ? grp * MSW + ms : ms) * d;
            int arg;
            unsigned best;
            search_tile<d>(x_s, XS, ch0, tab_s + ms * TB, sc[i], lane, arg, best);
            idx_s[lane * MSW + ms] = (uint8_t)arg;
            if (kAccumulate && t0 + lane < p.T) {
                // The accumulators of a sub-space belong to this wavefront alone, and its LDS
                // operations execute in order, so only lanes of the same instruction can collide.
                // One lane per distinct code (the last to write its number into the code's tag)
                // adds its sub-vector with plain loads and stores; the others, about a fifth of the
                // lanes for evenly used codes, follow with atomics (ds_add_f32 costs roughly two
                // cycles per active lane: 0.35 ms of a 0.82 ms iteration when every lane used it).
                float *a = acc_s + ((size_t)ms * kCentroids + arg) * (d + 1);
                volatile uint8_t *tag = tag_s + ms * kCentroids + arg;
                *tag = (uint8_t)lane;
                if (*tag == (uint8_t)lane) {
                    float row[d + 1];
#pragma unroll
                    for (int j = 0; j <= d; ++j) row[j] = a[j];
#pragma unroll
                    for (int j = 0; j < d; ++j) a[j] = row[j] + x_s[lane * XS + ch0 + j];
                    a[d] = row[d] + 1.0f;           // (counts stay exact in fp32: far below 2^24 per run)
                } else {
#pragma unroll
                    for (int j = 0; j < d; ++j) atomicAdd(a + j, x_s[lane * XS + ch0 + j]);
                    atomicAdd(a + d, 1.0f);
                }
                err += __uint_as_float(best);
            }
        }
        __syncthreads();
        // ---- the group's MSW code bytes of each token
        if (!kAccumulate && p.tiled) {
            for (int e = tid; e < kEncTokens * MSW; e += kVqBlock) {
                const int tl = e / MSW, m = grp * MSW + (e - tl * MSW);
                const long long t = t0 + tl;
                if (t < p.T) p.idx[(size_t)bg * p.n_cap * M + v_tiled_offset(p.pos0 + t, m, M)] = idx_s[e];
            }
        } else if constexpr (MSW == 8) {
            if (tid < kEncTokens && t0 + tid < p.T)
                *reinterpret_cast<uint2 *>(p.idx + ((size_t)bg * p.n_cap + p.pos0 + t0 + tid) * M + grp * MSW) =
                    reinterpret_cast<const uint2 *>(idx_s)[tid];
        } else {
            constexpr int QPT = MSW / 16;      // 16-byte pieces per token
            const int tl = tid / QPT, q = tid % QPT;
            if (tid < kEncTokens * QPT && t0 + tl < p.T)
                *reinterpret_cast<uint4 *>(p.idx + ((size_t)bg * p.n_cap + p.pos0 + t0 + tl) * M + grp * MSW + 16 * q) =
                    reinterpret_cast<const uint4 *>(idx_s)[tid];
        }
    }
    if constexpr (kAccumulate) {
        __syncthreads();
        // the run's partial sums -> memory
        for (int e = tid; e < MSW * kCentroids; e += kVqBlock) {
            const float *a = acc_s + (size_t)e * (d + 1);
            const int n = (int)a[d];
            if (n > 0) {
                const size_t cen = ((size_t)g * M + (size_t)grp * MSW) * kCentroids + e;
#pragma unroll
                for (int j = 0; j < d; ++j) unsafeAtomicAdd(p.km_sums + cen * d + j, a[j]);
                atomicAdd(p.km_counts + cen, n);
            }
        }
        double e64 = (double)err;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) e64 += __shfl_xor(e64, o);
        if (lane == 0 && state) unsafeAtomicAdd(&state->err_cur, e64);
    }
}


// Start of a training iteration: sums and counts cleared, the error accumulator reset (and, before
// the first iteration, the whole state).
__global__ void kmeans_begin_kernel(float *sums, int32_t *counts, size_t n_sums, size_t n_counts, int iter,
                                    KmeansState *state)
{
    if (iter > 0 && iter > state->stop_at) return;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_sums) sums[i] = 0.f;
    if (i < n_counts) counts[i] = 0;
    if (i == 0) {
        state->err_cur = 0.0;
        if (iter == 0) {
            state->err_prev = 0.0;
            state->stop_at = 0x7fffffff;
        }
    }
}

// End of a training iteration: the centroid update in place (an empty cluster keeps its centroid),
// the cluster sizes, the iteration's error, and the stopping rule: the training stops after this
// update when the error improved by no more than tol times the error of the iteration before.
__global__ void kmeans_end_kernel(const float *sums, const int32_t *counts, __half *cb, int32_t *counts_out,
                                  size_t n_centroids, int d, int iter, float tol, KmeansState *state,
                                  int32_t *iters_run, double *errors)
{
    if (iter > 0 && iter > state->stop_at) return;
    const size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c == 0) {
        const double e = state->err_cur, prev = state->err_prev;
        if (errors) errors[iter] = e;
        if (iters_run) *iters_run = iter + 1;
        if (iter >= 1 && prev - e <= (double)tol * prev) state->stop_at = iter;
        state->err_prev = e;
    }
    if (c >= n_centroids) return;
    const int n = counts[c];
    if (counts_out) counts_out[c] = n;
    if (n > 0)
        for (int j = 0; j < d; ++j) cb[c * d + j] = __float2half(sums[c * d + j] / (float)n);
}

// Decode-time append (Eq. 9) and other short inputs: one workgroup per (token, batch, KV head).
// The token is transformed in LDS with the same butterfly order as the tiled kernel (so both
// produce bit-identical k~).  Then, 32 sub-spaces at a time: thread c writes the distance of
// every sub-vector to centroid c into LDS; eight threads per sub-space each scan 32 of its 256
// distances in increasing centroid order (strict "<": lowest index wins) and combine through
// 64-bit (distance bits, index) keys -- a non-negative fp32 orders like its bit pattern.
constexpr int kTokRowStride = kCentroids + 1;    // padded LDS row: scanning threads hit distinct banks
constexpr int kTokMaxPass = 32;                  // sub-spaces per pass
constexpr int kTokDistFloats = kTokMaxPass * kTokRowStride;

template <int D, int d, bool kTransform>
__device__ __forceinline__ void encode_token(const EncodeParams &p, float *x_s, float *dist_s)
{
    constexpr int M = D / d;
    constexpr int MC = M < kTokMaxPass ? M : kTokMaxPass;   // sub-spaces per pass
    constexpr int RS = kTokRowStride;

    const int tid = threadIdx.x;
    const long long t = blockIdx.x;
    const int bg = blockIdx.z;
    const int g = bg % p.Hkv;
    long long pos = p.pos0 + t;
    if (p.seq_lens) {                          // per-sequence position: the last token of the sequence
        const long long v = p.seq_lens[bg / p.Hkv];
        const long long len = v < 0 ? 0 : (v > p.len_max ? p.len_max : v);
        if (len == 0) return;                  // uniform over the workgroup
        pos = len - 1;
    }

    if (tid < D) {
        float v = __half2float(p.x[((size_t)bg * p.T + t) * D + tid]);
        if (kTransform) v = v / p.lam[(size_t)g * D + tid];
        x_s[tid] = v;
    }
    __syncthreads();
    if (kTransform) {
        for (int st = 1; st < D; st <<= 1) {
            float mine = 0.f, other = 0.f;
            if (tid < D) {
                mine = x_s[tid];
                other = x_s[tid ^ st];
            }
            __syncthreads();
            if (tid < D) x_s[tid] = (tid & st) ? (other - mine) : (mine + other);
            __syncthreads();
        }
        const float hs = 1.0f / sqrtf((float)D);
        if (tid < D) x_s[tid] *= hs;
        __syncthreads();
    }

    const __half *cb = p.cb + (size_t)g * M * kCentroids * d + (size_t)tid * d;
    for (int m0 = 0; m0 < M; m0 += MC) {
#pragma unroll 8
        for (int mm = 0; mm < MC; ++mm) {
            const int m = m0 + mm;
            float dist = 0.f;
#pragma unroll
            for (int j = 0; j < d; ++j) {
                const float tdiff = x_s[m * d + j] - __half2float(cb[(size_t)m * kCentroids * d + j]);
                dist = fmaf(tdiff, tdiff, dist);
            }
            dist_s[mm * RS + tid] = dist;
        }
        __syncthreads();
        {
            const int mm = tid >> 3, part = tid & 7;
            float best = INFINITY;
            unsigned arg = 0;
            if (mm < MC) {
#pragma unroll 8
                for (int i = 0; i < kCentroids / 8; ++i) {
                    const unsigned c = part + 8 * i;
                    const float v = dist_s[mm * RS + c];
                    if (v < best) {
                        best = v;
                        arg = c;
                    }
                }
            }
            unsigned long long key = ((unsigned long long)__float_as_uint(best) << 32) | arg;
#pragma unroll
            for (int o = 4; o > 0; o >>= 1) {
                const unsigned long long other = __shfl_xor(key, o);
                key = other < key ? other : key;
            }
            if (part == 0 && mm < MC)
                p.idx[(size_t)bg * p.n_cap * M + (p.tiled ? v_tiled_offset(pos, m0 + mm, M) : (size_t)pos * M + m0 + mm)] =
                    (uint8_t)(key & 255u);
        }
        __syncthreads();
    }
}

template <int D, int d, bool kTransform>
__global__ __launch_bounds__(kCentroids) void encode_token_kernel(EncodeParams p)
{
    __shared__ float x_s[D];
    __shared__ float dist_s[kTokDistFloats];
    encode_token<D, d, kTransform>(p, x_s, dist_s);
}

// Eq. 9 in one launch: blockIdx.y = 0 appends the key codes (transform + VQ), 1 the value codes.
template <int D, int dk, int dv>
__global__ __launch_bounds__(kCentroids) void append_kv_kernel(EncodeParams pk, EncodeParams pv)
{
    __shared__ float x_s[D];
    __shared__ float dist_s[kTokDistFloats];
    if (blockIdx.y == 0)
        encode_token<D, dk, true>(pk, x_s, dist_s);
    else
        encode_token<D, dv, false>(pv, x_s, dist_s);
}

constexpr long long kTokenKernelMaxT = 16;     // below this many tokens per (b, g) the per-token kernel wins

// ---------------------------------------------------------------------------------------------
// Codes wider than 8 bits (10 or 12; d8b12, d4b12, d4b10 of Sec. 4.1): one table of C = 2^b
// centroids per KV head, shared by its sub-spaces (the codebook of Sec. 2.2 and Alg. 1), and a
// token's M codes packed end to end, b bits each, in M b / 8 bytes.  D = 128, or D = 64 where a row
// is a whole number of 32-bit words (not d = 8 with 10-bit codes).
//
// What is written is the centroid at the smallest squared distance, summed directly in channel order
// in fp32, lowest index among equals: the rule of the 8-bit kernels.

template <int d>
__device__ __forceinline__ void load_centroid(const __half *tab, unsigned c, float (&cen)[d])
{
    if constexpr (d == 8) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(tab + (size_t)c * 8);
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            cen[2 * j] = __low2float(h[j]);
            cen[2 * j + 1] = __high2float(h[j]);
        }
    } else {
        const uint2 raw = *reinterpret_cast<const uint2 *>(tab + (size_t)c * 4);
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
        cen[0] = __low2float(h[0]); cen[1] = __high2float(h[0]);
        cen[2] = __low2float(h[1]); cen[3] = __high2float(h[1]);
    }
}

template <int d>
__device__ __forceinline__ unsigned dist_bits_of(const float (&x)[d], const float (&cen)[d])
{
    float dist = 0.f;
#pragma unroll
    for (int j = 0; j < d; ++j) {
        const float t = x[j] - cen[j];
        dist = fmaf(t, t, dist);
    }
    return __float_as_uint(dist);      // a non-negative fp32 orders like its bit pattern
}

// Packs the M codes of each of `rows` tokens (LDS, uint16 [rows][M]) into the token's row of
// M BITS / 8 bytes and writes whole 32-bit words; word w of a row holds bits 32 w .. 32 w + 31.
template <int M, int BITS>
__device__ __forceinline__ void store_packed_rows(const EncodeParams &p, const unsigned short *idx_s, long long t0,
                                                  int rows, int bg, int nthreads)
{
    constexpr int WPT = M * BITS / 32;         // words per token row
    for (int e = threadIdx.x; e < rows * WPT; e += nthreads) {
        const int tl = e / WPT, w = e - tl * WPT;
        const long long t = t0 + tl;
        if (t >= p.T) continue;
        unsigned word = 0;
        const int m_lo = 32 * w / BITS, m_hi = (32 * w + 31) / BITS;
        for (int m = m_lo; m <= m_hi && m < M; ++m) {
            const int sh = m * BITS - 32 * w;  // position of the code's bit 0 inside this word
            const unsigned c = idx_s[tl * M + m];
            word |= sh >= 0 ? c << sh : c >> (-sh);
        }
        reinterpret_cast<uint32_t *>(p.idx + ((size_t)bg * p.n_cap + p.pos0 + t) * (M * BITS / 8))[w] = word;
    }
}

// Tiled kernel: as vq_tile_kernel, with one table for all sub-spaces.  A workgroup (8 wavefronts)
// builds the search tables of its KV head's codebook once (the fp16 table as it is, 8 - 64 KB, and
// -sigma |c|^2 / 2, 4 - 16 KB) and walks over a run of 64-token tiles; per tile every wavefront
// searches M / 8 sub-spaces, 256 centroids at a time (screen_search_shared: matrix-core screen,
// exact fp32 distances of what it keeps, the plain search where it gives up), and the tile's codes
// are packed into rows.  K-Means (km_sums set): every sub-vector also joins the sum of its centroid
// in the head's one table (fp32 hardware atomics, order of the additions not fixed) and its squared
// distance the iteration's error.
template <int D, int d, int BITS>
constexpr size_t vq_wide_smem_bytes()
{
    return (size_t)ScreenTab<d, (1 << BITS)>::kBytes + sizeof(float) * kEncTokens * (D + 4) +
           sizeof(unsigned short) * kEncTokens * (D / d);
}
// K-Means with a shared table: a run's partial sums and counts [C][d + 1] stay in LDS where that
// fits beside the search tables (1024 centroids: 20 or 36 KB), and go to memory once per run with
// one atomic per non-empty centroid and channel; with 4096 centroids every sub-vector adds to
// memory directly.
template <int D, int d, int BITS>
constexpr bool vq_wide_lds_sums()
{
    return vq_wide_smem_bytes<D, d, BITS>() + sizeof(float) * (size_t)(1 << BITS) * (d + 1) <= 96 * 1024;
}

template <int D, int d, int BITS, bool kTransform>
__global__ __launch_bounds__(kVqBlock) void vq_tile_wide_kernel(EncodeParams p, int tiles_per_wg)
{
    constexpr int M = D / d, C = 1 << BITS;
    static_assert(M * BITS % 32 == 0, "rows of whole 32-bit words");
    constexpr int NW = kVqBlock / 64;
    constexpr int SPW = M / NW;                            // sub-spaces per wavefront: 1, 2 or 4
    static_assert(M % NW == 0, "sub-spaces dealt evenly to the wavefronts");
    constexpr int XS = D + 4;
    using Tab = ScreenTab<d, C>;
    extern __shared__ __align__(16) unsigned char vqw_smem[];
    unsigned char *const tab_s = vqw_smem;                                                  // the head's search tables
    float *const x_s = reinterpret_cast<float *>(tab_s + Tab::kBytes);                      // [64][XS] transformed tile
    unsigned short *const idx_s = reinterpret_cast<unsigned short *>(x_s + kEncTokens * XS);   // [64][M] codes of the tile
    constexpr bool kLdsSums = vq_wide_lds_sums<D, d, BITS>();
    float *const acc_s = reinterpret_cast<float *>(vqw_smem + vq_wide_smem_bytes<D, d, BITS>());   // [C][d + 1] (K-Means)

    KmeansState *const state = static_cast<KmeansState *>(p.km_state);
    if (p.km_sums && p.km_iter > 0 && p.km_iter > state->stop_at) return;   // training already stopped
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int bg = blockIdx.z, g = bg % p.Hkv;
    const long long tile0 = (long long)blockIdx.x * tiles_per_wg;

    if (kLdsSums && p.km_sums)
        for (int e = tid; e < C * (d + 1); e += kVqBlock) acc_s[e] = 0.f;     // (the barriers of the table set-up follow)
    const ScreenConsts sc = screen_prepare_shared<d, C, kVqBlock>(p.cb + (size_t)g * C * d, tab_s, x_s);

    float err = 0.f;
    TileRows<D, kVqBlock> rows;
    if (tile0 * kEncTokens < p.T) tile_request<D, kTransform, kVqBlock>(p, rows, tile0 * kEncTokens, bg);
    for (int ti = 0; ti < tiles_per_wg; ++ti) {
        const long long t0 = (tile0 + ti) * kEncTokens;
        if (t0 >= p.T) break;
        if (ti > 0) __syncthreads();           // previous tile's x_s and idx_s consumed
        tile_finish<D, kTransform, kVqBlock>(p, rows, x_s, g);
        __syncthreads();
        // the next tile's rows travel while this one is searched
        if (ti + 1 < tiles_per_wg && t0 + kEncTokens < p.T)
            tile_request<D, kTransform, kVqBlock>(p, rows, t0 + kEncTokens, bg);
#pragma unroll 1
        for (int i = 0; i < SPW; ++i) {        // (not unrolled: the searches are long and share nothing but the tables)
            const int m = wave + NW * i;
            int arg;
            unsigned best;
            search_tile<d, C>(x_s, XS, m * d, tab_s, sc, lane, arg, best);
            idx_s[lane * M + m] = (unsigned short)arg;
            if (t0 + lane < p.T) err += __uint_as_float(best);
        }
        __syncthreads();
        store_packed_rows<M, BITS>(p, idx_s, t0, kEncTokens, bg, kVqBlock);
        if (p.km_sums) {
            for (int e = tid; e < kEncTokens * M; e += kVqBlock) {
                const int tl = e / M, m = e - tl * M;
                if (t0 + tl < p.T) {
                    if constexpr (kLdsSums) {
                        float *a = acc_s + (size_t)idx_s[tl * M + m] * (d + 1);
#pragma unroll
                        for (int j = 0; j < d; ++j) atomicAdd(a + j, x_s[tl * XS + m * d + j]);
                        atomicAdd(a + d, 1.0f);        // (counts stay exact in fp32: far below 2^24 per run)
                    } else {
                        const size_t cen = (size_t)g * C + idx_s[tl * M + m];
#pragma unroll
                        for (int j = 0; j < d; ++j) unsafeAtomicAdd(p.km_sums + cen * d + j, x_s[tl * XS + m * d + j]);
                        atomicAdd(p.km_counts + cen, 1);
                    }
                }
            }
        }
    }
    if (p.km_sums) {
        if constexpr (kLdsSums) {
            __syncthreads();
            // the run's partial sums -> memory
            for (int e = tid; e < C; e += kVqBlock) {
                const float *a = acc_s + (size_t)e * (d + 1);
                const int n = (int)a[d];
                if (n > 0) {
                    const size_t cen = (size_t)g * C + e;
#pragma unroll
                    for (int j = 0; j < d; ++j) unsafeAtomicAdd(p.km_sums + cen * d + j, a[j]);
                    atomicAdd(p.km_counts + cen, n);
                }
            }
        }
        double e64 = (double)err;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) e64 += __shfl_xor(e64, o);
        if (lane == 0) unsafeAtomicAdd(&state->err_cur, e64);
    }
}

// Decode-time append and other short inputs with wide codes: one workgroup per (token, group of
// 4 sub-spaces, batch x KV head).  The token is transformed as in encode_token (same butterfly
// order: bit-identical k~).  Thread c tries centroids c, c + 256, ... (increasing, strict "<":
// its lowest index wins) against the 4 sub-vectors; the threads combine through 64-bit
// (distance bits, index) keys, and the group's 4 b bits (a whole number of bytes) go out as bytes.
constexpr int kTokWideSub = 4;

template <int D, int d, int BITS, bool kTransform>
__device__ __forceinline__ void encode_token_wide(const EncodeParams &p, int group, float *x_s,
                                                  unsigned long long (*key_s)[kTokWideSub], unsigned *code_s)
{
    constexpr int M = D / d, C = 1 << BITS, MS = kTokWideSub;
    const int tid = threadIdx.x;
    const long long t = blockIdx.x;
    const int m0 = group * MS;
    const int bg = blockIdx.z;
    const int g = bg % p.Hkv;
    long long pos = p.pos0 + t;
    if (p.seq_lens) {                          // per-sequence position: the last token of the sequence
        const long long v = p.seq_lens[bg / p.Hkv];
        const long long len = v < 0 ? 0 : (v > p.len_max ? p.len_max : v);
        if (len == 0) return;                  // uniform over the workgroup
        pos = len - 1;
    }

    if (tid < D) {
        float v = __half2float(p.x[((size_t)bg * p.T + t) * D + tid]);
        if (kTransform) v = v / p.lam[(size_t)g * D + tid];
        x_s[tid] = v;
    }
    __syncthreads();
    if (kTransform) {
        for (int st = 1; st < D; st <<= 1) {
            float mine = 0.f, other = 0.f;
            if (tid < D) {
                mine = x_s[tid];
                other = x_s[tid ^ st];
            }
            __syncthreads();
            if (tid < D) x_s[tid] = (tid & st) ? (other - mine) : (mine + other);
            __syncthreads();
        }
        const float hs = 1.0f / sqrtf((float)D);
        if (tid < D) x_s[tid] *= hs;
        __syncthreads();
    }

    float x[MS][d];
#pragma unroll
    for (int i = 0; i < MS; ++i)
#pragma unroll
        for (int j = 0; j < d; ++j) x[i][j] = x_s[(m0 + i) * d + j];
    unsigned best[MS], arg[MS];
#pragma unroll
    for (int i = 0; i < MS; ++i) {
        best[i] = 0x7f800000u;
        arg[i] = 0;
    }
    const __half *tab = p.cb + (size_t)g * C * d;
#pragma unroll 4
    for (int c = tid; c < C; c += kCentroids) {
        float cen[d];
        load_centroid<d>(tab, c, cen);
#pragma unroll
        for (int i = 0; i < MS; ++i) {
            const unsigned v = dist_bits_of<d>(x[i], cen);
            if (v < best[i]) {
                best[i] = v;
                arg[i] = c;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < MS; ++i) {
        unsigned long long key = ((unsigned long long)best[i] << 32) | arg[i];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long other = __shfl_xor(key, o);
            key = other < key ? other : key;
        }
        if ((tid & 63) == 0) key_s[tid >> 6][i] = key;
    }
    __syncthreads();
    if (tid < MS) {
        unsigned long long key = key_s[0][tid];
#pragma unroll
        for (int w = 1; w < kCentroids / 64; ++w) key = key_s[w][tid] < key ? key_s[w][tid] : key;
        code_s[tid] = (unsigned)(key & 0xffffffffu);
    }
    __syncthreads();
    // the group's MS codes = MS BITS / 8 whole bytes at byte m0 BITS / 8 of the row
    constexpr int GB = MS * BITS / 8;
    if (tid < GB) {
        unsigned long long bits = 0;
#pragma unroll
        for (int i = 0; i < MS; ++i) bits |= (unsigned long long)code_s[i] << (i * BITS);
        p.idx[((size_t)bg * p.n_cap + pos) * (M * BITS / 8) + (size_t)m0 * BITS / 8 + tid] = (uint8_t)(bits >> (8 * tid));
    }
}

template <int D, int d, int BITS, bool kTransform>
__global__ __launch_bounds__(kCentroids) void encode_token_wide_kernel(EncodeParams p)
{
    __shared__ float x_s[D];
    __shared__ unsigned long long key_s[kCentroids / 64][kTokWideSub];
    __shared__ unsigned code_s[kTokWideSub];
    encode_token_wide<D, d, BITS, kTransform>(p, blockIdx.y, x_s, key_s, code_s);
}

// Eq. 9 with wide codes on both sides in one launch: the first M_k / 4 workgroups along y take the
// key's sub-space groups, the others the value's.
template <int D, int dk, int BK, int dv, int BV>
__global__ __launch_bounds__(kCentroids) void append_wide_kernel(EncodeParams pk, EncodeParams pv)
{
    __shared__ float x_s[D];
    __shared__ unsigned long long key_s[kCentroids / 64][kTokWideSub];
    __shared__ unsigned code_s[kTokWideSub];
    constexpr int GK = D / dk / kTokWideSub;
    if (blockIdx.y < GK)
        encode_token_wide<D, dk, BK, true>(pk, blockIdx.y, x_s, key_s, code_s);
    else
        encode_token_wide<D, dv, BV, false>(pv, blockIdx.y - GK, x_s, key_s, code_s);
}

template <int D, int dk, int BK, int dv, int BV>
int launch_append_wide_typed(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream)
{
    dim3 grid((unsigned)pk.T, (D / dk + D / dv) / kTokWideSub, pk.B * pk.Hkv);
    hipLaunchKernelGGL((append_wide_kernel<D, dk, BK, dv, BV>), grid, dim3(kCentroids), 0, stream, pk, pv);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

template <int D, int dk, int BK>
int launch_append_wide_v(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream)
{
    switch (pv.d * 100 + pv.bits) {
    case 810:
        if constexpr (D == 128) return launch_append_wide_typed<D, dk, BK, 8, 10>(pk, pv, stream);
        else return -2;
    case 812: return launch_append_wide_typed<D, dk, BK, 8, 12>(pk, pv, stream);
    case 410: return launch_append_wide_typed<D, dk, BK, 4, 10>(pk, pv, stream);
    case 412: return launch_append_wide_typed<D, dk, BK, 4, 12>(pk, pv, stream);
    default: return -2;
    }
}

template <int D>
int launch_append_wide_d(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream)
{
    switch (pk.d * 100 + pk.bits) {
    case 810:
        if constexpr (D == 128) return launch_append_wide_v<D, 8, 10>(pk, pv, stream);
        else return -2;
    case 812: return launch_append_wide_v<D, 8, 12>(pk, pv, stream);
    case 410: return launch_append_wide_v<D, 4, 10>(pk, pv, stream);
    case 412: return launch_append_wide_v<D, 4, 12>(pk, pv, stream);
    default: return -2;
    }
}

// both sides wide: one launch
int launch_append_wide(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream)
{
    if (pk.D == 128) return launch_append_wide_d<128>(pk, pv, stream);
    if (pk.D == 64) return launch_append_wide_d<64>(pk, pv, stream);
    return -2;
}

template <int D, int d, int BITS>
int launch_wide_typed(const EncodeParams &p, hipStream_t stream)
{
    constexpr int M = D / d;
    if (p.T <= kTokenKernelMaxT && !p.km_sums) {
        dim3 tgrid((unsigned)p.T, M / kTokWideSub, p.B * p.Hkv);
        if (p.lam)
            hipLaunchKernelGGL((encode_token_wide_kernel<D, d, BITS, true>), tgrid, dim3(kCentroids), 0, stream, p);
        else
            hipLaunchKernelGGL((encode_token_wide_kernel<D, d, BITS, false>), tgrid, dim3(kCentroids), 0, stream, p);
        return hipGetLastError() == hipSuccess ? 0 : -4;
    }
    constexpr size_t smem_fill = vq_wide_smem_bytes<D, d, BITS>();
    constexpr size_t smem = smem_fill + (vq_wide_lds_sums<D, d, BITS>() ? sizeof(float) * (size_t)(1 << BITS) * (d + 1) : 0);
    static_assert(smem <= 160 * 1024, "LDS of a compute unit");
    static const bool configured =
        hipFuncSetAttribute(reinterpret_cast<const void *>(vq_tile_wide_kernel<D, d, BITS, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(vq_tile_wide_kernel<D, d, BITS, false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    if (!configured) return -4;
    // runs: the tables are built a few times per compute unit only, the grid still fills the chip
    const long long tiles = (p.T + kEncTokens - 1) / kEncTokens;
    long long per = tiles * p.B * p.Hkv / (4LL * num_cus());
    if (per < 1) per = 1;
    if (per > 256) per = 256;
    dim3 grid((unsigned)((tiles + per - 1) / per), 1, p.B * p.Hkv);
    const size_t smem_now = p.km_sums ? smem : smem_fill;     // (the partial sums only where they are used)
    if (p.lam)
        hipLaunchKernelGGL((vq_tile_wide_kernel<D, d, BITS, true>), grid, dim3(kVqBlock), smem_now, stream, p, (int)per);
    else
        hipLaunchKernelGGL((vq_tile_wide_kernel<D, d, BITS, false>), grid, dim3(kVqBlock), smem_now, stream, p, (int)per);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

int launch_encode_wide(const EncodeParams &p, hipStream_t stream)
{
    const int key = p.D * 1000 + p.d * 100 + p.bits;
    switch (key) {
    case 128810: return launch_wide_typed<128, 8, 10>(p, stream);
    case 128812: return launch_wide_typed<128, 8, 12>(p, stream);
    case 128410: return launch_wide_typed<128, 4, 10>(p, stream);
    case 128412: return launch_wide_typed<128, 4, 12>(p, stream);
    case 64812: return launch_wide_typed<64, 8, 12>(p, stream);     // (d = 8 with 10-bit codes: 10-byte rows, not built)
    case 64410: return launch_wide_typed<64, 4, 10>(p, stream);
    case 64412: return launch_wide_typed<64, 4, 12>(p, stream);
    default: return -2;
    }
}

// vq_tile_kernel over the T tokens of p: runs long enough that the tables are built a few times per
// compute unit only (and, for K-Means, that a workgroup meets each centroid many times), short
// enough that the grid still fills the chip several times over.
template <int D, int d, bool kAccumulate>
int launch_vq_tiles(const EncodeParams &p, int iter, void *state, hipStream_t stream)
{
    constexpr int M = D / d, MSW = vq_group<d, kAccumulate>(M);
    constexpr size_t smem = vq_smem_bytes<D, d, kAccumulate>();
    static_assert(smem <= 160 * 1024, "LDS of a compute unit");
    static const bool configured =
        hipFuncSetAttribute(reinterpret_cast<const void *>(vq_tile_kernel<D, d, true, kAccumulate>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess &&
        hipFuncSetAttribute(reinterpret_cast<const void *>(vq_tile_kernel<D, d, false, kAccumulate>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) == hipSuccess;
    if (!configured) return -4;
    const long long tiles = (p.T + kEncTokens - 1) / kEncTokens;
    const long long groups = (long long)(M / MSW) * p.B * p.Hkv;
    // (K-Means: one workgroup per compute unit where the input allows, so that the partial sums are
    // flushed as rarely as possible: 21 M global atomics per iteration at 65536 x 8 tokens with four)
    long long per = tiles * groups / ((kAccumulate ? 1LL : 4LL) * num_cus());
    if (per < 1) per = 1;
    if (per > 256) per = 256;
    dim3 grid((unsigned)((tiles + per - 1) / per), M / MSW, p.B * p.Hkv);
    if (p.lam)
        hipLaunchKernelGGL((vq_tile_kernel<D, d, true, kAccumulate>), grid, dim3(kVqBlock), smem, stream, p, (int)per, iter,
                           static_cast<KmeansState *>(state));
    else
        hipLaunchKernelGGL((vq_tile_kernel<D, d, false, kAccumulate>), grid, dim3(kVqBlock), smem, stream, p, (int)per, iter,
                           static_cast<KmeansState *>(state));
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

template <int D, int d>
int launch_typed(const EncodeParams &p, hipStream_t stream)
{
    if (p.T <= kTokenKernelMaxT && !p.km_sums) {
        dim3 tgrid((unsigned)p.T, 1, p.B * p.Hkv);
        if (p.lam)
            hipLaunchKernelGGL((encode_token_kernel<D, d, true>), tgrid, dim3(kCentroids), 0, stream, p);
        else
            hipLaunchKernelGGL((encode_token_kernel<D, d, false>), tgrid, dim3(kCentroids), 0, stream, p);
        return hipGetLastError() == hipSuccess ? 0 : -4;
    }
    return launch_vq_tiles<D, d, false>(p, 0, nullptr, stream);
}

template <int D, int dk>
int launch_append_dv(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream)
{
    dim3 grid((unsigned)pk.T, 2, pk.B * pk.Hkv);
    if (pv.d == 2)
        hipLaunchKernelGGL((append_kv_kernel<D, dk, 2>), grid, dim3(kCentroids), 0, stream, pk, pv);
    else if (pv.d == 4)
        hipLaunchKernelGGL((append_kv_kernel<D, dk, 4>), grid, dim3(kCentroids), 0, stream, pk, pv);
    else if (pv.d == 8)
        hipLaunchKernelGGL((append_kv_kernel<D, dk, 8>), grid, dim3(kCentroids), 0, stream, pk, pv);
    else
        return -2;
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

template <int D>
int launch_append_dk(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream)
{
    if (pk.d == 2) return launch_append_dv<D, 2>(pk, pv, stream);
    if (pk.d == 4) return launch_append_dv<D, 4>(pk, pv, stream);
    if (pk.d == 8) return launch_append_dv<D, 8>(pk, pv, stream);
    return -2;
}

} // namespace

// Tiled value codes -> rows (the N x M code matrix of each (sequence, KV head)).
namespace {
__global__ void export_value_codes_kernel(const uint8_t *tiled, uint8_t *rows, int M, long long N, long long n_cap)
{
    const size_t bg = blockIdx.y;
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;      // byte of the rows form
    if (e >= N * M) return;
    const long long n = e / M;
    const int m = (int)(e - n * M);
    rows[bg * (size_t)n_cap * M + e] = tiled[bg * (size_t)n_cap * M + v_tiled_offset(n, m, M)];
}
} // namespace

int launch_export_value_codes(const uint8_t *tiled, uint8_t *rows, int BH, int M, long long N, long long n_cap,
                              hipStream_t stream)
{
    const long long blocks = (N * M + 255) / 256;
    if (BH < 1 || BH > 65535 || blocks > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(export_value_codes_kernel, dim3((unsigned)blocks, BH), dim3(256), 0, stream, tiled, rows, M, N, n_cap);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

int append_max_tokens() { return (int)kTokenKernelMaxT; }

size_t kmeans_state_bytes() { return sizeof(KmeansState); }

// Assignment + accumulation of one training iteration for 8-bit codes (rows layout of the codes).
int launch_kmeans_assign(const EncodeParams &p, int iter, void *state, hipStream_t stream)
{
    if (p.bits != 8 || !p.km_sums || p.tiled) return -2;
    if ((p.T + kEncTokens - 1) / kEncTokens > 0x7fffffffLL || p.B * p.Hkv > 65535) return -2;
    const int key = p.D * 10 + p.d;
    switch (key) {
    case 1282: return launch_vq_tiles<128, 2, true>(p, iter, state, stream);
    case 1284: return launch_vq_tiles<128, 4, true>(p, iter, state, stream);
    case 1288: return launch_vq_tiles<128, 8, true>(p, iter, state, stream);
    case 642: return launch_vq_tiles<64, 2, true>(p, iter, state, stream);
    case 644: return launch_vq_tiles<64, 4, true>(p, iter, state, stream);
    case 648: return launch_vq_tiles<64, 8, true>(p, iter, state, stream);
    default: return -2;
    }
}

int launch_kmeans_begin(float *sums, int32_t *counts, size_t n_sums, size_t n_counts, int iter, void *state,
                        hipStream_t stream)
{
    const size_t n = n_sums > n_counts ? n_sums : n_counts;
    hipLaunchKernelGGL(kmeans_begin_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, sums, counts,
                       n_sums, n_counts, iter, static_cast<KmeansState *>(state));
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

int launch_kmeans_end(const float *sums, const int32_t *counts, __half *cb, int32_t *counts_out, size_t n_centroids,
                      int d, int iter, float tol, void *state, int32_t *iters_run, double *errors, hipStream_t stream)
{
    hipLaunchKernelGGL(kmeans_end_kernel, dim3((unsigned)((n_centroids + 255) / 256)), dim3(256), 0, stream, sums,
                       counts, cb, counts_out, n_centroids, d, iter, tol, static_cast<KmeansState *>(state), iters_run,
                       errors);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

int launch_append(const EncodeParams &pk, const EncodeParams &pv, hipStream_t stream)
{
    if (pk.T > kTokenKernelMaxT) return -2;
    if (pk.bits != 8 && pv.bits != 8) return launch_append_wide(pk, pv, stream);
    if (pk.bits != 8 || pv.bits != 8) {
        // one wide side, one 8-bit side: each has its own per-token kernel (launch_encode picks
        // it for T <= kTokenKernelMaxT), so keys and values go out as two launches
        const int rc = launch_encode(pk, stream);
        return rc != 0 ? rc : launch_encode(pv, stream);
    }
    if (pk.D == 128) return launch_append_dk<128>(pk, pv, stream);
    if (pk.D == 64) return launch_append_dk<64>(pk, pv, stream);
    return -2;
}

int launch_encode(const EncodeParams &p, hipStream_t stream)
{
    if (p.bits != 8) return launch_encode_wide(p, stream);
    if (p.D == 128) {
        if (p.d == 2) return launch_typed<128, 2>(p, stream);
        if (p.d == 4) return launch_typed<128, 4>(p, stream);
        if (p.d == 8) return launch_typed<128, 8>(p, stream);
    } else if (p.D == 64) {
        if (p.d == 2) return launch_typed<64, 2>(p, stream);
        if (p.d == 4) return launch_typed<64, 4>(p, stream);
        if (p.d == 8) return launch_typed<64, 8>(p, stream);
    }
    return -2;
}

} // namespace vecinfer
