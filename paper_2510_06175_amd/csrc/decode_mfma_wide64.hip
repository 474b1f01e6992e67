// Matrix-core decode attention with 10- or 12-bit codes on the key side, the value side or both
// (d8b12, d4b12, K-d4b10 / V-d8b12, K-d8b12 / V-d8b8, ... of Sec. 4.1) at head dim 64:
// instantiations and dispatch (kernel: decode_mfma_kernel.h).  d = 4 or 8 on both sides (not d = 8 with 10-bit codes:
// its 10-byte rows are not whole words; d_v = 8 runs as two halves of 4 channels per code).
#include "decode_mfma_kernel.h"

namespace vecinfer {

namespace {

constexpr int kHeadDim = 64;
// a packed row must be a whole number of 32-bit words
constexpr bool row_ok(int d, int bits) { return bits == 8 || (kHeadDim / d * bits) % 32 == 0; }

template <int DK, int BK, int DV>
int pick_bv(const DecodeParams &p, hipStream_t stream)
{
    switch (p.bv) {
    case 8:
        if constexpr (BK != 8) return launch_typed<kHeadDim, DK, DV, 8, true, BK, 8>(p, stream);
        else return -2;                                    // both sides 8 bits: not this file's
    case 10:
        if constexpr (row_ok(DV, 10)) return launch_typed<kHeadDim, DK, DV, 8, true, BK, 10>(p, stream);
        else return -2;
    case 12: return launch_typed<kHeadDim, DK, DV, 8, true, BK, 12>(p, stream);
    default: return -2;
    }
}

template <int DK, int BK>
int pick_dv(const DecodeParams &p, hipStream_t stream)
{
    if (p.dv == 4) return pick_bv<DK, BK, 4>(p, stream);
    if (p.dv == 8) return pick_bv<DK, BK, 8>(p, stream);
    return -2;
}

template <int DK>
int pick_bk(const DecodeParams &p, hipStream_t stream)
{
    switch (p.bk) {
    case 8: return pick_dv<DK, 8>(p, stream);
    case 10:
        if constexpr (row_ok(DK, 10)) return pick_dv<DK, 10>(p, stream);
        else return -2;
    case 12: return pick_dv<DK, 12>(p, stream);
    default: return -2;
    }
}

} // namespace

int launch_decode_mfma_wide64(const DecodeParams &p, hipStream_t stream)
{
    if (p.D != kHeadDim) return -2;
    if (p.dk == 4) return pick_bk<4>(p, stream);
    if (p.dk == 8) return pick_bk<8>(p, stream);
    return -2;
}

} // namespace vecinfer
