// Matrix-core decode attention, 8-bit codes: instantiations and dispatch (kernel: decode_mfma_kernel.h).
#include "decode_mfma_kernel.h"

namespace vecinfer {

bool decode_mfma_supports(const DecodeParams &p)
{
    const bool dk_ok = p.dk == 8 || p.dk == 4 || p.dk == 2;
    const bool dv_ok = p.dv == 8 || p.dv == 4 || p.dv == 2;
    // 10- and 12-bit codes: d = 4 or 8 on that side (rows of whole 32-bit words: not d = 8 with 10 bits
    // at D = 64), d = 4 or 8 on the other side too
    auto wide = [](int b) { return b == 10 || b == 12; };
    auto row_ok = [&](int d, int b) { return b == 8 || (wide(b) && (p.D / d * b) % 32 == 0); };
    bool bits_ok = p.bk == 8 && p.bv == 8;
    if (wide(p.bk) || wide(p.bv)) bits_ok = row_ok(p.dk, p.bk) && row_ok(p.dv, p.bv) && p.dk >= 4 && p.dv >= 4;
    // code rows are addressed with 32-bit byte offsets (a row is at most D / 2 bytes)
    // tiled value codes: 8-bit codes on both sides (the instantiations built)
    // (and not d_v = 8 at D = 64: fewer than the 16 sub-spaces the block order is made of)
    const bool tiled_ok = !p.v_tiled || (p.bk == 8 && p.bv == 8 && p.n_cap % 64 == 0 && !(p.D == 64 && p.dv == 8));
    return (p.D == 128 || p.D == 64) && p.G >= 1 && p.G <= 8 && dk_ok && dv_ok && bits_ok && tiled_ok &&
           (p.v_tiled ? (p.N + 63) / 64 * 64 : p.N) * (long long)(p.D / 2) < (1LL << 31);
}

int launch_decode_mfma(const DecodeParams &p, hipStream_t stream)
{
    if (!decode_mfma_supports(p)) return -2;
    if (p.bk != 8 || p.bv != 8) return p.D == 128 ? launch_decode_mfma_wide128(p, stream) : launch_decode_mfma_wide64(p, stream);
    if (p.v_tiled) return launch_decode_mfma_tiled(p, stream);
    // 8 wavefronts per workgroup (2 per SIMD): 12 measured slower, 4 is latency-bound
    const int key = p.D * 100 + p.dk * 10 + p.dv;
    switch (key) {
    case 12844: return launch_typed<128, 4, 4, 8, true>(p, stream);
    case 12822: return launch_typed<128, 2, 2, 8, true>(p, stream);
    case 12824: return launch_typed<128, 2, 4, 8, true>(p, stream);
    case 12842: return launch_typed<128, 4, 2, 8, true>(p, stream);
    case 12888: return launch_typed<128, 8, 8, 8, true>(p, stream);
    case 12884: return launch_typed<128, 8, 4, 8, true>(p, stream);
    case 12882: return launch_typed<128, 8, 2, 8, true>(p, stream);
    case 12848: return launch_typed<128, 4, 8, 8, true>(p, stream);
    case 12828: return launch_typed<128, 2, 8, 8, true>(p, stream);
    case 6488: return launch_typed<64, 8, 8, 8, true>(p, stream);
    case 6448: return launch_typed<64, 4, 8, 8, true>(p, stream);
    case 6428: return launch_typed<64, 2, 8, 8, true>(p, stream);
    case 6484: return launch_typed<64, 8, 4, 8, true>(p, stream);
    case 6482: return launch_typed<64, 8, 2, 8, true>(p, stream);
    case 6444: return launch_typed<64, 4, 4, 8, true>(p, stream);
    case 6422: return launch_typed<64, 2, 2, 8, true>(p, stream);
    case 6424: return launch_typed<64, 2, 4, 8, true>(p, stream);
    case 6442: return launch_typed<64, 4, 2, 8, true>(p, stream);
    default: return -2;
    }
}

} // namespace vecinfer
