// Matrix-core decode attention, 8-bit codes with the value codes stored in tiles of 64 tokens
// (cfg.v_tiled): instantiations and dispatch (kernel: decode_mfma_kernel.h).
#include "decode_mfma_kernel.h"

namespace vecinfer {

int launch_decode_mfma_tiled(const DecodeParams &p, hipStream_t stream)
{
    if (!decode_mfma_supports(p) || !p.v_tiled || p.bk != 8 || p.bv != 8) return -2;
    const int key = p.D * 100 + p.dk * 10 + p.dv;
    switch (key) {
    case 12844: return launch_typed<128, 4, 4, 8, true, 8, 8, true>(p, stream);
    case 12822: return launch_typed<128, 2, 2, 8, true, 8, 8, true>(p, stream);
    case 12824: return launch_typed<128, 2, 4, 8, true, 8, 8, true>(p, stream);
    case 12842: return launch_typed<128, 4, 2, 8, true, 8, 8, true>(p, stream);
    case 12888: return launch_typed<128, 8, 8, 8, true, 8, 8, true>(p, stream);
    case 12884: return launch_typed<128, 8, 4, 8, true, 8, 8, true>(p, stream);
    case 12882: return launch_typed<128, 8, 2, 8, true, 8, 8, true>(p, stream);
    case 12848: return launch_typed<128, 4, 8, 8, true, 8, 8, true>(p, stream);
    case 12828: return launch_typed<128, 2, 8, 8, true, 8, 8, true>(p, stream);
    case 6484: return launch_typed<64, 8, 4, 8, true, 8, 8, true>(p, stream);
    case 6482: return launch_typed<64, 8, 2, 8, true, 8, 8, true>(p, stream);
    case 6444: return launch_typed<64, 4, 4, 8, true, 8, 8, true>(p, stream);
    case 6422: return launch_typed<64, 2, 2, 8, true, 8, 8, true>(p, stream);
    case 6424: return launch_typed<64, 2, 4, 8, true, 8, 8, true>(p, stream);
    case 6442: return launch_typed<64, 4, 2, 8, true, 8, 8, true>(p, stream);
    default: return -2;
    }
}

} // namespace vecinfer
