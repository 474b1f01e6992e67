// Matrix-core decode attention with score and value wavefronts: instantiations and dispatch
// (kernel: decode_roles_kernel.h).  8-bit codes, D = 128, G <= 4, d_k and d_v in {4, 2}, value
// codes in rows or in tiles.
#include "decode_roles_kernel.h"

namespace vecinfer {

bool decode_roles_supports(const DecodeParams &p)
{
    return p.D == 128 && p.bk == 8 && p.bv == 8 && p.G >= 1 && p.G <= 4 && (p.dk == 4 || p.dk == 2) &&
           (p.dv == 4 || p.dv == 2);
}

int launch_decode_roles(const DecodeParams &p, hipStream_t stream)
{
    if (!decode_roles_supports(p)) return -2;
    const int key = p.dk * 10 + p.dv;
    if (p.v_tiled) {
        switch (key) {
        case 44: return launch_roles<128, 4, 4, true>(p, stream);
        case 22: return launch_roles<128, 2, 2, true>(p, stream);
        case 24: return launch_roles<128, 2, 4, true>(p, stream);
        case 42: return launch_roles<128, 4, 2, true>(p, stream);
        default: return -2;
        }
    }
    switch (key) {
    case 44: return launch_roles<128, 4, 4, false>(p, stream);
    case 22: return launch_roles<128, 2, 2, false>(p, stream);
    case 24: return launch_roles<128, 2, 4, false>(p, stream);
    case 42: return launch_roles<128, 4, 2, false>(p, stream);
    default: return -2;
    }
}

} // namespace vecinfer
