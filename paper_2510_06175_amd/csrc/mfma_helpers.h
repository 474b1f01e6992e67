// Small device helpers shared by the matrix-core decode kernels: LDS loads from absolute addresses,
// DPP / permlane cross-lane primitives, operand packing.
#pragma once
#include "common.h"

namespace vecinfer {

namespace {

#define MFMA16(a, b, c, x, y, z) __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, x, y, z)

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned short ushortx2 __attribute__((ext_vector_type(2)));

constexpr int kG = 4;              // head slots of one MFMA pass; spare slots (G not a multiple of 4) run on a zero query
constexpr int kTile = 64;          // tokens per wavefront iteration (4 sub-tiles of 16)
// Cache policy of the code-stream loads (aux argument of the raw buffer loads): non-temporal.  The
// codes are read once, so they need not displace the codebooks, q and the partials from the L2
// and the Infinity Cache: 0.7 us per call at 196608 tokens against the default policy.
constexpr int kStreamPolicy = 2;

// loads from an absolute LDS byte address
__device__ __forceinline__ uint2 lds_load_b64(unsigned addr)
{
    typedef uintx2 __attribute__((address_space(3))) *lds_ptr;
    const uintx2 v = *(lds_ptr)(addr);
    return make_uint2(v[0], v[1]);
}
__device__ __forceinline__ unsigned lds_load_b32(unsigned addr)
{
    typedef unsigned __attribute__((address_space(3))) *lds_ptr;
    return *(lds_ptr)(addr);
}

__device__ __forceinline__ uintx4 lds_load_b128(unsigned addr)
{
    typedef uintx4 __attribute__((address_space(3))) *lds_ptr;
    return *(lds_ptr)(addr);
}

__device__ __forceinline__ half8 as_half8(unsigned a, unsigned b, unsigned c, unsigned d)
{
    uintx4 u = {a, b, c, d};
    return __builtin_bit_cast(half8, u);
}

// value of quad lane L (0..3) broadcast to the whole quad (DPP quad_perm:[L,L,L,L])
template <int L>
__device__ __forceinline__ unsigned quad_bcast(unsigned x)
{
    return (unsigned)__builtin_amdgcn_mov_dpp((int)x, L * 0x55, 0xf, 0xf, true);
}

// value of the lane whose index within the quad differs by XOR (1 or 2)
template <int XOR>
__device__ __forceinline__ float quad_xor(float x)
{
    constexpr int ctrl = XOR == 1 ? 0xB1 : 0x4E;     // quad_perm:[1,0,3,2] / [2,3,0,1]
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), ctrl, 0xf, 0xf, true));
}

// max over the four 16-lane rows of the wavefront, on the vector ALU (v_permlane16_swap /
// v_permlane32_swap exchange rows between two copies of the value; no LDS round trip)
__device__ __forceinline__ float rows_max(float x)
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    auto s16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    float m = fmaxf(__builtin_bit_cast(float, (unsigned)s16[0]), __builtin_bit_cast(float, (unsigned)s16[1]));
    const unsigned w = __builtin_bit_cast(unsigned, m);
    auto s32 = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    return fmaxf(__builtin_bit_cast(float, (unsigned)s32[0]), __builtin_bit_cast(float, (unsigned)s32[1]));
}

// unsigned minimum over the wavefront, in every lane: DPP inside the 16-lane rows
// (quad_perm xor 1, 2, then row rotations by 4 and 8), row swaps across them
__device__ __forceinline__ unsigned wave_umin(unsigned x)
{
    auto dpp = [](unsigned v, auto ctrl) {
        return (unsigned)__builtin_amdgcn_mov_dpp((int)v, decltype(ctrl)::value, 0xf, 0xf, true);
    };
    x = min(x, dpp(x, std::integral_constant<int, 0xB1>{}));      // quad_perm:[1,0,3,2]
    x = min(x, dpp(x, std::integral_constant<int, 0x4E>{}));      // quad_perm:[2,3,0,1]
    x = min(x, dpp(x, std::integral_constant<int, 0x124>{}));     // row_ror:4
    x = min(x, dpp(x, std::integral_constant<int, 0x128>{}));     // row_ror:8
    auto s16 = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    x = min((unsigned)s16[0], (unsigned)s16[1]);
    auto s32 = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return min((unsigned)s32[0], (unsigned)s32[1]);
}

__device__ __forceinline__ unsigned pack_dup_f16(float p)
{
    // (p, p) as two fp16, round-to-nearest-even (one packed conversion)
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    const half2v h = {(_Float16)p, (_Float16)p};
    return __builtin_bit_cast(unsigned, h);
}

} // namespace

} // namespace vecinfer
