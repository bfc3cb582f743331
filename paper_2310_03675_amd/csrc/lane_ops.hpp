// Lane-level building blocks of the tuned quantization kernels (gfx950):
// cross-lane butterfly stages, the in-register butterfly over eight values,
// and rounding / packing of codes through the 1.5 * 2^23 addition.
#pragma once
#include "common.hpp"

namespace hdqt {
namespace lanes {

typedef unsigned v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float as_f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __float_as_uint(f); }

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// value held by lane (lane ^ M), M in {1, 2, 4, 8}
template <int M>
__device__ __forceinline__ float lane_xor(float x)
{
    if (M == 1) return dpp_move<0xB1>(x);                      // quad_perm [1,0,3,2]
    if (M == 2) return dpp_move<0x4E>(x);                      // quad_perm [2,3,0,1]
    if (M == 4) return dpp_move<0x1B>(dpp_move<0x141>(x));     // half-row mirror, then quad reverse
    return dpp_move<0x128>(x);                                 // row rotate by 8
}

// Butterfly stage pairing lane and lane ^ M.  `flip` is 0x80000000 in the lane
// that holds the upper half (it computes other - own) and 0 in the other.
template <int M>
__device__ __forceinline__ float stage_dpp(float own, uint32_t flip)
{
    return lane_xor<M>(own) + as_f(as_u(own) ^ flip);
}

// The same stage in one multiply-add: own + c * other with c = +1 in the lane that
// holds the lower half and -1 in the other (multiplying by +-1 is exact, so the
// rounding is that of the plain sum).  The lower lane gets lower + upper as
// before; the upper lane gets upper - lower, the NEGATED butterfly output.  A
// caller therefore tracks one sign per lane: with values stored as sigma * true,
// pairs whose two lanes carry the same sigma use c = +-1 as described, and sigma
// flips in the upper lane.  Signs do not matter to max|.|, and a quantizer
// multiplies by sigma * (1 / step) instead of 1 / step.
// Written as v_fmac_f32 with a DPP source, eight values per statement: the
// compiler keeps the lane move and the multiply-add apart (two instructions per
// value), the hardware does both in one.  A DPP source may not be read within
// two wait states of the VALU instruction that wrote it; inside a statement the
// eight values are independent, and the s_nop at either end covers the
// instructions around it.
#define HDQT_FMA8(CTRL)                                                                           \
    asm("s_nop 1\n\t"                                                                             \
        "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                       \
        "s_nop 1"                                                                                 \
        : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]),     \
          "+v"(w[7])                                                                              \
        : "v"(c))

// w[k] <- w[k] + c * (w[k] of lane ^ M), k < 8, M in {1, 2, 4, 8}
template <int M>
__device__ __forceinline__ void stage_fma8(float w[8], float c)
{
    if (M == 1) {
        HDQT_FMA8("quad_perm:[1,0,3,2]");
    } else if (M == 2) {
        HDQT_FMA8("quad_perm:[2,3,0,1]");
    } else if (M == 8) {
        HDQT_FMA8("row_ror:8");
    } else {
        // lane ^ 4 = half-row mirror, then quad reverse: eight moves, then eight multiply-adds
        float t[8];
        asm("s_nop 1\n\t"
            "v_mov_b32_dpp %0, %8 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_dpp %1, %9 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_dpp %2, %10 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_dpp %3, %11 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_dpp %4, %12 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_dpp %5, %13 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_dpp %6, %14 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "v_mov_b32_dpp %7, %15 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
            "s_nop 1"
            : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]),
              "=&v"(t[7])
            : "v"(w[0]), "v"(w[1]), "v"(w[2]), "v"(w[3]), "v"(w[4]), "v"(w[5]), "v"(w[6]), "v"(w[7]));
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %8, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %1, %9, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %2, %10, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %3, %11, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %4, %12, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %5, %13, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %6, %14, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %7, %15, %16 quad_perm:[3,2,1,0] row_mask:0xf bank_mask:0xf\n\t"
            "s_nop 1"
            : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]), "+v"(w[4]), "+v"(w[5]), "+v"(w[6]),
              "+v"(w[7])
            : "v"(t[0]), "v"(t[1]), "v"(t[2]), "v"(t[3]), "v"(t[4]), "v"(t[5]), "v"(t[6]), "v"(t[7]),
              "v"(c));
    }
}

// Butterfly stage pairing lane and lane ^ 16 (W32 = false) or lane ^ 32 (true),
// on two values at once.  The swap brings, into one lane, the two halves of a
// pair (of `a` in the lower lanes, of `b` in the upper lanes); sum and
// difference are formed there and swapped back.
template <bool W32>
__device__ __forceinline__ void stage_swap(float& a, float& b)
{
    v2u r = W32 ? __builtin_amdgcn_permlane32_swap(as_u(a), as_u(b), false, false)
                : __builtin_amdgcn_permlane16_swap(as_u(a), as_u(b), false, false);
    const float lo = as_f(r[0]), hi = as_f(r[1]);
    const float s = lo + hi, d = lo - hi;
    r = W32 ? __builtin_amdgcn_permlane32_swap(as_u(s), as_u(d), false, false)
            : __builtin_amdgcn_permlane16_swap(as_u(s), as_u(d), false, false);
    a = as_f(r[0]);
    b = as_f(r[1]);
}

// strides 1, 2, 4 over eight register values, limited to strides < 2^log2n
__device__ __forceinline__ void butterfly8(float v[8], int log2n)
{
    if (log2n >= 1) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            const float a = v[i], c = v[i + 1];
            v[i] = a + c;
            v[i + 1] = a - c;
        }
    }
    if (log2n >= 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (!(i & 2)) {
                const float a = v[i], c = v[i + 2];
                v[i] = a + c;
                v[i + 2] = a - c;
            }
    }
    if (log2n >= 3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float a = v[i], c = v[i + 4];
            v[i] = a + c;
            v[i + 4] = a - c;
        }
    }
}

__device__ __forceinline__ float wave_max(float m)
{
    m = fmaxf(m, lane_xor<1>(m));
    m = fmaxf(m, lane_xor<2>(m));
    m = fmaxf(m, lane_xor<4>(m));
    m = fmaxf(m, lane_xor<8>(m));
    m = fmaxf(m, __shfl_xor(m, 16, kWave));
    m = fmaxf(m, __shfl_xor(m, 32, kWave));
    return m;
}

// ---- rounding and packing -------------------------------------------------
// code_word() returns 0x4B400000 + code + offset, offset = 8 (b <= 4) or 128:
// adding 1.5 * 2^23 (+ offset) to a binary32 value of magnitude below 2^22 rounds
// it to the nearest integer, ties to even, and leaves that integer in the low
// mantissa bits.  The clamp is applied first; clamp and rounding commute because
// the bounds are integers.  The stochastic path adds the same constant to an
// integer, which is exact.
constexpr float kMagic = 12582912.0f;          // 1.5 * 2^23, bit pattern 0x4B400000
constexpr uint32_t kMagicBits = 0x4B400000u;

template <bool STOCH>
__device__ __forceinline__ uint32_t code_word(float y, float inv, float qminf, float qmaxf,
                                              float magic, uint32_t u16)
{
    const float v = y * inv;
    if (!STOCH) return __float_as_uint(__builtin_amdgcn_fmed3f(v, qminf, qmaxf) + magic);
    const float fl = floorf(v);
    const float frac = v - fl;
    const float up = fl + (((float)u16 < frac * 65536.0f) ? 1.0f : 0.0f);
    return __float_as_uint(__builtin_amdgcn_fmed3f(up, qminf, qmaxf) + magic);
}

constexpr uint32_t pack_bias(int fields, int width)
{
    uint32_t c = 0;
    for (int i = 0; i < fields; ++i) c += kMagicBits << (width * i);
    return c;
}

// eight words -> eight two's-complement nibbles (low nibble = first code)
__device__ __forceinline__ uint32_t pack_nibbles(const uint32_t w[8])
{
    uint32_t acc = w[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) acc += w[i] << (4 * i);
    return (acc - pack_bias(8, 4)) ^ 0x88888888u;
}

// four words -> four two's-complement bytes
__device__ __forceinline__ uint32_t pack_bytes(const uint32_t w[4])
{
    uint32_t acc = w[0];
#pragma unroll
    for (int i = 1; i < 4; ++i) acc += w[i] << (8 * i);
    return (acc - pack_bias(4, 8)) ^ 0x80808080u;
}

} // namespace lanes
} // namespace hdqt
