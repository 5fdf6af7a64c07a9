// Device helpers shared by the DAQ kernels (Step 3, eq. (4)).  Not part of the public ABI.
#pragma once
#include "ql_internal.h"

namespace ql {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float half_bits_to_float(unsigned h)
{
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// running packed max of |a|,|b| over the two fp16 lanes of a word
__device__ __forceinline__ unsigned absmax_word(unsigned m, unsigned w)
{
    us2 a = __builtin_bit_cast(us2, w & 0x7fff7fffu);
    us2 b = __builtin_bit_cast(us2, m);
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(a, b));
}

// maximum over the 64 lanes: rotations inside each row of 16 lanes (DPP, no LDS traffic), then the four row
// results are combined in scalar registers; the result is wave-uniform
__device__ __forceinline__ unsigned wave_max_u32(unsigned m)
{
#define QL_ROR_MAX(ctrl)                                                                       \
    {                                                                                          \
        const unsigned o = (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, ctrl, 0xF, 0xF, false); \
        m = m > o ? m : o;                                                                     \
    }
    QL_ROR_MAX(0x128)  // row_ror:8
    QL_ROR_MAX(0x124)  // row_ror:4
    QL_ROR_MAX(0x122)  // row_ror:2
    QL_ROR_MAX(0x121)  // row_ror:1
#undef QL_ROR_MAX
    const unsigned a = (unsigned)__builtin_amdgcn_readlane((int)m, 0), b = (unsigned)__builtin_amdgcn_readlane((int)m, 16);
    const unsigned c = (unsigned)__builtin_amdgcn_readlane((int)m, 32), d = (unsigned)__builtin_amdgcn_readlane((int)m, 48);
    const unsigned ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

// eq. (4), last line without the multiplication back by alpha
__device__ __forceinline__ int daq_code(float v, float alpha)
{
    float t = v / alpha;                 // IEEE correctly rounded fp32 division
    float r = __builtin_rintf(t);        // round half to even
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// four fp16 values (two words) -> four int8 codes in one word, lowest k in the lowest byte
__device__ __forceinline__ unsigned daq_pack4(unsigned w0, unsigned w1, float alpha)
{
    int c0 = daq_code(half_bits_to_float(w0 & 0xffffu), alpha);
    int c1 = daq_code(half_bits_to_float(w0 >> 16), alpha);
    int c2 = daq_code(half_bits_to_float(w1 & 0xffffu), alpha);
    int c3 = daq_code(half_bits_to_float(w1 >> 16), alpha);
    return (unsigned)(c0 & 0xff) | ((unsigned)(c1 & 0xff) << 8) | ((unsigned)(c2 & 0xff) << 16) | ((unsigned)c3 << 24);
}

// Eight codes of one 16-byte piece without a division per element, bit-identical to daq_code().
//
// With rcp = fl(1/alpha) the exact product p = x*rcp differs from the correctly rounded quotient Q = fl(x/alpha) by at
// most |x/alpha| * 2^-23 <= 1.52e-5 (|x/alpha| <= 127).  y = fma(x, rcp, 1.5*2^23) rounds p to the nearest integer r
// (ties to even) and leaves r's two's-complement byte in the low mantissa bits.  d = fma(x, rcp, -r) is p - r; if
// |d| < 0.5 - 2^-15 then p and Q lie in the same open interval (r - 0.5, r + 0.5), so rint(Q) = r.  Otherwise (6e-5 of
// the elements, every exact tie of Q among them) the piece is redone with the division.  |r| <= 127 follows from
// |x| <= amax, so the clamp of eq. (4) is the identity here.
constexpr float DAQ_MAGIC = 12582912.0f;               // 1.5 * 2^23
constexpr float DAQ_NEAR_TIE = 0.5f - 0.000030517578125f;  // 0.5 - 2^-15

__device__ __forceinline__ unsigned daq_fast_code(unsigned hbits, float rcp, float &dmax)
{
    const float x = half_bits_to_float(hbits);
    const float y = __builtin_fmaf(x, rcp, DAQ_MAGIC);
    const float r = y - DAQ_MAGIC;
    const float d = __builtin_fmaf(x, rcp, -r);
    dmax = fmaxf(dmax, fabsf(d));
    return __builtin_bit_cast(unsigned, y);
}

__device__ __forceinline__ unsigned daq_fast_pack4(unsigned w0, unsigned w1, float rcp, float &dmax)
{
    const unsigned y0 = daq_fast_code(w0 & 0xffffu, rcp, dmax), y1 = daq_fast_code(w0 >> 16, rcp, dmax);
    const unsigned y2 = daq_fast_code(w1 & 0xffffu, rcp, dmax), y3 = daq_fast_code(w1 >> 16, rcp, dmax);
    const unsigned p01 = __builtin_amdgcn_perm(y1, y0, 0x0c0c0400u);  // bytes: y0.0, y1.0, 0, 0
    const unsigned p23 = __builtin_amdgcn_perm(y3, y2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(p23, p01, 0x05040100u);
}

__device__ __forceinline__ uint2 daq_piece(const uint4 &v, float alpha, float rcp)
{
    float dmax = 0.0f;
    uint2 out = make_uint2(daq_fast_pack4(v.x, v.y, rcp, dmax), daq_fast_pack4(v.z, v.w, rcp, dmax));
    if (__builtin_expect(!(dmax < DAQ_NEAR_TIE), 0))
        out = make_uint2(daq_pack4(v.x, v.y, alpha), daq_pack4(v.z, v.w, alpha));
    return out;
}

__device__ __forceinline__ float alpha_from_bits(unsigned amax_bits)
{
    float amax = half_bits_to_float(amax_bits);
    return amax == 0.0f ? 1.0f : amax / 127.0f;
}

}  // namespace ql
