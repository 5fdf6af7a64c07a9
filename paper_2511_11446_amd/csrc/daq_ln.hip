// LayerNorm + adaptive modulation + dynamic activation quantization in one pass over a row, for gfx950.
//
// In a DiT block the quantized qkv and fc1 layers read  h = LN(x) * (1 + scale_b) + shift_b  (LayerNorm without affine
// parameters; shift and scale per image b from the conditioning), and the paper keeps LayerNorm in higher precision and
// counts it in the latency (Step 3; Section 6).  All three stages are per-row passes over the same row, so the row is
// read once, held in registers, normalised and modulated in fp32, rounded to fp16 (the value the unfused sequence
// would have stored), and quantized as in daq.hip (Step 3, eq. (4) with tau = the row's absolute maximum):
//   mu = mean(x),  var = mean((x - mu)^2),  n = (x - mu) / sqrt(var + eps)
//   h  = fp16(fma(n, 1 + scale[b,k], shift[b,k]))
//   alpha = max|h| / 127 (1 if zero),  q = clamp(rne(h / alpha), -127, 127)
#include "daq_device.h"

namespace ql {

__device__ __forceinline__ float wave_sum_f32(float v)
{
#define QL_ROR_ADDF(ctrl) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xF, 0xF, false));
    QL_ROR_ADDF(0x128)  // row_ror:8
    QL_ROR_ADDF(0x124)  // row_ror:4
    QL_ROR_ADDF(0x122)  // row_ror:2
    QL_ROR_ADDF(0x121)  // row_ror:1
#undef QL_ROR_ADDF
    const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (a + b) + (c + d);
}

typedef _Float16 h2v __attribute__((ext_vector_type(2)));

// one word (two fp16) of the row: normalise, modulate, round to fp16
__device__ __forceinline__ unsigned ln_word(unsigned xw, unsigned sw, unsigned bw, float mu, float rstd, bool has_scale, bool has_shift)
{
    const h2v x = __builtin_bit_cast(h2v, xw), s = __builtin_bit_cast(h2v, sw), b = __builtin_bit_cast(h2v, bw);
    h2v o;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const float n = ((float)x[e] - mu) * rstd;
        const float g = has_scale ? 1.0f + (float)s[e] : 1.0f;
        float t = has_shift ? __builtin_fmaf(n, g, (float)b[e]) : n * g;
        asm volatile("" : "+v"(t));   // keep the fp32 rounding before the fp16 one
        o[e] = (_Float16)t;
    }
    return __builtin_bit_cast(unsigned, o);
}

// CH 16-byte chunks per lane (K/8 <= 64*CH); one wavefront per row
template <int CH>
__global__ __launch_bounds__(256) void daq_ln_rows(LnDaqArgs a)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const int nch = a.K >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.x) + (size_t)row * a.K);
    const size_t mod_row = (size_t)(row / a.rows_per_mod) * a.K;
    const uint4 *sr = a.scale ? reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.scale) + mod_row) : nullptr;
    const uint4 *br = a.shift ? reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.shift) + mod_row) : nullptr;
    uint4 v[CH], sv[CH], bv[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = lane + 64 * i;
        v[i] = c < nch ? xr[c] : make_uint4(0, 0, 0, 0);
        sv[i] = (sr && c < nch) ? sr[c] : make_uint4(0, 0, 0, 0);
        bv[i] = (br && c < nch) ? br[c] : make_uint4(0, 0, 0, 0);
    }
    // mean, then the variance around it (two sums over the registers: no cancellation)
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const unsigned w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) s += half_bits_to_float(w[j] & 0xffffu) + half_bits_to_float(w[j] >> 16);
    }
    const float inv_k = 1.0f / (float)a.K;
    const float mu = wave_sum_f32(s) * inv_k;
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        if (lane + 64 * i < nch) {
            const unsigned w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float d0 = half_bits_to_float(w[j] & 0xffffu) - mu, d1 = half_bits_to_float(w[j] >> 16) - mu;
                ss = __builtin_fmaf(d0, d0, ss);
                ss = __builtin_fmaf(d1, d1, ss);
            }
        }
    }
    const float var = wave_sum_f32(ss) * inv_k;
    const float rstd = 1.0f / __builtin_sqrtf(var + a.eps);
    // h in place of x, and its absolute maximum on the bit patterns
    unsigned m = 0;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        if (lane + 64 * i < nch) {
            v[i].x = ln_word(v[i].x, sv[i].x, bv[i].x, mu, rstd, sr != nullptr, br != nullptr);
            v[i].y = ln_word(v[i].y, sv[i].y, bv[i].y, mu, rstd, sr != nullptr, br != nullptr);
            v[i].z = ln_word(v[i].z, sv[i].z, bv[i].z, mu, rstd, sr != nullptr, br != nullptr);
            v[i].w = ln_word(v[i].w, sv[i].w, bv[i].w, mu, rstd, sr != nullptr, br != nullptr);
        }
        m = absmax_word(m, v[i].x);
        m = absmax_word(m, v[i].y);
        m = absmax_word(m, v[i].z);
        m = absmax_word(m, v[i].w);
    }
    if (a.h) {
        uint4 *hr = reinterpret_cast<uint4 *>(static_cast<unsigned short *>(a.h) + (size_t)row * a.K);
#pragma unroll
        for (int i = 0; i < CH; ++i)
            if (lane + 64 * i < nch) hr[lane + 64 * i] = v[i];
    }
    if (!a.q) return;
    m = (m & 0xffffu) > (m >> 16) ? (m & 0xffffu) : (m >> 16);
    const unsigned bits = wave_max_u32(m);
    const float alpha = alpha_from_bits(bits);
    const float rcp = 1.0f / alpha;
    if (lane == 0) a.scales[row] = alpha;
    uint2 *qr = reinterpret_cast<uint2 *>(a.q + (size_t)row * a.K);
#pragma unroll
    for (int i = 0; i < CH; ++i)
        if (lane + 64 * i < nch) qr[lane + 64 * i] = daq_piece(v[i], alpha, rcp);
}

hipError_t launch_daq_ln(const LnDaqArgs &a, hipStream_t stream)
{
    const dim3 grid((a.M + 3) / 4);
    const int per_lane = (a.K / 8 + 63) / 64;
    if (per_lane <= 1) hipLaunchKernelGGL(daq_ln_rows<1>, grid, dim3(256), 0, stream, a);
    else if (per_lane <= 2) hipLaunchKernelGGL(daq_ln_rows<2>, grid, dim3(256), 0, stream, a);
    else if (per_lane <= 3) hipLaunchKernelGGL(daq_ln_rows<3>, grid, dim3(256), 0, stream, a);
    else if (per_lane <= 6) hipLaunchKernelGGL(daq_ln_rows<6>, grid, dim3(256), 0, stream, a);
    else if (per_lane <= 9) hipLaunchKernelGGL(daq_ln_rows<9>, grid, dim3(256), 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ql
