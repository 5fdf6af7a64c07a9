// Dynamic activation quantization kernels for gfx950 (wave64).
//
// Step 3, eq. (4) of the paper with tau = the absolute maximum of the scale
// block: alpha = amax / 127 (1 for an all-zero block),
// code = clamp(round_half_even(x / alpha), -127, 127).
//
// One wavefront owns one row.  The row is read once with 16-byte loads and
// kept in registers (2 bytes in, 1 byte out per element is all the HBM traffic
// of the per-token mode).  The absolute maximum is taken on the fp16 bit
// patterns: for non-negative binary16 numbers the integer order of the
// patterns is the numeric order, so a packed 16-bit integer max is exact.
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

__device__ __forceinline__ unsigned wave_max_u32(unsigned m)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        unsigned o = (unsigned)__shfl_xor((int)m, off, 64);
        m = m > o ? m : o;
    }
    return m;
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

__device__ __forceinline__ float alpha_from_bits(unsigned amax_bits)
{
    float amax = half_bits_to_float(amax_bits);
    return amax == 0.0f ? 1.0f : amax / 127.0f;
}

__device__ __forceinline__ void publish_block_max(unsigned *slot, unsigned bits)
{
    // most rows lose against an earlier, larger maximum: look before the atomic
    if (__hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < bits) atomicMax(slot, bits);
}

constexpr int ROWS_PER_BLOCK = 4;  // 4 wavefronts, one row each

// Row held in registers: CH 16-byte chunks per lane, K/8 <= 64*CH.
template <int CH>
__global__ __launch_bounds__(256) void daq_rows_cached(DaqArgs a, int mode)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const int nch = a.K >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.x) + (size_t)row * a.K);
    uint4 v[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        int c = lane + 64 * i;
        v[i] = c < nch ? xr[c] : make_uint4(0, 0, 0, 0);
    }
    unsigned bits;
    if (mode != DAQ_QUANT) {
        unsigned m = 0;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            m = absmax_word(m, v[i].x);
            m = absmax_word(m, v[i].y);
            m = absmax_word(m, v[i].z);
            m = absmax_word(m, v[i].w);
        }
        m = (m & 0xffffu) > (m >> 16) ? (m & 0xffffu) : (m >> 16);
        bits = wave_max_u32(m);
        if (mode == DAQ_ABSMAX) {
            if (lane == 0) publish_block_max(a.blockmax + row / a.R, bits);
            return;
        }
    } else {
        bits = a.blockmax[row / a.R];
    }
    const float alpha = alpha_from_bits(bits);
    if (lane == 0 && (row % a.R) == 0) a.scales[row / a.R] = alpha;
    uint2 *qr = reinterpret_cast<uint2 *>(a.q + (size_t)row * a.K);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        int c = lane + 64 * i;
        if (c < nch) qr[c] = make_uint2(daq_pack4(v[i].x, v[i].y, alpha), daq_pack4(v[i].z, v[i].w, alpha));
    }
}

// Any row length: the row is read twice (the second read normally hits L2).
// VEC = 8: 16-byte loads (K % 8 == 0, aligned); VEC = 1: element-wise, no alignment needs.
template <int VEC>
__global__ __launch_bounds__(256) void daq_rows_loop(DaqArgs a, int mode)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const unsigned short *xs = static_cast<const unsigned short *>(a.x) + (size_t)row * a.K;
    const int nch = a.K / VEC;
    unsigned bits;
    if (mode != DAQ_QUANT) {
        unsigned m = 0;
        for (int c = lane; c < nch; c += 64) {
            if (VEC == 8) {
                uint4 v = reinterpret_cast<const uint4 *>(xs)[c];
                m = absmax_word(m, v.x);
                m = absmax_word(m, v.y);
                m = absmax_word(m, v.z);
                m = absmax_word(m, v.w);
            } else {
                m = absmax_word(m, xs[c]);
            }
        }
        m = (m & 0xffffu) > (m >> 16) ? (m & 0xffffu) : (m >> 16);
        bits = wave_max_u32(m);
        if (mode == DAQ_ABSMAX) {
            if (lane == 0) publish_block_max(a.blockmax + row / a.R, bits);
            return;
        }
    } else {
        bits = a.blockmax[row / a.R];
    }
    const float alpha = alpha_from_bits(bits);
    if (lane == 0 && (row % a.R) == 0) a.scales[row / a.R] = alpha;
    int8_t *qs = a.q + (size_t)row * a.K;
    for (int c = lane; c < nch; c += 64) {
        if (VEC == 8) {
            uint4 v = reinterpret_cast<const uint4 *>(xs)[c];
            reinterpret_cast<uint2 *>(qs)[c] = make_uint2(daq_pack4(v.x, v.y, alpha), daq_pack4(v.z, v.w, alpha));
        } else {
            qs[c] = (int8_t)daq_code(half_bits_to_float(xs[c]), alpha);
        }
    }
}

__global__ void fill_u32(unsigned *p, int n, unsigned v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

template <int CH>
static void run_cached(const DaqArgs &a, int mode, dim3 grid, hipStream_t s)
{
    hipLaunchKernelGGL(daq_rows_cached<CH>, grid, dim3(256), 0, s, a, mode);
}

static void run_rows(const DaqArgs &a, int mode, hipStream_t s)
{
    dim3 grid((a.M + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK);
    const bool vec = (a.K % 8 == 0) && ((uintptr_t)a.x % 16 == 0) && ((uintptr_t)a.q % 8 == 0);
    if (!vec) {
        hipLaunchKernelGGL(daq_rows_loop<1>, grid, dim3(256), 0, s, a, mode);
        return;
    }
    const int per_lane = (a.K / 8 + 63) / 64;
    if (per_lane <= 1) run_cached<1>(a, mode, grid, s);
    else if (per_lane <= 2) run_cached<2>(a, mode, grid, s);
    else if (per_lane <= 3) run_cached<3>(a, mode, grid, s);
    else if (per_lane <= 4) run_cached<4>(a, mode, grid, s);
    else if (per_lane <= 6) run_cached<6>(a, mode, grid, s);
    else if (per_lane <= 9) run_cached<9>(a, mode, grid, s);
    else if (per_lane <= 12) run_cached<12>(a, mode, grid, s);
    else if (per_lane <= 16) run_cached<16>(a, mode, grid, s);
    else hipLaunchKernelGGL(daq_rows_loop<8>, grid, dim3(256), 0, s, a, mode);
}

hipError_t launch_daq(const DaqArgs &a, hipStream_t stream)
{
    if (a.R == 1) {
        run_rows(a, DAQ_FUSED, stream);
    } else {
        const int nblk = a.M / a.R;
        hipLaunchKernelGGL(fill_u32, dim3((nblk + 255) / 256), dim3(256), 0, stream, a.blockmax, nblk, 0u);
        run_rows(a, DAQ_ABSMAX, stream);
        run_rows(a, DAQ_QUANT, stream);
    }
    return hipGetLastError();
}

}  // namespace ql
