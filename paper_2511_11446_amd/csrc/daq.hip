// Dynamic activation quantization kernels for gfx950 (wave64).
//
// Step 3, eq. (4) of the paper with tau = the absolute maximum of the scale
// block: alpha = amax / 127 (1 for an all-zero block),
// code = clamp(round_half_even(x / alpha), -127, 127).
//
// One wavefront owns one or a few rows.  A row is read once with 16-byte loads and
// kept in registers (2 bytes in, 1 byte out per element is all the HBM traffic
// of the per-token mode).  The absolute maximum is taken on the fp16 bit
// patterns: for non-negative binary16 numbers the integer order of the
// patterns is the numeric order, so a packed 16-bit integer max is exact.
#include "daq_device.h"

namespace ql {

__device__ __forceinline__ void publish_block_max(unsigned *slot, unsigned bits)
{
    // most rows lose against an earlier, larger maximum: look before the atomic
    if (__hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < bits) atomicMax(slot, bits);
}

// Second pass of the modes with several rows per scale: the maximum of scale block b, either reduced already
// (blockmax) or, when the block has few parts, taken here from its partial maxima (saves a launch)
__device__ __forceinline__ unsigned block_max_bits(const DaqArgs &a, int b, int lane)
{
    if (a.quant_parts <= 0) return a.blockmax[b];
    const unsigned *pm = a.partmax + (size_t)b * a.quant_parts;
    unsigned m = 0;
    for (int i = lane; i < a.quant_parts; i += 64) {
        const unsigned o = pm[i];
        m = m > o ? m : o;
    }
    return wave_max_u32(m);
}

constexpr int ROWS_PER_BLOCK = 4;  // 4 wavefronts, one row each (loop kernels)

// Rows held in registers: CH 16-byte chunks per lane and row (K/8 <= 64*CH), RW rows per wavefront (all loads of the
// RW rows are issued before the first reduction).  The dispatcher uses RW = 1: see run_rows().
template <int CH, int RW>
__global__ __launch_bounds__(256) void daq_rows_cached(DaqArgs a, int mode)
{
    const int lane = threadIdx.x & 63;
    // the second pass of the two-pass modes walks the rows backwards: the rows read last by the first pass are
    // the ones most likely still in cache
    const int wg = mode == DAQ_QUANT ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
    const int row0 = (wg * 4 + (threadIdx.x >> 6)) * RW;
    if (row0 >= a.M) return;
    const int nch = a.K >> 3;
    uint4 v[RW][CH];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int row = min(row0 + r, a.M - 1);
        const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.x) + (size_t)row * a.K);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = lane + 64 * i;
            v[r][i] = c < nch ? xr[c] : make_uint4(0, 0, 0, 0);
        }
    }
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int row = row0 + r;
        if (row >= a.M) break;
        unsigned bits;
        if (mode != DAQ_QUANT) {
            unsigned m = 0;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                m = absmax_word(m, v[r][i].x);
                m = absmax_word(m, v[r][i].y);
                m = absmax_word(m, v[r][i].z);
                m = absmax_word(m, v[r][i].w);
            }
            m = (m & 0xffffu) > (m >> 16) ? (m & 0xffffu) : (m >> 16);
            bits = wave_max_u32(m);
            if (mode == DAQ_ABSMAX) {
                if (lane == 0) publish_block_max(a.blockmax + row / a.R, bits);
                continue;
            }
        } else {
            bits = block_max_bits(a, row / a.R, lane);
        }
        const float alpha = alpha_from_bits(bits);
        const float rcp = 1.0f / alpha;
        if (lane == 0 && (row % a.R) == 0) a.scales[row / a.R] = alpha;
        uint2 *qr = reinterpret_cast<uint2 *>(a.q + (size_t)row * a.K);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = lane + 64 * i;
            if (c < nch) qr[c] = daq_piece(v[r][i], alpha, rcp);
        }
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
        bits = block_max_bits(a, row / a.R, lane);
    }
    const float alpha = alpha_from_bits(bits);
    const float rcp = 1.0f / alpha;
    if (lane == 0 && (row % a.R) == 0) a.scales[row / a.R] = alpha;
    int8_t *qs = a.q + (size_t)row * a.K;
    for (int c = lane; c < nch; c += 64) {
        if (VEC == 8) {
            uint4 v = reinterpret_cast<const uint4 *>(xs)[c];
            reinterpret_cast<uint2 *>(qs)[c] = daq_piece(v, alpha, rcp);
        } else {
            qs[c] = (int8_t)daq_code(half_bits_to_float(xs[c]), alpha);
        }
    }
}

// First pass of the modes with several rows per scale: a scale block is one contiguous run of R*K values, cut into
// parts of DAQ_PART_PIECES 16-byte pieces; one workgroup per part leaves the part's maximum in partmax (plain stores:
// thousands of atomics on a few neighbouring words cost more than the whole pass).
constexpr int ABSMAX_U = DAQ_PART_PIECES / 256;
__global__ __launch_bounds__(256) void daq_part_absmax(const uint4 *x, unsigned pieces_per_block, unsigned parts_per_block,
                                                       unsigned *partmax)
{
    __shared__ unsigned wave_max[4];
    const unsigned b = blockIdx.x / parts_per_block, part = blockIdx.x - b * parts_per_block;
    const uint4 *xb = x + (size_t)b * pieces_per_block;
    const unsigned c0 = part * DAQ_PART_PIECES + threadIdx.x;
    uint4 v[ABSMAX_U];
#pragma unroll
    for (int i = 0; i < ABSMAX_U; ++i) {
        const unsigned c = c0 + 256 * i;
        v[i] = c < pieces_per_block ? xb[c] : make_uint4(0, 0, 0, 0);
    }
    unsigned m = 0;
#pragma unroll
    for (int i = 0; i < ABSMAX_U; ++i) {
        m = absmax_word(m, v[i].x);
        m = absmax_word(m, v[i].y);
        m = absmax_word(m, v[i].z);
        m = absmax_word(m, v[i].w);
    }
    m = (m & 0xffffu) > (m >> 16) ? (m & 0xffffu) : (m >> 16);
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned m01 = wave_max[0] > wave_max[1] ? wave_max[0] : wave_max[1];
        const unsigned m23 = wave_max[2] > wave_max[3] ? wave_max[2] : wave_max[3];
        partmax[blockIdx.x] = m01 > m23 ? m01 : m23;
    }
}

// one workgroup per scale block: maximum of its partial maxima
__global__ __launch_bounds__(256) void daq_reduce_parts(const unsigned *partmax, unsigned parts_per_block, unsigned *blockmax)
{
    __shared__ unsigned wave_max[4];
    const unsigned *pm = partmax + (size_t)blockIdx.x * parts_per_block;
    unsigned m = 0;
    for (unsigned i = threadIdx.x; i < parts_per_block; i += 256) {
        const unsigned o = pm[i];
        m = m > o ? m : o;
    }
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned m01 = wave_max[0] > wave_max[1] ? wave_max[0] : wave_max[1];
        const unsigned m23 = wave_max[2] > wave_max[3] ? wave_max[2] : wave_max[3];
        blockmax[blockIdx.x] = m01 > m23 ? m01 : m23;
    }
}

__global__ void fill_u32(unsigned *p, int n, unsigned v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

template <int CH, int RW>
static void run_cached(const DaqArgs &a, int mode, hipStream_t s)
{
    dim3 grid((a.M + 4 * RW - 1) / (4 * RW));
    hipLaunchKernelGGL((daq_rows_cached<CH, RW>), grid, dim3(256), 0, s, a, mode);
}

static void run_rows(const DaqArgs &a, int mode, hipStream_t s)
{
    dim3 grid((a.M + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK);
    const bool vec = (a.K % 8 == 0) && ((uintptr_t)a.x % 16 == 0) && ((uintptr_t)a.q % 8 == 0);
    if (!vec) {
        hipLaunchKernelGGL(daq_rows_loop<1>, grid, dim3(256), 0, s, a, mode);
        return;
    }
    // one row per wavefront at every size: with the division-free codes the kernel is no longer VALU-bound, and more,
    // shorter wavefronts beat several rows per wavefront (measured 4.5 against 3.4 TB/s at M = 16384, K = 1152)
    const int per_lane = (a.K / 8 + 63) / 64;
    if (per_lane <= 1) run_cached<1, 1>(a, mode, s);
    else if (per_lane <= 2) run_cached<2, 1>(a, mode, s);
    else if (per_lane <= 3) run_cached<3, 1>(a, mode, s);
    else if (per_lane <= 4) run_cached<4, 1>(a, mode, s);
    else if (per_lane <= 6) run_cached<6, 1>(a, mode, s);
    else if (per_lane <= 9) run_cached<9, 1>(a, mode, s);
    else if (per_lane <= 12) run_cached<12, 1>(a, mode, s);
    else if (per_lane <= 16) run_cached<16, 1>(a, mode, s);
    else hipLaunchKernelGGL(daq_rows_loop<8>, grid, dim3(256), 0, s, a, mode);
}

// ---- eq. (4) with its channel groups: one scale per block of R rows AND group of `cg` consecutive channels ------------
// pass 1: every wavefront takes one row; a lane's 16-byte piece lies inside one channel group (cg % 8 == 0), its maximum
// goes to the wavefront's LDS table and from there, once per row and group, to blockmax[block][group]
constexpr int DAQ_CG_MAX_GROUPS = 1024;
__global__ __launch_bounds__(256) void daq_cg_absmax(DaqArgs a, int cg)
{
    __shared__ unsigned gmax[4][DAQ_CG_MAX_GROUPS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wave;
    const int G = a.K / cg, nch = a.K >> 3;
    for (int g = lane; g < G; g += 64) gmax[wave][g] = 0;
    __builtin_amdgcn_wave_barrier();
    if (row < a.M) {
        const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.x) + (size_t)row * a.K);
        for (int c = lane; c < nch; c += 64) {
            const uint4 v = xr[c];
            unsigned m = absmax_word(absmax_word(absmax_word(absmax_word(0, v.x), v.y), v.z), v.w);
            m = (m & 0xffffu) > (m >> 16) ? (m & 0xffffu) : (m >> 16);
            atomicMax(&gmax[wave][(c * 8) / cg], m);
        }
    }
    __syncthreads();
    if (row < a.M)
        for (int g = lane; g < G; g += 64) publish_block_max(a.blockmax + (size_t)(row / a.R) * G + g, gmax[wave][g]);
}

// pass 2: codes from the block maxima; the row is read again (the first read normally left it in L2)
__global__ __launch_bounds__(256) void daq_cg_quant(DaqArgs a, int cg)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const int G = a.K / cg, nch = a.K >> 3;
    const unsigned *bm = a.blockmax + (size_t)(row / a.R) * G;
    const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.x) + (size_t)row * a.K);
    uint2 *qr = reinterpret_cast<uint2 *>(a.q + (size_t)row * a.K);
    for (int c = lane; c < nch; c += 64) {
        const float alpha = alpha_from_bits(bm[(c * 8) / cg]);
        qr[c] = daq_piece(xr[c], alpha, 1.0f / alpha);
    }
    if (row % a.R == 0)
        for (int g = lane; g < G; g += 64) a.scales[(size_t)(row / a.R) * G + g] = alpha_from_bits(bm[g]);
}

hipError_t launch_daq_cg(const DaqArgs &a, int cg, hipStream_t stream)
{
    const int n = (a.M / a.R) * (a.K / cg);
    hipLaunchKernelGGL(fill_u32, dim3((n + 255) / 256), dim3(256), 0, stream, a.blockmax, n, 0u);
    hipLaunchKernelGGL(daq_cg_absmax, dim3((a.M + 3) / 4), dim3(256), 0, stream, a, cg);
    hipLaunchKernelGGL(daq_cg_quant, dim3((a.M + 3) / 4), dim3(256), 0, stream, a, cg);
    return hipGetLastError();
}

hipError_t launch_daq(const DaqArgs &a, hipStream_t stream)
{
    if (a.R == 1) {
        run_rows(a, DAQ_FUSED, stream);
    } else {
        const int nblk = a.M / a.R;
        const size_t parts = daq_parts_per_block(a.K, a.R);
        if (parts > 0 && (uintptr_t)a.x % 16 == 0 && parts * nblk < (1ull << 31)) {
            hipLaunchKernelGGL(daq_part_absmax, dim3((unsigned)(parts * nblk)), dim3(256), 0, stream,
                               static_cast<const uint4 *>(a.x), (unsigned)((size_t)a.R * a.K / 8), (unsigned)parts, a.partmax);
            if (parts <= 256) {
                // few parts per block: every wavefront of the quantize pass reduces them itself
                DaqArgs q = a;
                q.quant_parts = (int)parts;
                run_rows(q, DAQ_QUANT, stream);
                return hipGetLastError();
            }
            hipLaunchKernelGGL(daq_reduce_parts, dim3(nblk), dim3(256), 0, stream, a.partmax, (unsigned)parts, a.blockmax);
        } else {
            hipLaunchKernelGGL(fill_u32, dim3((nblk + 255) / 256), dim3(256), 0, stream, a.blockmax, nblk, 0u);
            run_rows(a, DAQ_ABSMAX, stream);
        }
        run_rows(a, DAQ_QUANT, stream);
    }
    return hipGetLastError();
}

hipError_t launch_fill_u32(unsigned *p, int n, unsigned v, hipStream_t stream)
{
    hipLaunchKernelGGL(fill_u32, dim3((n + 255) / 256), dim3(256), 0, stream, p, n, v);
    return hipGetLastError();
}

// The first pass is already done: the producing layer's epilogue left every row's maximum.  A block's R row maxima are
// laid out like the partial maxima of the two-pass modes, so the quantize pass reduces them itself (R <= 256) or after
// one reduction launch.
hipError_t launch_daq_from_rowmax(const DaqArgs &a, const unsigned *row_absmax, hipStream_t stream)
{
    DaqArgs q = a;
    q.partmax = const_cast<unsigned *>(row_absmax);
    if (a.R <= 256) {
        q.quant_parts = a.R;
    } else {
        hipLaunchKernelGGL(daq_reduce_parts, dim3(a.M / a.R), dim3(256), 0, stream, row_absmax, (unsigned)a.R, a.blockmax);
        q.quant_parts = 0;
    }
    run_rows(q, DAQ_QUANT, stream);
    return hipGetLastError();
}

}  // namespace ql
