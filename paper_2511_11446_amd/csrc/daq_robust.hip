// Percentile-clipped dynamic activation quantization (Step 3, eq. (4) as printed; activation width b from the
// time-bin policy of Step 6 / Algorithm 2 Phase B) for gfx950.
//
//   tau   = the c-th largest magnitude of the scale block (nearest-rank percentile: c = n - ceil(n p) + 1)
//   alpha = tau / qmax, qmax = 2^(b-1) - 1   (1 if tau = 0)
//   code  = clamp(round_half_even(clip(x, -tau, tau) / alpha), -qmax, qmax)
//
// The selection is exact and works on the 15-bit magnitude patterns of binary16 (their integer order is the numeric
// order).  One row per scale: the row sits in registers and tau is found by a bitwise binary search (15 counting
// rounds over the registers).  Several rows per scale: two histogram passes (upper 8 bits, then the lower 7 bits of
// the values that share the selected upper bits), each followed by a scan that walks the bins from the top.
#include "daq_device.h"

namespace ql {

__device__ __forceinline__ unsigned wave_sum_u32(unsigned m)
{
#define QL_ROR_ADD(ctrl) m += (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, ctrl, 0xF, 0xF, false);
    QL_ROR_ADD(0x128)  // row_ror:8
    QL_ROR_ADD(0x124)  // row_ror:4
    QL_ROR_ADD(0x122)  // row_ror:2
    QL_ROR_ADD(0x121)  // row_ror:1
#undef QL_ROR_ADD
    return (unsigned)__builtin_amdgcn_readlane((int)m, 0) + (unsigned)__builtin_amdgcn_readlane((int)m, 16) +
           (unsigned)__builtin_amdgcn_readlane((int)m, 32) + (unsigned)__builtin_amdgcn_readlane((int)m, 48);
}

// clip to [-tau, tau], then the code with the given full scale (same arithmetic as the oracle's: IEEE division)
__device__ __forceinline__ int robust_code(float v, float tau, float alpha, float qmax)
{
    v = fminf(fmaxf(v, -tau), tau);
    float r = __builtin_rintf(v / alpha);
    r = fminf(fmaxf(r, -qmax), qmax);
    return (int)r;
}

__device__ __forceinline__ unsigned robust_pack4(unsigned w0, unsigned w1, float tau, float alpha, float qmax)
{
    const int c0 = robust_code(half_bits_to_float(w0 & 0xffffu), tau, alpha, qmax);
    const int c1 = robust_code(half_bits_to_float(w0 >> 16), tau, alpha, qmax);
    const int c2 = robust_code(half_bits_to_float(w1 & 0xffffu), tau, alpha, qmax);
    const int c3 = robust_code(half_bits_to_float(w1 >> 16), tau, alpha, qmax);
    return (unsigned)(c0 & 0xff) | ((unsigned)(c1 & 0xff) << 8) | ((unsigned)(c2 & 0xff) << 16) | ((unsigned)c3 << 24);
}

// division-free form, as in daq_piece(): |clip(x)/alpha| <= qmax <= 127, so the same error bound holds
__device__ __forceinline__ unsigned robust_fast_code(unsigned hbits, float tau, float rcp, float &dmax)
{
    float x = half_bits_to_float(hbits);
    x = fminf(fmaxf(x, -tau), tau);
    const float y = __builtin_fmaf(x, rcp, DAQ_MAGIC);
    const float r = y - DAQ_MAGIC;
    const float d = __builtin_fmaf(x, rcp, -r);
    dmax = fmaxf(dmax, fabsf(d));
    return __builtin_bit_cast(unsigned, y);
}

__device__ __forceinline__ uint2 robust_piece(const uint4 &v, float tau, float alpha, float rcp, float qmax)
{
    float dmax = 0.0f;
    unsigned y[8];
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        y[2 * i] = robust_fast_code(w[i] & 0xffffu, tau, rcp, dmax);
        y[2 * i + 1] = robust_fast_code(w[i] >> 16, tau, rcp, dmax);
    }
    uint2 out;
    out.x = __builtin_amdgcn_perm(__builtin_amdgcn_perm(y[3], y[2], 0x0c0c0400u), __builtin_amdgcn_perm(y[1], y[0], 0x0c0c0400u), 0x05040100u);
    out.y = __builtin_amdgcn_perm(__builtin_amdgcn_perm(y[7], y[6], 0x0c0c0400u), __builtin_amdgcn_perm(y[5], y[4], 0x0c0c0400u), 0x05040100u);
    if (__builtin_expect(!(dmax < DAQ_NEAR_TIE), 0))
        out = make_uint2(robust_pack4(v.x, v.y, tau, alpha, qmax), robust_pack4(v.z, v.w, tau, alpha, qmax));
    return out;
}

struct RobustScale {
    float tau, alpha, rcp;
};
__device__ __forceinline__ RobustScale robust_scale(unsigned tau_bits, float qmax)
{
    RobustScale s;
    s.tau = half_bits_to_float(tau_bits);
    s.alpha = s.tau == 0.0f ? 1.0f : s.tau / qmax;
    s.rcp = 1.0f / s.alpha;
    return s;
}

// ---- one row per scale, row in registers ------------------------------------------------------------------------
// mode DAQ_FUSED: select tau, then quantize; mode DAQ_QUANT: tau of the row's block comes from blockmax
template <int CH>
__global__ __launch_bounds__(256) void daq_rows_robust(DaqArgs a, int mode)
{
    const int lane = threadIdx.x & 63;
    const int wg = mode == DAQ_QUANT ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
    const int row = wg * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const int nch = a.K >> 3;
    const uint4 *xr = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(a.x) + (size_t)row * a.K);
    uint4 v[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = lane + 64 * i;
        v[i] = c < nch ? xr[c] : make_uint4(0, 0, 0, 0);
    }
    unsigned tau_bits;
    if (mode == DAQ_QUANT) {
        tau_bits = a.blockmax[row / a.R];
    } else {
        // Each half word is 0x8000 | magnitude (OR-ing 0x8000 in overwrites the sign bit); subtracting T from both
        // halves at once leaves bit 15 of a half set iff its magnitude >= T (no half can borrow from its neighbour:
        // every half result is >= 1).  Lanes past the end of the row hold zeros, which no T >= 1 counts.
        auto count_ge = [&](unsigned t) {
            const unsigned t2 = t * 0x00010001u;
            unsigned cnt = 0;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                cnt += (((v[i].x | 0x80008000u) - t2) >> 15) & 0x00010001u;
                cnt += (((v[i].y | 0x80008000u) - t2) >> 15) & 0x00010001u;
                cnt += (((v[i].z | 0x80008000u) - t2) >> 15) & 0x00010001u;
                cnt += (((v[i].w | 0x80008000u) - t2) >> 15) & 0x00010001u;
            }
            return wave_sum_u32((cnt & 0xffffu) + (cnt >> 16));
        };
        unsigned T = 0;
        if (a.top_rank <= 8) {
            // tau is among the few largest values (the paper's p = 99.9 %: the 2nd largest of 1152, the 5th of 4608):
            // walk down the distinct magnitudes from the top.  One sweep over the registers finds the next magnitude
            // below `prev` and, with the same comparison, counts the values at or above `prev`; the walk ends at the
            // first magnitude with top_rank values at or above it (after at most top_rank + 1 sweeps).
            unsigned prev = 0x8000u;   // above every magnitude: nothing lies at or above it
            for (unsigned pass = 0; pass <= a.top_rank; ++pass) {
                const unsigned p2 = prev * 0x00010001u;
                unsigned m2 = 0, cnt = 0;
                auto sweep = [&](unsigned w) {
                    const unsigned mag = w & 0x7fff7fffu;
                    const unsigned ge = (((mag | 0x80008000u) - p2) >> 15) & 0x00010001u;   // bit 0 / 16: magnitude >= prev
                    cnt += ge;
                    m2 = absmax_word(m2, mag & ((ge ^ 0x00010001u) * 0xffffu));              // the halves below prev
                };
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    sweep(v[i].x);
                    sweep(v[i].y);
                    sweep(v[i].z);
                    sweep(v[i].w);
                }
                if (pass > 0 && wave_sum_u32((cnt & 0xffffu) + (cnt >> 16)) >= a.top_rank) {
                    T = prev;
                    break;
                }
                const unsigned m = wave_max_u32((m2 & 0xffffu) > (m2 >> 16) ? (m2 & 0xffffu) : (m2 >> 16));
                if (m == 0) break;                      // everything left is zero: tau = 0
                prev = m;
            }
        } else {
            // largest T with count(magnitude >= T) >= top_rank, built bit by bit from the top; a candidate above the
            // row maximum cannot succeed and costs no counting round
            unsigned mx = 0;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                mx = absmax_word(mx, v[i].x);
                mx = absmax_word(mx, v[i].y);
                mx = absmax_word(mx, v[i].z);
                mx = absmax_word(mx, v[i].w);
            }
            mx = wave_max_u32((mx & 0xffffu) > (mx >> 16) ? (mx & 0xffffu) : (mx >> 16));
            for (int bit = 14; bit >= 0; --bit) {
                const unsigned cand = T | (1u << bit);
                if (cand <= mx && count_ge(cand) >= a.top_rank) T = cand;
            }
        }
        tau_bits = T;
    }
    const float qmax = (float)a.qmax;
    const RobustScale s = robust_scale(tau_bits, qmax);
    if (lane == 0 && (row % a.R) == 0) a.scales[row / a.R] = s.alpha;
    uint2 *qr = reinterpret_cast<uint2 *>(a.q + (size_t)row * a.K);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) qr[c] = robust_piece(v[i], s.tau, s.alpha, s.rcp, qmax);
    }
}

// any row length and alignment: the row is re-read from memory (cache) in every counting round
__global__ __launch_bounds__(256) void daq_rows_robust_loop(DaqArgs a, int mode)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.M) return;
    const unsigned short *xs = static_cast<const unsigned short *>(a.x) + (size_t)row * a.K;
    unsigned tau_bits;
    if (mode == DAQ_QUANT) {
        tau_bits = a.blockmax[row / a.R];
    } else {
        unsigned T = 0;
        for (int bit = 14; bit >= 0; --bit) {
            const unsigned cand = T | (1u << bit);
            unsigned cnt = 0;
            for (int k = lane; k < a.K; k += 64) cnt += ((unsigned)(xs[k] & 0x7fffu) >= cand) ? 1u : 0u;
            cnt = wave_sum_u32(cnt);
            if (cnt >= a.top_rank) T = cand;
        }
        tau_bits = T;
    }
    const float qmax = (float)a.qmax;
    const RobustScale s = robust_scale(tau_bits, qmax);
    if (lane == 0 && (row % a.R) == 0) a.scales[row / a.R] = s.alpha;
    int8_t *qs = a.q + (size_t)row * a.K;
    for (int k = lane; k < a.K; k += 64) qs[k] = (int8_t)robust_code(half_bits_to_float(xs[k]), s.tau, s.alpha, qmax);
}

// ---- several rows per scale: histogram selection ------------------------------------------------------------------
// Scratch per scale block b (32-bit words): hist[b*HIST_WORDS + 0..255] counts by magnitude bits 14..7,
// [256] the selected upper bits, [257] the rank that is left inside that bin, [258..385] counts by bits 6..0.
constexpr int HIST_WORDS = DAQ_ROBUST_WORDS;
constexpr int HIST_PART = 16384;   // elements per workgroup

// level 0: bins = bits 14..7 of every magnitude; level 1: bins = bits 6..0 of the magnitudes whose upper bits were selected
__global__ __launch_bounds__(256) void daq_hist(const unsigned short *x, size_t n_per_block, unsigned parts_per_block, int level,
                                                unsigned *hist)
{
    __shared__ unsigned h[256];
    const unsigned b = blockIdx.x / parts_per_block, part = blockIdx.x - b * parts_per_block;
    unsigned *hb = hist + (size_t)b * HIST_WORDS;
    h[threadIdx.x] = 0;
    __syncthreads();
    const unsigned prefix = level ? hb[256] : 0;
    const unsigned short *xb = x + (size_t)b * n_per_block;
    const size_t i0 = (size_t)part * HIST_PART;
    const size_t i1 = i0 + HIST_PART < n_per_block ? i0 + HIST_PART : n_per_block;
    const bool vec = ((uintptr_t)(xb + i0) % 16 == 0);
    auto tally = [&](unsigned m) {
        if (level == 0) atomicAdd(&h[m >> 7], 1u);
        else if ((m >> 7) == prefix) atomicAdd(&h[m & 127u], 1u);
    };
    if (vec) {
        const size_t pieces = (i1 - i0) / 8;
        const uint4 *xp = reinterpret_cast<const uint4 *>(xb + i0);
        for (size_t p = threadIdx.x; p < pieces; p += 256) {
            const uint4 v = xp[p];
            const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                tally(w[j] & 0x7fffu);
                tally((w[j] >> 16) & 0x7fffu);
            }
        }
        for (size_t i = i0 + pieces * 8 + threadIdx.x; i < i1; i += 256) tally(xb[i] & 0x7fffu);
    } else {
        for (size_t i = i0 + threadIdx.x; i < i1; i += 256) tally(xb[i] & 0x7fffu);
    }
    __syncthreads();
    const unsigned cnt = h[threadIdx.x];
    if (cnt && (level == 0 || threadIdx.x < 128)) atomicAdd(hb + (level ? 258 : 0) + threadIdx.x, cnt);
}

// one thread per scale block walks the bins from the top until the wanted rank falls inside one
__global__ void daq_hist_select(unsigned *hist, int nblk, int level, unsigned top_rank, unsigned *blockmax)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= nblk) return;
    unsigned *hb = hist + (size_t)b * HIST_WORDS;
    unsigned left = level ? hb[257] : top_rank;
    const unsigned *bins = hb + (level ? 258 : 0);
    int bin = (level ? 128 : 256) - 1;
    for (; bin > 0; --bin) {
        const unsigned c = bins[bin];
        if (c >= left) break;
        left -= c;
    }
    if (level == 0) {
        hb[256] = (unsigned)bin;
        hb[257] = left;
    } else {
        blockmax[b] = (hb[256] << 7) | (unsigned)bin;
    }
}

__global__ void fill_zero_u32(unsigned *p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

template <int CH>
static void run_robust_cached(const DaqArgs &a, int mode, hipStream_t s)
{
    hipLaunchKernelGGL(daq_rows_robust<CH>, dim3((a.M + 3) / 4), dim3(256), 0, s, a, mode);
}

static void run_robust_rows(const DaqArgs &a, int mode, hipStream_t s)
{
    const bool vec = (a.K % 8 == 0) && ((uintptr_t)a.x % 16 == 0) && ((uintptr_t)a.q % 8 == 0);
    const int per_lane = (a.K / 8 + 63) / 64;
    if (!vec || per_lane > 16) {
        hipLaunchKernelGGL(daq_rows_robust_loop, dim3((a.M + 3) / 4), dim3(256), 0, s, a, mode);
        return;
    }
    if (per_lane <= 1) run_robust_cached<1>(a, mode, s);
    else if (per_lane <= 2) run_robust_cached<2>(a, mode, s);
    else if (per_lane <= 3) run_robust_cached<3>(a, mode, s);
    else if (per_lane <= 4) run_robust_cached<4>(a, mode, s);
    else if (per_lane <= 6) run_robust_cached<6>(a, mode, s);
    else if (per_lane <= 9) run_robust_cached<9>(a, mode, s);
    else if (per_lane <= 12) run_robust_cached<12>(a, mode, s);
    else run_robust_cached<16>(a, mode, s);
}

hipError_t launch_daq_robust(const DaqArgs &a, hipStream_t stream)
{
    if (a.R == 1) {
        run_robust_rows(a, DAQ_FUSED, stream);
        return hipGetLastError();
    }
    const int nblk = a.M / a.R;
    const size_t n = (size_t)a.R * a.K;
    const size_t parts = (n + HIST_PART - 1) / HIST_PART;
    const size_t words = (size_t)nblk * HIST_WORDS;
    hipLaunchKernelGGL(fill_zero_u32, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, stream, a.hist, words);
    for (int level = 0; level < 2; ++level) {
        hipLaunchKernelGGL(daq_hist, dim3((unsigned)(parts * nblk)), dim3(256), 0, stream, static_cast<const unsigned short *>(a.x), n,
                           (unsigned)parts, level, a.hist);
        hipLaunchKernelGGL(daq_hist_select, dim3((nblk + 63) / 64), dim3(64), 0, stream, a.hist, nblk, level, a.top_rank, a.blockmax);
    }
    run_robust_rows(a, DAQ_QUANT, stream);
    return hipGetLastError();
}

}  // namespace ql
