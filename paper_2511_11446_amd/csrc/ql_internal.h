// Internal launch interface between the host API (api.hip) and the kernels.
// Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ql {

// ---- DAQ (Step 3, eq. (4), tau = block absmax) ---------------------------
// mode of the row kernels
enum DaqMode : int {
    DAQ_FUSED = 0,   // per-token: absmax, scale, codes in one pass over a row held in registers
    DAQ_ABSMAX = 1,  // R > 1, phase 1 (fallback): row absmax -> atomic max into blockmax[row / R]
    DAQ_QUANT = 2    // R > 1, phase 2: codes from blockmax[row / R]
};

struct DaqArgs {
    const void *x;       // [M,K] fp16
    int8_t *q;           // [M,K]
    float *scales;       // [M/R]
    unsigned *blockmax;  // [M/R] fp16 bit patterns of block maxima (workspace), R > 1 only
    unsigned *partmax;   // [M/R][daq_parts_per_block] partial maxima (workspace), R > 1 only
    int M, K, R;
    int quant_parts;     // > 0: the quantize pass takes each block's maximum from this many partial maxima itself
    // percentile-clipped variant only (launch_daq_robust)
    int qmax;            // 2^(b-1) - 1 for b-bit activation codes
    unsigned top_rank;   // tau = the top_rank-th largest magnitude of a scale block (1 = the maximum)
    unsigned *hist;      // [M/R][DAQ_ROBUST_WORDS] selection scratch (workspace), R > 1 only
};
constexpr int DAQ_ROBUST_WORDS = 256 + 2 + 128;

// R > 1: the first pass cuts every scale block (R*K contiguous values) into this many parts and leaves one partial
// maximum per part; 0 when the shape takes the row kernels instead (no partials needed).
constexpr int DAQ_PART_PIECES = 2048;  // 16-byte pieces per part: 256 threads x 8 loads
inline size_t daq_parts_per_block(int64_t K, int64_t R)
{
    if (R <= 1 || K % 8 != 0) return 0;
    const size_t pieces = (size_t)R * (size_t)K / 8;
    if (pieces < (size_t)DAQ_PART_PIECES || pieces >= (1ull << 31)) return 0;
    return (pieces + DAQ_PART_PIECES - 1) / DAQ_PART_PIECES;
}

hipError_t launch_daq(const DaqArgs &a, hipStream_t stream);
// eq. (4) with channel groups: scales [M/R, K/cg], blockmax workspace of the same count; K % 8 == 0, cg % 8 == 0, K/cg <= 1024
hipError_t launch_daq_cg(const DaqArgs &a, int cg, hipStream_t stream);
// DAQ whose row maxima are already known (row_absmax [M], binary16 bit patterns): scales and the quantize pass only
hipError_t launch_daq_from_rowmax(const DaqArgs &a, const unsigned *row_absmax, hipStream_t stream);
hipError_t launch_fill_u32(unsigned *p, int n, unsigned v, hipStream_t stream);
// eq. (4) with tau = a percentile of the magnitudes and a selectable code width
hipError_t launch_daq_robust(const DaqArgs &a, hipStream_t stream);

// LayerNorm + modulation + per-token DAQ in one pass (daq_ln.hip); K % 8 == 0, K <= 4608, 16-byte aligned rows
struct LnDaqArgs {
    const void *x;       // [M,K] fp16
    const void *shift;   // [M/rows_per_mod, K] fp16 or null (0)
    const void *scale;   // [M/rows_per_mod, K] fp16 or null (0): h = n * (1 + scale) + shift
    void *h;             // [M,K] fp16 out, or null
    int8_t *q;           // [M,K] out, or null (then only h is produced)
    float *scales;       // [M] out
    int M, K, rows_per_mod;
    float eps;
};
hipError_t launch_daq_ln(const LnDaqArgs &a, hipStream_t stream);

// ---- GEMM + dequantization -------------------------------------------------
struct GemmArgs {
    const int8_t *q;      // [M,K] activation codes
    const float *s_a;     // [M/R]
    const void *w;        // int8 [N,K] or packed 4-bit [N,K/2]
    const void *s_w;      // fp32 [N] (W8) or fp16 [N,K/group] (W4)
    const void *bias;     // fp16 [N] or null
    void *y;              // fp16 [M,N]
    int32_t *acc_out;     // optional export: [M,N] (W8) or [M,K/group,N] (W4)
    int M, N, K, R;
    int w_bits;           // 8 or 4
    int group;            // 4-bit weights: k per weight scale (a multiple of 32 dividing K); 128 unless stated
    // block glue folded into the epilogue (all zero = none):  h = f16(act(u));  y = f16(fma(g, h, r))
    int act;              // 0 identity, 1 GELU (tanh form) on the fp32 value u
    const void *residual; // fp16 [M,N] r, or null (0)
    const void *gate;     // fp16 [M/gate_rows, N] g, or null (1)
    int gate_rows;        // rows sharing one gate row
    // plan-space generality (Step 2, Algorithm 1, eq. (4)'s channel groups); all zero = none
    int w_grouped;        // 1: w holds int8 codes [N,K] (W3, W6, W8 or asymmetric codes stored as code - zero) with fp16 scales
                          //    [N,K/group] like the 4-bit layers (w_bits stays 8)
    const float *s_ag;    // activation scales per (scale block, channel group) [M/R, K/group] instead of s_a; the channel
                          //    groups are the weight groups
    unsigned *row_absmax; // optional side output [M] (cleared by the caller of the launch): the largest |y[m,:]| as a binary16
                          //    bit pattern, taken on the fp16 values the layer writes (what the next layer's DAQ would find)
};

int num_gemm_variants();
const char *gemm_variant_name(int v);
// variant < 0: choose by shape
hipError_t launch_qgemm(const GemmArgs &a, int variant, hipStream_t stream);

// the pipelined 4-bit kernel (qgemm_w4.hip): shapes it takes, and its launch (group 128 or any 32 j, exports, glue)
bool qgemm_w4_takes(const GemmArgs &a);
hipError_t launch_qgemm_w4(const GemmArgs &a, hipStream_t stream);
// pair-order nibbles (device) -> the 4-bit storage order (device); blocks = N*K/8 four-byte blocks
hipError_t launch_prepack_w4(const void *pairs, void *packed, long long blocks, hipStream_t stream);

}  // namespace ql
