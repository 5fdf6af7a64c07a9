/*
 * diffpro_qlinear.h - C ABI of the MI355X (gfx950) quantized DiT linear layer
 * of DiffPro (arXiv 2511.11446): dynamic activation quantization (DAQ) ->
 * INT8 x INT8 -> INT32 GEMM -> dequantization + bias, and a runner that walks
 * a per-layer {4,8}-bit weight plan.
 *
 * General rules
 *   - Every pointer marked (device) is GPU memory owned by the caller; the
 *     library reads inputs, writes outputs, never frees or keeps them past the
 *     call (a plan keeps the weight/scale/bias pointers it was created with).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without synchronizing.  Calls on
 *     different streams may run concurrently if their buffers are disjoint.
 *   - No call allocates device memory.  Scratch comes from the caller through
 *     (workspace, workspace_bytes); the matching *_workspace_bytes() gives the
 *     size.  workspace must be 256-byte aligned.
 *   - Every call returns a ql_status.  All argument checks happen before the
 *     first HIP call, so they behave the same on a machine without a GPU.
 *   - Inputs are assumed finite; NaN/Inf activations give unspecified codes.
 *   - Matrices are row-major and dense (row pitch = number of columns).
 *   - Limits: 1 <= M, N, K; M*K, M*N and N*K below 2^31; K <= 133143
 *     (so that K * 127 * 127 fits an int32); M % R == 0.
 *     The fast (MFMA) kernels need K % 16 == 0 and 16-byte aligned x, q, w;
 *     other shapes or alignments are served by slower generic kernels with the
 *     same results.  4-bit weights need K % group == 0 (group = 128 unless the
 *     call takes one), K % 8 == 0 and group <= 132096 (the kernels multiply
 *     the nibbles as value * 16, and 127 * 8 * 16 * group must fit an int32).
 */
#ifndef DIFFPRO_QLINEAR_H
#define DIFFPRO_QLINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ql_status {
    QL_OK = 0,
    QL_ERR_NULL = 1,        /* a required pointer is NULL */
    QL_ERR_SHAPE = 2,       /* a size is out of the limits above */
    QL_ERR_ALIGN = 3,       /* workspace not 256-byte aligned, or a 2/4-byte typed pointer misaligned */
    QL_ERR_UNSUPPORTED = 4, /* w_bits not in {4,8}, group not 0 (8-bit) / not a multiple of 32 (4-bit), DAQ parameters out of range */
    QL_ERR_WORKSPACE = 5,   /* workspace missing or too small */
    QL_ERR_DEVICE = 6       /* a HIP call failed; see ql_last_device_error() */
} ql_status;

/* Human-readable name of a status code (static storage, host). */
const char *ql_status_string(int status);

/* The hipError_t of the most recent failed HIP call on this thread (0 if none). */
int ql_last_device_error(void);

/* Library version: major * 1000 + minor. */
int ql_version(void);

/* ------------------------------------------------------------------------
 * DAQ: Step 3, eq. (4) with tau = the absolute maximum of the scale block
 * (percentile p -> 100, i.e. the min/max scales taken per sample and timestep
 * that Section 2.3 describes), b = 8, zero-point 0.
 *   alpha_r = amax_r / 127            (1 if the block is all zero)
 *   q[m,k]  = clamp(round_half_even(x[m,k] / alpha_r), -127, 127)
 * A scale block r is R consecutive rows: R = 1 per token, R = tokens per image
 * per sample, R = M per tensor.
 *   x       (device) [M,K] fp16, in
 *   q       (device) [M,K] int8, out
 *   scales  (device) [M/R] fp32 alpha, out
 *   workspace: needed only when R > 1 (daq_workspace_bytes)
 * ---------------------------------------------------------------------- */
size_t daq_workspace_bytes(int64_t M, int64_t K, int64_t R);

int daq_quantize(const void *x, int64_t M, int64_t K, int64_t R,
                 void *q, void *scales,
                 void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * LayerNorm + adaptive modulation + DAQ in one pass (Step 3 keeps LayerNorm in
 * higher precision in front of the quantized qkv and fc1 layers; Section 6
 * counts it in the latency).  Per row, in fp32:
 *   mu = mean(x), var = mean((x - mu)^2), n = (x - mu) / sqrt(var + eps)
 *   h  = fp16( fma(n, 1 + scale[m / rows_per_mod, k], shift[m / rows_per_mod, k]) )
 * then daq_quantize(h) -> q, scales.  LayerNorm has no affine parameters; shift
 * and scale are the per-image modulation vectors of an adaptive-LayerNorm block
 * (either may be NULL: 0).
 *   x (device) [M,K] fp16;  shift, scale (device) [M/rows_per_mod, K] fp16 or NULL
 *   h (device) [M,K] fp16 out or NULL: the normalised, modulated rows
 *   q (device) [M,K] int8 out or NULL (then only h is written);  scales [M/R] fp32
 * R = 1 runs in a single pass with the row held in registers; R > 1 needs h
 * (the rows are staged there) and the workspace of daq_quantize.  Needs
 * K % 8 == 0, K <= 4608 and 16-byte aligned x, shift, scale, h (QL_ERR_SHAPE /
 * QL_ERR_ALIGN otherwise).
 * ---------------------------------------------------------------------- */
int daq_quantize_ln(const void *x, int64_t M, int64_t K, int64_t R,
                    const void *shift, const void *scale, int64_t rows_per_mod, float eps,
                    void *h, void *q, void *scales,
                    void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Optional exports of the integer intermediates, for verification.  Any
 * member may be NULL; the struct pointer itself may be NULL.  They are written
 * by the same kernels that produce y.
 *   q         (device) [M,K] int8 activation codes
 *   a_scales  (device) [M/R] fp32 activation scales alpha
 *   acc       (device) int32: [M,N] accumulators for 8-bit weights;
 *             [M, K/128, N] per-group partial sums for 4-bit weights
 * ---------------------------------------------------------------------- */
typedef struct ql_debug {
    void *q;
    void *a_scales;
    void *acc;
} ql_debug;

/* Scratch for one quantized linear on M rows of K inputs (codes + scales + block maxima). */
size_t qlinear_workspace_bytes(int64_t M, int64_t K, int64_t R);

/* ------------------------------------------------------------------------
 * Quantized linear with 8-bit weights (Step 3 and Step 5: all linears run as
 * int8 x int8 products accumulated in int32, one weight scale per output channel;
 * Section 6 counts DAQ, requantization and dequantization in the latency):
 *   q, alpha = DAQ(x, R)
 *   acc[m,n] = sum_k q[m,k] * w[n,k]                       (int32)
 *   t        = float(acc) * alpha[m/R]                      (fp32)
 *   y[m,n]   = fp16( fma(t, w_scale[n], bias[n]) )          (t * w_scale[n] without a bias)
 * one fp32 rounding per operation, then round-to-nearest-even into fp16.
 *   x        (device) [M,K] fp16
 *   w        (device) [N,K] int8 codes in [-127,127], K contiguous
 *   w_scale  (device) [N] fp32
 *   bias     (device) [N] fp16, or NULL
 *   y        (device) [M,N] fp16, out
 * ---------------------------------------------------------------------- */
int qlinear_w8a8(const void *x, int64_t M, int64_t K, int64_t R,
                 const void *w, const void *w_scale, const void *bias, int64_t N,
                 void *y, const ql_debug *dbg,
                 void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * qlinear_w8a8 for callers that cannot allocate or hand over device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arithmetic, same results and same argument meaning as
 * qlinear_w8a8 without the debug exports; the scratch (codes, activation scales,
 * partial maxima) is a fixed array inside the library, qlinear_noalloc_max_bytes()
 * = 24 MiB per GPU, held by every GPU the library runs on until the process ends.
 *   - The call allocates nothing (no hipMalloc / hipFree, no allocating library
 *     routine); the first call on a device looks the array's address up once.
 *   - QL_ERR_WORKSPACE if qlinear_workspace_bytes(M, K, R) exceeds the array
 *     (M*K up to about 25 million, e.g. 16384 x 1152); the other errors as
 *     qlinear_w8a8.
 *   - All calls on one GPU share the array, which keeps the last call's contents
 *     (nothing in it needs clearing between calls): calls that overlap in time on
 *     one GPU, on any streams, race.  Calls in order on one stream are safe.
 * ---------------------------------------------------------------------- */
size_t qlinear_noalloc_max_bytes(void);
int qlinear_w8a8_noalloc(const void *x, int64_t M, int64_t K, int64_t R,
                         const void *w, const void *w_scale, const void *bias, int64_t N,
                         void *y, void *stream);

/* ------------------------------------------------------------------------
 * Quantized linear with 4-bit group-128 weights (Step 2: integer weights with
 * per-group scales; symmetric, zero-point 0, as in the ablation section):
 *   P[m,g,n] = sum_{k in group g} q[m,k] * w4[n,k]          (int32, g = k/128)
 *   f        = fma(float(P[m,g,n]), w_scale[n,g], f)        (fp32, g ascending, f starts at 0)
 *   y[m,n]   = fp16( fma(f, alpha[m/R], bias[n]) )          (f * alpha[m/R] without a bias)
 *   w4       (device) [N, K/2] bytes, two's-complement nibbles in [-8,7].
 *            Storage order: inside every run of 8 consecutive k (4 bytes),
 *            byte j (0..3) holds k = 8b+j in its low nibble and k = 8b+4+j in
 *            its high nibble.  ql_pack_w4_host() produces it.
 *   w_scale  (device) [N, K/128] fp16
 * ---------------------------------------------------------------------- */
int qlinear_w4a8(const void *x, int64_t M, int64_t K, int64_t R,
                 const void *w4, const void *w_scale, const void *bias, int64_t N,
                 void *y, const ql_debug *dbg,
                 void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * The GEMM + dequantization stage alone, on codes a previous daq_quantize()
 * produced (used to time the two stages separately).  Same formulas as above.
 *   q         (device) [M,K] int8
 *   a_scales  (device) [M/R] fp32
 *   acc       (device) optional int32 export as in ql_debug, or NULL
 * ---------------------------------------------------------------------- */
int qgemm_w8a8(const void *q, const void *a_scales, int64_t M, int64_t K, int64_t R,
               const void *w, const void *w_scale, const void *bias, int64_t N,
               void *y, void *acc, void *stream);

int qgemm_w4a8(const void *q, const void *a_scales, int64_t M, int64_t K, int64_t R,
               const void *w4, const void *w_scale, const void *bias, int64_t N,
               void *y, void *acc, void *stream);

/* The 4-bit layer with weight groups of `group` consecutive k per scale instead
 * of 128 (Step 2 and Algorithm 1 choose the group size per layer; the final plan
 * of Step 2 uses 32, 64, 128, 192 and 288).  group: a multiple of 32
 * (else QL_ERR_UNSUPPORTED) that divides K (else QL_ERR_SHAPE).
 *   w_scale (device) fp16 [N, K/group];  dbg->acc, acc: int32 [M, K/group, N]
 *   f = sum over groups g ascending of fma(float(P[m,g,n]), w_scale[n,g], f)
 * Everything else as qlinear_w4a8 / qgemm_w4a8 (group = 128 gives their result). */
int qlinear_w4a8_g(const void *x, int64_t M, int64_t K, int64_t R,
                   const void *w4, const void *w_scale, int64_t group, const void *bias, int64_t N,
                   void *y, const ql_debug *dbg,
                   void *workspace, size_t workspace_bytes, void *stream);
int qgemm_w4a8_g(const void *q, const void *a_scales, int64_t M, int64_t K, int64_t R,
                 const void *w4, const void *w_scale, int64_t group, const void *bias, int64_t N,
                 void *y, void *acc, void *stream);

/* ------------------------------------------------------------------------
 * The rest of the plan space (Step 2 and Algorithm 1: W3/W4/W6/W8 with group
 * scales and zero points; Step 3, eq. (4): activation scales per sample,
 * timestep AND channel group).
 *
 * daq_quantize_cg: eq. (4) with tau = the absolute maximum of each sub-block of
 * R rows (a sample's tokens) x act_group consecutive channels:
 *   alpha[r, c] = amax / 127 (1 if zero),  q = clamp(rne(x / alpha[m/R, k/act_group]), -127, 127)
 *   scales (device) [M/R, K/act_group] fp32.  act_group: a multiple of 8 that
 *   divides K, K/act_group <= 1024 (QL_ERR_UNSUPPORTED / QL_ERR_SHAPE); x 16-byte
 *   aligned; workspace daq_cg_workspace_bytes().
 *
 * qlinear_grouped: the layer with group-wise weight scales for any width:
 *   w_storage = 4: w is packed 4-bit [N,K/2] as in qlinear_w4a8
 *   w_storage = 8: w is int8 [N,K] holding codes of ANY width up to 8 bits:
 *                  W3 in [-4,3], W6 in [-32,31] (ql_unpack_bits_host expands their
 *                  dense storage), W8 in [-127,127], or codes with a zero point
 *                  stored as code - zero (ql_zero_point_fold_host; widths <= 7)
 *   P[m,g,n] = sum_{k in group g} q[m,k] * w[n,k]
 *   act_group = 0:      q, alpha = daq_quantize(x, R);
 *                       f = fma(float(P), w_scale[n,g], f);  y = fp16(fma(f, alpha[m/R], bias[n]))
 *   act_group = group:  q, alpha = daq_quantize_cg(x, R, group);  c = w_scale[n,g] * alpha[m/R, g] (fp32)
 *                       f = fma(float(P), c, f);  y = fp16(f + bias[n])
 *   (other act_group values: QL_ERR_UNSUPPORTED.)  w_scale fp16 [N,K/group];
 *   dbg->a_scales is [M/R] or [M/R, K/group]; dbg->acc [M, K/group, N].
 * The pipelined kernel takes K % 128 == 0, K/group <= 40 (4-bit storage: <= 144)
 * and, with channel-group activation scales, R % 128 == 0; other shapes run on
 * the generic kernel.
 * Workspace: qlinear_grouped_workspace_bytes().
 *
 * Host helpers: ql_pack_bits_host / ql_unpack_bits_host store b-bit two's-
 * complement codes (2 <= b <= 7) densely, a row's codes concatenated LSB first
 * (K * b must be a multiple of 8); ql_zero_point_fold_host turns codes and
 * per-group zero points (both as ql_gptq_quantize_host returns them) into
 * int8 differences code - zero (QL_ERR_UNSUPPORTED if one does not fit int8).
 * ---------------------------------------------------------------------- */
size_t daq_cg_workspace_bytes(int64_t M, int64_t K, int64_t R, int64_t act_group);
int daq_quantize_cg(const void *x, int64_t M, int64_t K, int64_t R, int64_t act_group,
                    void *q, void *scales, void *workspace, size_t workspace_bytes, void *stream);
size_t qlinear_grouped_workspace_bytes(int64_t M, int64_t K, int64_t R, int64_t act_group);
int qlinear_grouped(const void *x, int64_t M, int64_t K, int64_t R, int64_t act_group,
                    const void *w, int32_t w_storage, const void *w_scale, int64_t group,
                    const void *bias, int64_t N, void *y, const ql_debug *dbg,
                    void *workspace, size_t workspace_bytes, void *stream);
int ql_pack_bits_host(const int8_t *codes, int64_t N, int64_t K, int32_t bits, uint8_t *packed);
int ql_unpack_bits_host(const uint8_t *packed, int64_t N, int64_t K, int32_t bits, int8_t *codes);
int ql_zero_point_fold_host(const int8_t *codes, const int32_t *zeros, int64_t N, int64_t K, int64_t group, int8_t *out);

/* ------------------------------------------------------------------------
 * Block glue folded into the layer's epilogue (Section 6 counts the residual
 * additions in the latency; Step 3 keeps them in higher precision; the MLP's
 * activation sits between its two quantized linears).  With u the layer's
 * fp32 value before its rounding to fp16 (formulas above):
 *   h = fp16( act(u) )                  act: QL_ACT_NONE, or QL_ACT_GELU_TANH
 *                                       gelu(u) = u * sigmoid(2z), z = sqrt(2/pi) (u + 0.044715 u^3)
 *   y = h                               without gate and residual
 *   y = fp16( fma(g, float(h), r) )     g = gate[m / gate_rows, n] (1 if gate is NULL),
 *                                       r = residual[m, n]         (0 if residual is NULL)
 * i.e. the result of the unfused sequence layer -> fp16 -> gated residual add.
 *   residual  (device) [M,N] fp16 or NULL;  gate (device) [M/gate_rows, N] fp16 or NULL
 *   gate_rows: rows sharing one gate row (tokens per image); M % gate_rows == 0
 *   row_absmax (device) [M] uint32 or NULL: side output for the DAQ of the layer
 *              that consumes y (the MLP's second linear after the first one's
 *              GELU): entry m receives max_n |y[m,n]| as a binary16 bit pattern
 *              (for non-negative binary16 numbers the integer order of the
 *              patterns is the numeric order), taken on the fp16 values written
 *              to y.  The call clears it first.  daq_quantize_rowmax consumes it.
 * The GELU is evaluated in fp32 on the GPU (relative error about 1e-6 before the
 * fp16 rounding).  fusion == NULL or all-zero gives the plain layer.  group: as in
 * qlinear_w4a8_g.  Errors: QL_ERR_UNSUPPORTED for an unknown act, QL_ERR_SHAPE for
 * a bad gate_rows, QL_ERR_ALIGN for odd pointers; the rest as the plain calls.
 * ---------------------------------------------------------------------- */
enum { QL_ACT_NONE = 0, QL_ACT_GELU_TANH = 1 };

typedef struct ql_fusion {
    int32_t act;
    int32_t reserved;      /* 0 */
    const void *residual;
    const void *gate;
    int64_t gate_rows;
    void *row_absmax;      /* side output or NULL, see above */
} ql_fusion;

int qlinear_w8a8_fused(const void *x, int64_t M, int64_t K, int64_t R,
                       const void *w, const void *w_scale, const void *bias, int64_t N,
                       const ql_fusion *fusion, void *y,
                       void *workspace, size_t workspace_bytes, void *stream);
int qlinear_w4a8_fused(const void *x, int64_t M, int64_t K, int64_t R,
                       const void *w4, const void *w_scale, int64_t group, const void *bias, int64_t N,
                       const ql_fusion *fusion, void *y,
                       void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * A layer the plan leaves in FP16 (Step 2 freezes the most sensitive layers;
 * its final plan keeps 22 of 113 layers in FP16): no quantization,
 *   y[m,n] = fp16( sum_k x[m,k] * w[n,k] + bias[n] )
 * with fp32 accumulation on the matrix cores (the sum's rounding error is
 * bounded by K * 2^-24 * sum_k |x w|; the oracle sums in fp64).
 *   x (device) [M,K] fp16;  w (device) [N,K] fp16;  bias (device) [N] fp16 or NULL
 *   fusion: as in the *_fused calls, or NULL.  No workspace.
 * In a plan such a layer has w_bits = 16, group = 0 and w_scale = NULL.
 * ---------------------------------------------------------------------- */
int qlinear_f16(const void *x, int64_t M, int64_t K,
                const void *w, const void *bias, int64_t N,
                const ql_fusion *fusion, void *y, void *stream);

/* Host helper: pack int8 codes in [-8,7], [N,K] row-major (host), into the
 * 4-bit storage order described at qlinear_w4a8 ([N,K/2] bytes, host).
 * K % 8 == 0.  Returns QL_ERR_SHAPE for a code outside [-8,7]. */
int ql_pack_w4_host(const int8_t *codes, int64_t N, int64_t K, uint8_t *packed);

/* Host helper for weights that already sit two per byte in the common pair order
 * (byte i of a row holds k = 2i in its low nibble and k = 2i+1 in its high nibble,
 * two's-complement nibbles): rewrites them, [N,K/2] bytes (host) to [N,K/2] bytes
 * (host), into the storage order qlinear_w4a8 reads.  K % 8 == 0; in place is not
 * supported (QL_ERR_UNSUPPORTED). */
int ql_repack_w4_pairs_host(const uint8_t *pairs, int64_t N, int64_t K, uint8_t *packed);

/* The same re-layout on the device, for weights that arrive in the common pair
 * order (Step 2 packs the weights offline, once): pairs (device) [N,K/2] bytes,
 * byte i of a row = k = 2i (low nibble) and k = 2i+1 (high nibble); packed
 * (device) [N,K/2] bytes in the storage order qlinear_w4a8 reads.  Both buffers
 * are the caller's, 4-byte aligned, and must not overlap (the same pointer is
 * QL_ERR_UNSUPPORTED).  K % 8 == 0.  Asynchronous on `stream`. */
int ql_prepack_w4(const void *pairs, int64_t N, int64_t K, void *packed, void *stream);

/* ------------------------------------------------------------------------
 * Plan runner: Algorithm 2, Phase B (every layer wrapped as its plan entry says,
 * then the forward pass on quantized weights and activations) and Step 6,
 * restricted to the quantized linears.  A plan is a list of layers, each with its own weight
 * width; qlinear_plan_run enqueues DAQ + GEMM + epilogue for every layer in
 * order on one stream.
 * ---------------------------------------------------------------------- */
typedef struct ql_layer_desc {
    int64_t K;            /* input features */
    int64_t N;            /* output features */
    int32_t w_bits;       /* 8 or 4; 16 = the layer stays in FP16 (w fp16 [N,K], w_scale NULL, group 0) */
    int32_t group;        /* 0 = one scale per output channel (8-bit); 4-bit: k per scale, a multiple of 32 dividing K */
    const void *w;        /* (device) int8 [N,K] or packed 4-bit [N,K/2] */
    const void *w_scale;  /* (device) fp32 [N] (8-bit) or fp16 [N,K/group] (4-bit) */
    const void *bias;     /* (device) fp16 [N] or NULL */
} ql_layer_desc;

typedef struct ql_plan ql_plan; /* opaque, host object owned by the library */

/* Validates and copies the descriptors (host memory only; no device call).
 * M_max bounds the rows of later runs. */
int ql_plan_create(const ql_layer_desc *layers, int32_t n_layers, int64_t M_max, ql_plan **plan_out);
void ql_plan_destroy(ql_plan *plan);
int32_t ql_plan_num_layers(const ql_plan *plan);

/* Scratch for a run on M rows (sized for the widest layer input). */
size_t ql_plan_workspace_bytes(const ql_plan *plan, int64_t M, int64_t R);

/* x_in[l] (device) [M, K_l] fp16 and y_out[l] (device) [M, N_l] fp16 for every
 * layer l; the two pointer arrays themselves are host memory.  Layers run in
 * order on `stream`, so y_out[l] may alias x_in[l+1]. */
int qlinear_plan_run(const ql_plan *plan, const void *const *x_in, void *const *y_out,
                     int64_t M, int64_t R,
                     void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Percentile-clipped DAQ with a selectable activation width: eq. (4) as
 * printed (Step 3), b set per time bin (Step 6, Algorithm 2 Phase B).
 *   tau   = Percentile(|v|, p) over each scale block of R rows, nearest rank:
 *           the k-th smallest magnitude, k = ceil(n * p_ppm / 10^6), n = R*K
 *   alpha = tau / (2^(a_bits-1) - 1)      (1 if tau = 0)
 *   code  = round_half_even(clip(v, -tau, tau) / alpha), stored as int8
 * p_ppm in [1, 10^6] (999000 = the paper's p = 99.9), a_bits in [2, 8], else
 * QL_ERR_UNSUPPORTED; {1000000, 8} gives daq_quantize()'s result.  All other
 * arguments, the workspace (daq_workspace_bytes / ql_plan_workspace_bytes)
 * and the error behaviour are those of daq_quantize / qlinear_plan_run.
 * params: host memory, read during the call.
 * ---------------------------------------------------------------------- */
typedef struct ql_daq_params {
    int32_t p_ppm;
    int32_t a_bits;
} ql_daq_params;

/* DAQ (Step 3, eq. (4), absolute maximum, 8 bits) of a tensor whose row maxima are
 * already known: row_absmax (device) [M] uint32, entry m = max_k |x[m,k]| as a
 * binary16 bit pattern, as the row_absmax side output of the layer that wrote x
 * leaves it.  The pass over x that finds the maxima is skipped: scales come from
 * the R row maxima of each scale block and x is read once, by the quantize pass.
 * Results are those of daq_quantize when row_absmax is right (not checked).
 * Arguments, workspace (daq_workspace_bytes) and errors as daq_quantize. */
int daq_quantize_rowmax(const void *x, int64_t M, int64_t K, int64_t R, const void *row_absmax,
                        void *q, void *scales, void *workspace, size_t workspace_bytes, void *stream);

int daq_quantize_robust(const void *x, int64_t M, int64_t K, int64_t R, const ql_daq_params *params,
                        void *q, void *scales, void *workspace, size_t workspace_bytes, void *stream);

int qlinear_plan_run_robust(const ql_plan *plan, const void *const *x_in, void *const *y_out,
                            int64_t M, int64_t R, const ql_daq_params *params,
                            void *workspace, size_t workspace_bytes, void *stream);

/* The plan walk with everything optional switched per call (Algorithm 2 Phase B, the quantized forward pass of one step of the schedule): params as in qlinear_plan_run_robust or NULL (absolute maximum, 8 bits;
 * FP16 layers ignore it), fusion = NULL or a host array of n_layers pointers, entry l NULL or the glue folded into
 * layer l's epilogue (see ql_fusion).  Everything else as qlinear_plan_run. */
int qlinear_plan_run_ex(const ql_plan *plan, const void *const *x_in, void *const *y_out,
                        int64_t M, int64_t R, const ql_daq_params *params, const ql_fusion *const *fusion,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Host helper for the time-bin policy of Step 6: bin of step `step` (0-based, in
 * sampling order) out of num_steps, equal thirds: 0 early, 1 mid, 2 late;
 * -1 for arguments out of range.  The caller maps the bin to a_bits. */
int ql_time_bin(int64_t step, int64_t num_steps);

/* ------------------------------------------------------------------------
 * Offline side, host memory only (no device call): the stages that produce what
 * the calls above consume.
 *
 * ql_schedule_topk: Step 4, eq. (6).  With T_tail = { t in C : t/T >= 1 - rho }
 * the kept schedule is T_tail united with the k - |T_tail| steps of C \ T_tail
 * that have the largest student-teacher error delta(t) of eq. (5) (equal delta:
 * the earlier step first).  delta: [T] doubles indexed by timestep; candidates:
 * n_candidates timesteps in [0, T) (duplicates ignored); rho in parts per
 * million (200000 = the paper's 0.2; the tail test is done in integers);
 * kept_out: k timesteps, ascending.  QL_ERR_SHAPE if k is below |T_tail| or
 * above |C|, or a candidate lies outside [0, T).
 *
 * ql_plan_greedy: Algorithm 2, Phase A.  Starts from every layer at its widest
 * option and all T steps kept, protects the last floor(rho T) steps, and while a
 * budget is exceeded takes the better of: pruning the prunable step of lowest
 * drift, scored c_step / (eps + D_e); or the best next-narrower move of a layer,
 * scored (c_lat(l,b) - c_lat(l,b')) / (eps + s_M(l)).  Costs are the caller's
 * numbers (for example per-layer latencies measured with this library):
 * C_lat = sum of c_step over kept steps + sum of c_lat(l, Pi(l)),
 * C_mem = sum of c_mem(l, Pi(l)).  While only the memory budget is exceeded no
 * step is pruned (a step frees no memory); when nothing is left to take the
 * plan is returned with *feasible_out = 0.  Outputs: bits_out[L] the chosen
 * width per layer, kept_out[T] 1/0 per step, the two totals.
 *
 * ql_gptq_quantize_host: Step 2, the GPTQ packer.  W [N,K] fp32 row-major, H
 * [K,K] doubles = the layer's X^T X over calibration inputs.  Inputs with
 * H_kk = 0 are dropped, damp * mean(diag H) is added to the diagonal, U = the
 * upper Cholesky factor of H^-1; columns are quantized in order, each group's
 * scale (and zero point) taken per row from the already compensated weights at
 * the group's first column, and each column's rounding error e = (w - w_hat) /
 * U_kk is subtracted as e * U_kj from the columns j > k.  symmetric: codes in
 * [-127,127] (8 bits) or [-2^(b-1), 2^(b-1)-1], zero point 0; otherwise codes
 * 0 .. 2^b - 1 with a zero point, both stored minus 2^(b-1) so that codes fit
 * int8 and (code - zero) is unchanged.  scale_fp16 != 0 rounds every scale to
 * binary16 before it is used (what the 4-bit kernels read).  codes [N,K] int8,
 * scales [N,K/group] fp32, zeros [N,K/group] int32 (may be NULL when symmetric).
 * The int8 codes of a symmetric 4-bit run go to ql_pack_w4_host.
 * QL_ERR_UNSUPPORTED: bits outside 2..8, or H not positive definite after damping.
 * ---------------------------------------------------------------------- */
int ql_schedule_topk(const double *delta, const int32_t *candidates, int32_t n_candidates, int32_t T,
                     int32_t rho_ppm, int32_t k, int32_t *kept_out);

typedef struct ql_planner_layer {
    int32_t n_options;     /* widths the layer may take */
    int32_t reserved;      /* 0 */
    const int32_t *bits;   /* [n_options] distinct widths, any order */
    const double *c_lat;   /* [n_options] latency cost at each width */
    const double *c_mem;   /* [n_options] memory cost at each width */
    double sensitivity;    /* s_M(l) */
} ql_planner_layer;

int ql_plan_greedy(const double *drift, const double *c_step, int32_t T,
                   const ql_planner_layer *layers, int32_t L,
                   double B_lat, double B_mem, int32_t rho_ppm, double eps,
                   int32_t *bits_out, uint8_t *kept_out,
                   double *C_lat_out, double *C_mem_out, int32_t *feasible_out);

int ql_gptq_quantize_host(const float *W, int64_t N, int64_t K, const double *H,
                          int32_t bits, int64_t group, int32_t symmetric, double damp, int32_t scale_fp16,
                          int8_t *codes, float *scales, int32_t *zeros);

/* ------------------------------------------------------------------------
 * Tuning hooks (benchmark sweeps).  ql_set_gemm_variant(v) forces GEMM tile
 * variant v for later calls from this process (-1 = choose by shape;
 * v == ql_num_gemm_variants() = the generic one-thread-per-element kernel);
 * ql_num_gemm_variants() gives the number of tiled variants;
 * ql_gemm_variant_name(v) a short description.  A forced variant that cannot
 * take a shape (K not a multiple of its K step, misaligned operands) falls
 * back to the generic kernel.  Results do not depend on the variant.
 * ---------------------------------------------------------------------- */
int ql_set_gemm_variant(int variant);
int ql_num_gemm_variants(void);
const char *ql_gemm_variant_name(int variant);

#ifdef __cplusplus
}
#endif
#endif /* DIFFPRO_QLINEAR_H */
