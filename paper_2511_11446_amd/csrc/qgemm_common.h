// Device helpers shared by the GEMM kernels (qgemm.hip, qgemm_w4.hip): vector types, the block glue folded into the
// epilogue, and the packed write-back of a dequantized tile.  Not part of the public ABI.
#pragma once
#include "ql_internal.h"

#include <type_traits>

namespace ql {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
// LDS staging is written as fp16 scalars and read back as 16-byte vectors: tell the compiler these may alias
typedef _Float16 half_alias __attribute__((may_alias));
typedef int v4i_alias __attribute__((ext_vector_type(4), may_alias));
typedef float v4f __attribute__((ext_vector_type(4)));

// Timing hook for kernel phase studies; expands to nothing in the library build.
#ifndef QL_PHASE
#define QL_PHASE(id)
#endif

constexpr int XCDS = 8;    // L2 domains of the chip; consecutive workgroup ids go round-robin over them
constexpr int GROUP_ROWS = 1024; // rows of A walked together so that one L2 sees few distinct A and W panels (512..2048 measure alike)

static int pick_group_m(int bm) { return GROUP_ROWS / bm > 0 ? GROUP_ROWS / bm : 1; }

__device__ __forceinline__ float half_to_float_dev(unsigned short h)
{
    return (float)__builtin_bit_cast(_Float16, h);
}

// ---- block glue folded into the epilogue: h = f16(act(u)); y = f16(fma(g, h, r)) -----------------------------------
// GELU in its tanh form, written with the logistic function: u * sigmoid(2 z), z = sqrt(2/pi) (u + 0.044715 u^3).
// This keeps the relative accuracy in the negative tail, where 1 + tanh z cancels.
// exp(-2z) = 2^(u (k0 + k1 u^2)) with k0 = -2 sqrt(2/pi) log2(e), k1 = 0.044715 k0: five plain operations and two
// transcendental ones per element (the epilogue's ALU work is not hidden behind the MFMAs).
__device__ __forceinline__ float gelu_tanh_dev(float u)
{
    const float k0 = -2.302208198f, k1 = -0.1029432396f;
    const float e = u * __builtin_fmaf(k1, u * u, k0);
    return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(e));
}

__device__ __forceinline__ bool has_glue(const GemmArgs &a) { return a.act != 0 || a.residual != nullptr || a.gate != nullptr || a.row_absmax != nullptr; }

// Gate row of tile row d (0 <= d < span) without a division per element: the tile starts at row m_first, whose gate
// row and remainder are computed once; rows of a tile cross at most one gate boundary when gate_rows >= span.
struct GateRows {
    int base, rem, rows;
    bool one_step;
    __device__ __forceinline__ GateRows(const void *gate, int gate_rows, int m_first, int span)
    {
        rows = gate ? gate_rows : 1;
        base = m_first / rows;
        rem = m_first - base * rows;
        one_step = rows >= span;
    }
    __device__ __forceinline__ int of(int d) const { return one_step ? base + (rem + d >= rows ? 1 : 0) : base + (rem + d) / rows; }
};

// one element: u is the layer's fp32 value, grow its gate row
__device__ __forceinline__ _Float16 glue_one(const GemmArgs &a, float u, int m, int n, int grow)
{
    if (a.act == 1) u = gelu_tanh_dev(u);
    asm volatile("" : "+v"(u));   // keep the fp32 value: it is rounded to fp16 here and nowhere earlier
    _Float16 h = (_Float16)u;
    if (a.residual || a.gate) {
        const float g = a.gate ? half_to_float_dev(static_cast<const unsigned short *>(a.gate)[(unsigned)(grow * a.N + n)]) : 1.0f;
        const float r = a.residual ? half_to_float_dev(static_cast<const unsigned short *>(a.residual)[(unsigned)(m * a.N + n)]) : 0.0f;
        float v = __builtin_fmaf(g, (float)h, r);
        asm volatile("" : "+v"(v));
        h = (_Float16)v;
    }
    // side output for the next layer's DAQ: the row's largest |y| as a binary16 bit pattern (integer order = numeric order)
    if (a.row_absmax) atomicMax(a.row_absmax + m, (unsigned)(__builtin_bit_cast(unsigned short, h) & 0x7fffu));
    return h;
}

// what the staged write-back needs of the glue, by value (a pointer to the kernel arguments would force them into
// scratch memory)
struct GluePieces {
    const _Float16 *gate = nullptr, *residual = nullptr;
    int gate_rows = 1;
    bool on = false;
    unsigned *rowmax = nullptr;   // side output: largest |y| of every row (binary16 bit patterns), or nullptr
};

// eight neighbouring elements of one row at once (16-byte pieces of the staged tile); g and r were loaded ahead
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ v4i glue_piece(bool has_g, bool has_r, v4i hv, h8 g, h8 r)
{
    h8 h = __builtin_bit_cast(h8, hv);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float v = __builtin_fmaf(has_g ? (float)g[e] : 1.0f, (float)h[e], has_r ? (float)r[e] : 0.0f);
        asm volatile("" : "+v"(v));
        h[e] = (_Float16)v;
    }
    return __builtin_bit_cast(v4i, h);
}

// ---------------------------------------------------------------------------------------------
// Epilogue for a full tile (no ragged edge, N % 8 == 0).  Each wavefront dequantizes one 32-row
// block of its accumulators at a time, parks the fp16 results in a private LDS strip
// [32 rows][TN*32 columns] (row pitch padded by 16 bytes), and reads the strip back as 16-byte
// pieces, so that every global store instruction writes whole contiguous row segments of
// TN*64 bytes instead of 2-byte elements.
//   value(i, j, r) -> fp32 result before the fp16 rounding (W8: fma(float(acc)*s_a, s_w, bias))
// ---------------------------------------------------------------------------------------------
// The MFMA result layout gives a lane ONE column (lane & 31) and 16 rows.  Two neighbouring lanes swap
// one value per pair of consecutive rows (DPP quad_perm), so that the even lane ends up with columns
// (n, n+1) of the even row and the odd lane with columns (n-1, n) of the odd row: every element then
// leaves the lane as half of a 4-byte word instead of a 2-byte store.
//   STAGED: the words go to the LDS strip and are read back as 16-byte pieces (whole row segments per store);
//   otherwise they are stored to global memory directly (64-byte row segments per half wavefront).
template <int TM, int TN, bool STAGED, int ROWS = 32, class ValueFn>
__device__ __forceinline__ void store_tile_staged(unsigned char *strip, int lane, _Float16 *y, int N, int m_base, int n_base,
                                                  ValueFn value, GluePieces glue = GluePieces())
{
    constexpr int PITCH = TN * 64 + 16;
    constexpr int CH = TN * 4;  // 16-byte pieces per row
    const int frag_row = lane & 31, frag_half = lane >> 5, odd = lane & 1;
    // v_perm_b32 selector: bytes of {hi source = neighbour's pair, lo source = own pair}
    //   even lane: (own.lo16, nbr.lo16) -> bytes 0,1 of own then 0,1 of neighbour = 0x05040100
    //   odd lane:  (nbr.hi16, own.hi16) -> bytes 2,3 of neighbour then 2,3 of own = 0x03020706
    const unsigned sel = odd ? 0x03020706u : 0x05040100u;
    unsigned char *wr = strip + (4 * frag_half + odd) * PITCH + (frag_row - odd) * 2;
    const unsigned g_off = (unsigned)((m_base + 4 * frag_half + odd) * N + n_base + frag_row - odd);
    static_assert(ROWS == 32 || ROWS == 16, "the strip holds a whole 32-row block or one half of it");
    constexpr int HALVES = 32 / ROWS;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int h = 0; h < HALVES; ++h) {
            // gate and residual of the pieces this lane will write back are requested before the block is dequantized
            constexpr int PIECES = ROWS * CH / 64;
            h8 pg[PIECES], pr[PIECES];
            if (glue.on) {
                const GateRows gr(glue.gate, glue.gate_rows, m_base, TM * 32);
#pragma unroll
                for (int t = 0; t < PIECES; ++t) {
                    const int id = lane + 64 * t;
                    const int row = i * 32 + h * ROWS + id / CH, col = n_base + (id % CH) * 8;
                    if (glue.gate) pg[t] = *reinterpret_cast<const h8 *>(glue.gate + (unsigned)(gr.of(row) * N + col));
                    if (glue.residual) pr[t] = *reinterpret_cast<const h8 *>(glue.residual + (unsigned)((m_base + row) * N + col));
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = h * (16 / HALVES); r < (h + 1) * (16 / HALVES); r += 2) {
                    float u0 = value(i, j, r), u1 = value(i, j, r + 1);
                    // keep the fp32 rounding of the fused multiply-add: without this the compiler may select a
                    // mixed-precision fma that rounds straight to fp16 (one rounding instead of the defined two)
                    asm volatile("" : "+v"(u0), "+v"(u1));
                    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                    const h2 pr = {(_Float16)u0, (_Float16)u1};
                    const unsigned own = __builtin_bit_cast(unsigned, pr);
                    // every lane has a valid source, so no fill value is needed (the update form would first clear the destination)
                    const unsigned nbr = (unsigned)__builtin_amdgcn_mov_dpp((int)own, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
                    const unsigned word = __builtin_amdgcn_perm(nbr, own, sel);
                    const int row = 8 * (r / 4) + (r % 4);  // + 4*frag_half + odd, already in the lane's base
                    if (STAGED)
                        *reinterpret_cast<unsigned __attribute__((may_alias)) *>(wr + (row - h * ROWS) * PITCH + j * 64) = word;
                    else
                        *reinterpret_cast<unsigned __attribute__((may_alias)) *>(y + (g_off + (unsigned)((i * 32 + row) * N + j * 32))) = word;
                }
            if (STAGED) {
                // row maxima of the block: collected in the 4 spare bytes after every strip row (LDS operations of one
                // wavefront complete in program order), then one global atomic per row
                typedef __attribute__((address_space(3))) unsigned lds_u32;
                if (glue.rowmax && lane < ROWS) *reinterpret_cast<unsigned __attribute__((may_alias)) *>(strip + lane * PITCH + TN * 64) = 0u;
                asm volatile("" ::: "memory");  // the strip reads below see other lanes' writes: keep program order
#pragma unroll
                for (int t = 0; t < ROWS * CH / 64; ++t) {
                    const int id = lane + 64 * t;
                    const int row = id / CH, ch = id % CH;
                    v4i v = *reinterpret_cast<const v4i_alias *>(strip + row * PITCH + ch * 16);
                    // gate and residual meet the fp16 result here, eight elements of a row at a time
                    if (glue.on) v = glue_piece(glue.gate != nullptr, glue.residual != nullptr, v, pg[t], pr[t]);
                    if (glue.rowmax) {
                        // packed 16-bit maxima of the magnitudes' bit patterns, then the larger half
                        typedef unsigned short us2 __attribute__((ext_vector_type(2)));
                        us2 pm = __builtin_bit_cast(us2, (unsigned)v[0] & 0x7fff7fffu);
#pragma unroll
                        for (int w = 1; w < 4; ++w) pm = __builtin_elementwise_max(pm, __builtin_bit_cast(us2, (unsigned)v[w] & 0x7fff7fffu));
                        const unsigned mx = pm[0] > pm[1] ? pm[0] : pm[1];
                        __hip_atomic_fetch_max((lds_u32 *)(strip + row * PITCH + TN * 64), mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    }
                    // the output is written once and not read again by this kernel: keep it from displacing the operand panels in L2
                    __builtin_nontemporal_store(v, reinterpret_cast<v4i_alias *>(y + (unsigned)((m_base + i * 32 + h * ROWS + row) * N + n_base + ch * 8)));
                }
                asm volatile("" ::: "memory");
                if (glue.rowmax && lane < ROWS) {
                    const unsigned mx = *reinterpret_cast<const unsigned __attribute__((may_alias)) *>(strip + lane * PITCH + TN * 64);
                    if (mx) atomicMax(glue.rowmax + (m_base + i * 32 + h * ROWS + lane), mx);
                    asm volatile("" ::: "memory");
                }
            }
        }
    }
}

typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// one 32x32 MFMA over a 16-byte fragment per lane: 32 int8 or 16 binary16 along K
template <bool F16, class Acc>
__device__ __forceinline__ Acc mfma_step(v4i a, v4i b, Acc c)
{
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}

}  // namespace ql
