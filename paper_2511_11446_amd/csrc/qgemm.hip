// INT8 x INT8 -> INT32 GEMM with fused dequantization for gfx950 (CDNA4).
//
// The paper's linears multiply int8 codes into int32 sums, with one weight scale per
// output channel (Step 3, Step 5, Section 6) or per weight group (Step 2).
// Here: acc[m,n] = sum_k q[m,k] * w[n,k] on v_mfma_i32_32x32x32_i8, both
// operands K-contiguous, and the dequantization + bias + fp16 conversion applied
// to the accumulators in registers.  Two kernel families:
//   qgemm_dma   tiles go global -> LDS by DMA through rings of 2-3 stages, optional
//               persistent walk over tiles; 8-bit weights, and binary16 operands for
//               the layers a plan leaves in FP16
//   qgemm_mfma  tiles staged through registers, two LDS buffers; 4-bit weights (nibbles
//               unpacked to int8 times 16 in registers, every weight group folded into
//               an fp32 sum with its scale) and 8-bit weights with K % 128 != 0
// plus a one-thread-per-element kernel for shapes and alignments neither takes.
// Activation, gate and residual can be folded into the epilogue (GLUE instantiations).
#include "qgemm_common.h"

namespace ql {

// Tile shape: a workgroup of WGM x WGN wavefronts, each owning TM x TN MFMA
// tiles of 32x32, walks K in steps of BK int8.
// WPS = wavefronts per SIMD the register budget must allow (512 / WPS registers per lane).
template <int TM_, int TN_, int WGM_, int WGN_, int BK_, bool W4_, int WPS_, bool GG_ = false>
struct Tile {
    static constexpr int TM = TM_, TN = TN_, WGM = WGM_, WGN = WGN_, BK = BK_, WPS = WPS_;
    static constexpr bool W4 = W4_;
    // 4-bit weights with a group size other than 128: any multiple of 32 that divides K (groups end at 32-wide K slices)
    static constexpr bool GG = GG_;
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int BM = WGM * TM * 32;
    static constexpr int BN = WGN * TN * 32;
    static constexpr int BKB = W4 ? BK / 2 : BK;  // bytes of one B row per K step
    static constexpr int LDA = BK + 16;            // LDS row pitch, padded against bank conflicts
    static constexpr int LDB = BKB + 16;
    static constexpr int A_ITERS = BM * BK / 16 / NT;
    static constexpr int B_ITERS = BN * BKB / 16 / NT;
    static constexpr int A_BYTES = BM * LDA;
    static constexpr int B_BYTES = BN * LDB;
    static constexpr int S_BYTES = W4 ? 2 * BN * 4 : 0;
    static constexpr int LDS_BYTES = 2 * A_BYTES + 2 * B_BYTES + S_BYTES;
    static_assert(BM * BK / 16 % NT == 0 && BN * BKB / 16 % NT == 0, "tile loads must divide over the threads");
    static_assert(!W4 || BK == 128, "one K step is one 128-wide weight group");
    static_assert(!GG || W4, "group sizes apply to 4-bit weights");
    static_assert(BM * 4 <= 2 * A_BYTES, "row-scale staging reuses the A buffers");
};

template <class T, bool GLUE = false>
__global__ __launch_bounds__(T::NT, T::WPS) void qgemm_mfma(GemmArgs a, int tiles_m, int tiles_n, int nblk_padded, int group_m)
{
    constexpr int TM = T::TM, TN = T::TN, BK = T::BK, BM = T::BM, BN = T::BN, NT = T::NT;
    constexpr int LDA = T::LDA, LDB = T::LDB, BKB = T::BKB;
    constexpr bool W4 = T::W4;
    constexpr int SLICE_UNROLL = T::GG ? 1 : BK / 32;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char *sA = smem;
    unsigned char *sB = smem + 2 * T::A_BYTES;
    float *sS = reinterpret_cast<float *>(sB + 2 * T::B_BYTES);

    // ---- which tile: spread consecutive logical tiles inside one XCD, walk group_m tile rows at a time
    // Workgroup ids go round-robin over the XCDs; each XCD owns per_xcd consecutive logical tiles and its resident
    // workgroups take them in order, gridDim.x / XCDS at a time (all of them at once unless the launch is persistent).
    const int per_xcd = nblk_padded / XCDS;
    const int slots_per_xcd = gridDim.x / XCDS;
    const int xcd_first = (blockIdx.x % XCDS) * per_xcd;
    int in_xcd = blockIdx.x / XCDS;
    if (in_xcd >= per_xcd || xcd_first + in_xcd >= tiles_m * tiles_n) return;
    int m0, n0;
    auto set_tile = [&](int logical) {
        const int group_sz = group_m * tiles_n;
        const int first_m = (logical / group_sz) * group_m;
        const int gm = min(tiles_m - first_m, group_m);
        m0 = (first_m + (logical % group_sz) % gm) * BM;
        n0 = ((logical % group_sz) / gm) * BN;
    };
    set_tile(xcd_first + in_xcd);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / T::WGN, wn = wave % T::WGN;
    const int M = a.M, N = a.N, K = a.K;
    const int KB = W4 ? K / 2 : K;  // bytes per weight row
    const int G = T::GG ? K / a.group : K / 128;   // weight groups along K
    const int QG = T::GG ? a.group / 32 : 4;         // 32-wide K slices per weight group
    const int nk = K / BK;  // the dispatcher only sends K % BK == 0 here

    // ---- global -> register staging of one K step
    v4i ga[T::A_ITERS], gb[T::B_ITERS];
    float gs = 0.0f;
    auto load_tile = [&](int kt) {
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < T::A_ITERS; ++i) {
            const int c = tid + i * NT;
            const int row = c / (BK / 16), cc = c % (BK / 16);
            const int gr = min(m0 + row, M - 1);
            ga[i] = *reinterpret_cast<const v4i *>(a.q + (size_t)gr * K + (k0 + cc * 16));
        }
        const int kb0 = W4 ? k0 / 2 : k0;
#pragma unroll
        for (int i = 0; i < T::B_ITERS; ++i) {
            const int c = tid + i * NT;
            const int row = c / (BKB / 16), cc = c % (BKB / 16);
            const int gr = min(n0 + row, N - 1);
            gb[i] = *reinterpret_cast<const v4i *>(static_cast<const unsigned char *>(a.w) + (size_t)gr * KB + (kb0 + cc * 16));
        }
        if (W4 && !T::GG && (k0 % 128) == 0 && tid < BN) {
            const int gr = min(n0 + tid, N - 1);
            // the nibbles are used as value*16, so the group scale carries the 1/16 (exact: a power of two)
            gs = half_to_float_dev(static_cast<const unsigned short *>(a.s_w)[(size_t)gr * G + k0 / 128]) * 0.0625f;
        }
    };
    auto store_tile = [&](int kt) {
        unsigned char *dA = sA + (kt & 1) * T::A_BYTES;
        unsigned char *dB = sB + (kt & 1) * T::B_BYTES;
#pragma unroll
        for (int i = 0; i < T::A_ITERS; ++i) {
            const int c = tid + i * NT;
            *reinterpret_cast<v4i *>(dA + (c / (BK / 16)) * LDA + (c % (BK / 16)) * 16) = ga[i];
        }
#pragma unroll
        for (int i = 0; i < T::B_ITERS; ++i) {
            const int c = tid + i * NT;
            *reinterpret_cast<v4i *>(dB + (c / (BKB / 16)) * LDB + (c % (BKB / 16)) * 16) = gb[i];
        }
        if (W4 && !T::GG && ((kt * BK) % 128) == 0 && tid < BN) sS[(((kt * BK) / 128) & 1) * BN + tid] = gs;
    };

    v16i acc[TM][TN];
    float fsum[W4 ? TM : 1][W4 ? TN : 1][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
            if (W4) {
#pragma unroll
                for (int r = 0; r < 16; ++r) fsum[i][j][r] = 0.0f;
            }
        }

    // lane -> fragment: row (lane & 31) of a 32-row tile, k offset 16 * (lane >> 5) inside a 32-wide K slice
    const int frag_row = lane & 31, frag_half = lane >> 5;
    const int a_off = (wm * TM * 32 + frag_row) * LDA + frag_half * 16;
    const int b_off = (wn * TN * 32 + frag_row) * LDB + frag_half * (W4 ? 8 : 16);

    int qs = 0, grp = 0;   // generic group size: slice inside the current weight group, and the group's number
    unsigned short sgrp[TN] = {};
    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_tile(kt + 1);
        const unsigned char *pa = sA + (kt & 1) * T::A_BYTES + a_off;
        const unsigned char *pb = sB + (kt & 1) * T::B_BYTES + b_off;
        // with run-time group ends the four slices share one copy of the code
#pragma unroll SLICE_UNROLL
        for (int ks = 0; ks < BK / 32; ++ks) {
            v4i af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const v4i *>(pa + i * 32 * LDA + ks * 32);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (W4) {
                    const v2i p = *reinterpret_cast<const v2i *>(pb + j * 32 * LDB + ks * 16);
                    // byte b of a packed word: low nibble = k b, high nibble = k 4+b  ->  int8 value * 16
                    bf[j] = v4i{(int)(((unsigned)p[0] << 4) & 0xf0f0f0f0u), (int)((unsigned)p[0] & 0xf0f0f0f0u),
                                (int)(((unsigned)p[1] << 4) & 0xf0f0f0f0u), (int)((unsigned)p[1] & 0xf0f0f0f0u)};
                } else {
                    bf[j] = *reinterpret_cast<const v4i *>(pb + j * 32 * LDB + ks * 32);
                }
            }
            if (T::GG) {
                // slice number qs of the current group (wavefront-uniform): the group's scales are requested at its
                // first slice; after its last slice the partial sums are folded into the fp32 sum and the accumulators
                // cleared (one code path for the MFMAs: a second one with a zero C operand doubled the register need)
                if (qs == 0) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        sgrp[j] = static_cast<const unsigned short *>(a.s_w)[(size_t)min(n0 + wn * TN * 32 + j * 32 + frag_row, N - 1) * G + grp];
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
                if (++qs == QG) {
                    qs = 0;
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int n = n0 + wn * TN * 32 + j * 32 + frag_row;
                        // the nibbles are used as value*16, so the group scale carries the 1/16 (exact: a power of two)
                        const float s16 = half_to_float_dev(sgrp[j]) * 0.0625f;
#pragma unroll
                        for (int i = 0; i < TM; ++i)
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                if (a.acc_out) {
                                    const int m = m0 + wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                                    if (m < M && n < N) a.acc_out[(unsigned)((m * G + grp) * N + n)] = acc[i][j][r] >> 4;
                                }
                                fsum[W4 ? i : 0][W4 ? j : 0][r] = __builtin_fmaf((float)acc[i][j][r], s16, fsum[W4 ? i : 0][W4 ? j : 0][r]);
                                acc[i][j][r] = 0;
                            }
                    }
                    ++grp;
                }
                continue;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    // a weight group (= one K step) starts from a zero accumulator
                    const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], (W4 && ks == 0) ? zero : acc[i][j], 0, 0, 0);
                }
        }
        if (W4 && !T::GG) {
            // the weight group ends here: fold its int32 partial sums into the fp32 sum with the group scale
            const int g = kt;
            const float *sc = sS + (g & 1) * BN + wn * TN * 32 + frag_row;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float s16 = sc[j * 32];
                const int n = n0 + wn * TN * 32 + j * 32 + frag_row;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        if (a.acc_out) {
                            const int m = m0 + wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                            if (m < M && n < N) a.acc_out[(unsigned)((m * G + g) * N + n)] = acc[i][j][r] >> 4;
                        }
                        fsum[i][j][r] = __builtin_fmaf((float)acc[i][j][r], s16, fsum[i][j][r]);
                    }
            }
        }
        if (kt + 1 < nk) store_tile(kt + 1);
        __syncthreads();
    }

    // ---- epilogue: activation scale per row (staged in LDS), weight scale and bias per column
    float *sRow = reinterpret_cast<float *>(smem);
    for (int t = tid; t < BM; t += NT) sRow[t] = a.s_a[min(m0 + t, M - 1) / a.R];
    __syncthreads();
    _Float16 *y = static_cast<_Float16 *>(a.y);
    const unsigned short *bias = static_cast<const unsigned short *>(a.bias);
    const bool full = (m0 + BM <= M) && (n0 + BN <= N);
    auto emit = [&](auto edge) {
        constexpr bool EDGE = decltype(edge)::value;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * TN * 32 + j * 32 + frag_row;
            const bool n_ok = !EDGE || n < N;
            const float sw = (!W4 && n_ok) ? static_cast<const float *>(a.s_w)[n] : 1.0f;
            const float b = (bias && n_ok) ? half_to_float_dev(bias[n]) : 0.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    const int m = m0 + row;
                    if (!EDGE || (m < M && n_ok)) {
                        const float sa = sRow[row];
                        const unsigned off = (unsigned)(m * N + n);
                        float u;
                        if (W4) {
                            u = bias ? __builtin_fmaf(fsum[i][j][r], sa, b) : fsum[i][j][r] * sa;
                        } else {
                            const float t = (float)acc[i][j][r] * sa;
                            u = bias ? __builtin_fmaf(t, sw, b) : t * sw;
                            if (a.acc_out) a.acc_out[off] = acc[i][j][r];
                        }
                        if (GLUE) __builtin_nontemporal_store(glue_one(a, u, m, n, GateRows(a.gate, a.gate_rows, m0, BM).of(row)), &y[off]);
                        else __builtin_nontemporal_store((_Float16)u, &y[off]);
                    }
                }
        }
    };
    if (full) emit(std::false_type{});
    else emit(std::true_type{});
}

// ---------------------------------------------------------------------------------------------
// Pipelined variant: tiles go from global memory straight into LDS (global_load_lds_dwordx4, no
// register staging) through a ring of S stages.  One K step is 128 int8 = one 128-byte LDS row, so
// every DMA instruction moves 8 rows x 128 contiguous bytes (whole cache lines; 64-byte pieces were
// measured at little more than half the L1 fill rate).  The 16-byte chunk c of row r is kept at slot
// c ^ ((r >> 1) & 7) of its row: rows are unpadded (a wavefront's DMA writes 1024 contiguous bytes),
// and the XOR spreads the 16 lanes that read one chunk index of 16 consecutive rows over all banks.
// The K step is multiplied in four 32-wide quarters with double-buffered fragments: the reads of
// the next quarter, the hand-over barrier and the next DMA issue all sit behind an MFMA that is
// already executing.
// ---------------------------------------------------------------------------------------------
template <int TM_, int TN_, int WGM_, int WGN_, int S_, int WPS_, bool STG_ = true, int EV_ = 0, bool W4_ = false, int SB_ = S_, bool PERSIST_ = false, bool F16_ = false>
struct TileD {
    static constexpr int TM = TM_, TN = TN_, WGM = WGM_, WGN = WGN_, WPS = WPS_;
    // ring depth of the activation tile and of the weight tile (K steps resident or in flight); they may differ by one
    static constexpr int SA = S_, SB = SB_;
    static constexpr bool W4 = W4_;
    // both operands binary16 (a layer the plan leaves unquantized): one K step is 64 values = the same 128 bytes per row
    static constexpr bool F16 = F16_;
    static_assert(!(F16_ && W4_), "FP16 layers have no packed weights");
    static constexpr int NW = WGM * WGN, NT = NW * 64;
    static constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32, BK = 128;
    // 1024-byte DMA groups per K step: A rows (8 rows x 128 B) and W rows (8 x 128 B, or 16 x 64 B packed 4-bit)
    static constexpr int A_GROUPS = BM / 8, B_GROUPS = W4 ? BN / 16 : BN / 8;
    static constexpr int NA = A_GROUPS / NW, NB = B_GROUPS / NW;   // DMA instructions per wavefront per K step
    static constexpr int A_BYTES = A_GROUPS * 1024, B_BYTES = B_GROUPS * 1024;
    static constexpr int B_RING = SA * A_BYTES;           // the weight ring follows the activation ring
    static constexpr bool STAGED_STORE = STG_;
    static constexpr int DMA_EVERY = EV_;                 // one DMA instruction behind every EV_-th MFMA; 0: all at the hand-over
    static constexpr int STRIP_OFF = (BM * 4 + 255) / 256 * 256;   // epilogue: row scales first, then one strip per wavefront
    // a persistent workgroup parks its epilogue beside stage 0; where a 32-row strip per wavefront does not fit there,
    // the strip holds 16 rows
    static constexpr int STRIP_ROWS = (PERSIST_ && (SA - 1) * A_BYTES < STRIP_OFF + NW * 32 * (TN * 64 + 16)) ? 16 : 32;
    static constexpr int STRIP_BYTES = STRIP_ROWS * (TN * 64 + 16);
    static constexpr int RINGS = SA * A_BYTES + SB * B_BYTES;
    static constexpr int RING_BYTES = RINGS > STRIP_OFF + NW * STRIP_BYTES ? RINGS : STRIP_OFF + NW * STRIP_BYTES;
    static constexpr int MAX_GROUPS_K = 40;               // 4-bit: group scales of the tile's columns live in LDS (K <= 5120)
    static constexpr int SCALE_BYTES = W4 ? BN * MAX_GROUPS_K * 2 : 0;
    static constexpr int LDS_BYTES = RING_BYTES + SCALE_BYTES;
    static constexpr int SMAX = SA > SB ? SA : SB;
    // Persistent launch: a workgroup walks several tiles and requests the first K step of the next tile before it
    // starts the epilogue of the current one, into stage 0 of both rings; the epilogue's scratch then lives in the
    // later stages of the activation ring.
    static constexpr bool PERSIST = PERSIST_;
    static constexpr int EPI_OFF = PERSIST ? A_BYTES : 0;
    static_assert(!PERSIST || (!W4 && (SA - 1) * A_BYTES >= STRIP_OFF + NW * STRIP_BYTES), "epilogue scratch beside stage 0");
    // loads that may still be in flight when K step 0 is first read, and at the hand-over from step kt to kt+1
    static constexpr int WAIT_START = (SA - 1) * NA + (SB - 1) * NB;
    static constexpr int WAIT_HAND = SA > SB ? NA + (SB - 2) * (NA + NB) : SA < SB ? NB + (SA - 2) * (NA + NB) : (SA - 2) * (NA + NB);
    static_assert(A_GROUPS % NW == 0 && B_GROUPS % NW == 0, "every wavefront issues the same number of DMA instructions");
    static_assert(SA >= 2 && SB >= 2 && (SA - SB) * (SA - SB) <= 1, "ring depths differ by at most one");
    static_assert(WAIT_START <= 63, "vmcnt is a 6-bit counter");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
};

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

template <class T, bool GLUE = false>
__global__ __launch_bounds__(T::NT, T::WPS) void qgemm_dma(GemmArgs a, int tiles_m, int tiles_n, int nblk_padded, int group_m)
{
    constexpr int TM = T::TM, TN = T::TN, BM = T::BM, BN = T::BN, NT = T::NT, NW = T::NW;
    constexpr bool W4 = T::W4, F16 = T::F16;
    constexpr int EB = F16 ? 2 : 1;   // bytes per element of both operands
    extern __shared__ __align__(1024) unsigned char smem[];

    // Workgroup ids go round-robin over the XCDs; each XCD owns per_xcd consecutive logical tiles and its resident
    // workgroups take them in order, gridDim.x / XCDS at a time (all of them at once unless the launch is persistent).
    const int per_xcd = nblk_padded / XCDS;
    const int slots_per_xcd = gridDim.x / XCDS;
    const int xcd_first = (blockIdx.x % XCDS) * per_xcd;
    int in_xcd = blockIdx.x / XCDS;
    if (in_xcd >= per_xcd || xcd_first + in_xcd >= tiles_m * tiles_n) return;
    int m0, n0;
    auto set_tile = [&](int logical) {
        const int group_sz = group_m * tiles_n;
        const int first_m = (logical / group_sz) * group_m;
        const int gm = min(tiles_m - first_m, group_m);
        m0 = (first_m + (logical % group_sz) % gm) * BM;
        n0 = ((logical % group_sz) / gm) * BN;
    };
    set_tile(xcd_first + in_xcd);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in a scalar register
    const int wm = wave / T::WGN, wn = wave % T::WGN;
    const int M = a.M, N = a.N, K = a.K;
    const int nk = K * EB / 128;   // K steps (128 bytes per row); for 4-bit weights also the number of weight groups
    QL_PHASE(0)

    // Everything the epilogue needs from global memory is requested now, ahead of the first DMA (the oldest loads
    // return first, so the vmcnt bookkeeping of the ring is unaffected): the activation scale of one tile row per
    // thread, and the weight scale and bias of this lane's columns.
    static_assert(BM <= NT, "one row scale per thread");
    float sa_pre, swt[TN], bj[TN];
    auto load_scales = [&]() {
        sa_pre = (!F16 && tid < BM) ? a.s_a[min(m0 + tid, M - 1) / a.R] : 1.0f;
        const unsigned short *bias_h = static_cast<const unsigned short *>(a.bias);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = min(n0 + wn * TN * 32 + j * 32 + (lane & 31), N - 1);
            swt[j] = (W4 || F16) ? 1.0f : static_cast<const float *>(a.s_w)[n];
            bj[j] = bias_h ? half_to_float_dev(bias_h[n]) : 0.0f;
        }
    };
    if (!T::PERSIST) load_scales();

    // 4-bit weights: the fp16 group scales of this tile's columns, [BN][nk], copied once (the first barrier of the
    // pipeline below orders the copy before their first use at the end of K step 0)
    unsigned short *sScale = reinterpret_cast<unsigned short *>(smem + T::RING_BYTES);
    if (W4) {
        const unsigned short *gsw = static_cast<const unsigned short *>(a.s_w);
        for (int idx = tid; idx < BN * nk; idx += NT)
            sScale[idx] = gsw[(size_t)min(n0 + idx / nk, N - 1) * nk + idx % nk];
    }

    // DMA addressing: lane l of a wavefront fills bytes [16 l, 16 l + 16) of a 1024-byte group = row l/8, slot l%8.
    // Group g covers tile rows [8 g, 8 g + 8) of its operand.  Wavefront w takes groups w, w+NW, ... of both operands.
    constexpr int SA = T::SA, SB = T::SB, NA = T::NA, NB = T::NB;
    unsigned goffA[NA], goffB[NB];
    auto set_goff = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int row = 8 * (wave + i * NW) + (lane >> 3);
            const int c = (lane & 7) ^ ((row >> 1) & 7);
            goffA[i] = (unsigned)(min(m0 + row, M - 1) * K * EB + 16 * c);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if (!W4) {
                const int row = 8 * (wave + i * NW) + (lane >> 3);
                const int c = (lane & 7) ^ ((row >> 1) & 7);
                goffB[i] = (unsigned)(min(n0 + row, N - 1) * K * EB + 16 * c);
            } else {
                // packed 4-bit rows are 64 bytes per K step: 16 rows per group, chunk c of row r at slot c ^ ((r >> 2) & 3)
                const int row = 16 * (wave + i * NW) + (lane >> 2);
                const int c = (lane & 3) ^ ((row >> 2) & 3);
                goffB[i] = (unsigned)(min(n0 + row, N - 1) * (K / 2) + 16 * c);
            }
        }
    };
    set_goff();
    auto issue_a = [&](int kt, int slot, int i) {
        __builtin_amdgcn_global_load_lds((global_void *)(a.q + (size_t)kt * 128 + goffA[i]),
                                         (lds_void *)(smem + slot * T::A_BYTES + (wave + i * NW) * 1024), 16, 0, 0);
    };
    auto issue_b = [&](int kt, int slot, int i) {
        __builtin_amdgcn_global_load_lds((global_void *)(static_cast<const int8_t *>(a.w) + (size_t)kt * (W4 ? 64 : 128) + goffB[i]),
                                         (lds_void *)(smem + T::B_RING + slot * T::B_BYTES + (wave + i * NW) * 1024), 16, 0, 0);
    };
    // Refill window j = the loads issued after the hand-over barrier of K step j, into the slots that step used:
    // weight tile of step j+SB and activation tile of step j+SA.  The operand with the shallower ring is needed sooner
    // and goes first.  li numbers the NA+NB instructions of the window.
    constexpr bool B_FIRST = SB <= SA;
    auto issue_win = [&](int j, int slot_a, int slot_b, int li) {
        const bool is_b = B_FIRST ? li < NB : li >= NA;
        if (is_b) {
            if (j + SB < nk) issue_b(j + SB, slot_b, B_FIRST ? li : li - NA);
        } else {
            if (j + SA < nk) issue_a(j + SA, slot_a, B_FIRST ? li - NB : li);
        }
    };
    auto wait_vm = [&](auto n_tag) {
        constexpr int n = decltype(n_tag)::value;
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory");
    };

    typedef typename std::conditional<F16, v16f, v16i>::type acc_t;   // fp32 accumulators for FP16 operands
    acc_t acc[TM][TN];
    // 4-bit weights: fp32 sum over the weight groups, f = sum_g fma(float(P_g), s_w[n,g], f)
    float fsum[W4 ? TM : 1][W4 ? TN : 1][16];
    auto clear_sums = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    acc[i][j][r] = 0;
                    if (W4) fsum[W4 ? i : 0][W4 ? j : 0][r] = 0.0f;
                }
    };

    // fragment of a lane: row (lane & 31) of a 32-row tile, 16 k starting at 32 * quarter + 16 * (lane >> 5)
    const int frag_row = lane & 31, frag_half = lane >> 5;
    const int key = (lane >> 1) & 7;  // swizzle key of this lane's row (tile rows start at multiples of 32)
    const int key4 = (lane >> 2) & 3; // the same for the 64-byte rows of packed 4-bit weights
    const int a_off = (wm * TM * 32 + frag_row) * 128;
    const int b_off = T::B_RING + (wn * TN * 32 + frag_row) * (W4 ? 64 : 128);
    auto read_frags = [&](int sl_a, int sl_b, int quarter, v4i(&af)[TM], v4i(&bf)[TN]) {
        const unsigned char *st = smem + sl_a * T::A_BYTES;
        const unsigned char *stb = smem + sl_b * T::B_BYTES;
        const int so = ((2 * quarter + frag_half) ^ key) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const v4i *>(st + a_off + i * 32 * 128 + so);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (W4) {
                // 16 k of a quarter's half = 8 packed bytes; byte b of a word: low nibble = k b, high nibble = k 4+b
                const v2i p = *reinterpret_cast<const v2i *>(stb + b_off + j * 32 * 64 + ((quarter ^ key4) * 16) + frag_half * 8);
                bf[j] = v4i{(int)(((unsigned)p[0] << 4) & 0xf0f0f0f0u), (int)((unsigned)p[0] & 0xf0f0f0f0u),
                            (int)(((unsigned)p[1] << 4) & 0xf0f0f0f0u), (int)((unsigned)p[1] & 0xf0f0f0f0u)};  // int8 value * 16
            } else {
                bf[j] = *reinterpret_cast<const v4i *>(stb + b_off + j * 32 * 128 + so);
            }
        }
    };
    // 4-bit weights: K step kt is weight group kt.  Its int32 partial sums (times 16) are folded into the fp32 sum
    // right before the accumulator is restarted; the group scale carries the 1/16 (exact: a power of two).
    int flush_group = -1;  // group whose partial sums are still in acc
    auto flush_tile = [&](int i, int j) {
        if constexpr (F16) return;
        else {
        const int n_loc = wn * TN * 32 + j * 32 + frag_row;
        const float s16 = half_to_float_dev(sScale[n_loc * nk + flush_group]) * 0.0625f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (a.acc_out) {
                const int m = m0 + wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4), n = n0 + n_loc;
                if (m < M && n < N) a.acc_out[(unsigned)((m * nk + flush_group) * N + n)] = acc[i][j][r] >> 4;
            }
            fsum[W4 ? i : 0][W4 ? j : 0][r] = __builtin_fmaf((float)acc[i][j][r], s16, fsum[W4 ? i : 0][W4 ? j : 0][r]);
        }
        }
    };
    // MFMAs number [first, last) of one quarter, in (i, j) order; restart = first quarter of a 4-bit weight group
    auto mma = [&](const v4i(&af)[TM], const v4i(&bf)[TN], int first, int last, bool restart = false) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                if (i * TN + j >= first && i * TN + j < last) {
                    if (W4 && restart) {
                        if (flush_group >= 0) flush_tile(i, j);
                        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                        if constexpr (!F16) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], zero, 0, 0, 0);
                    } else {
                        acc[i][j] = mfma_step<F16>(af[i], bf[j], acc[i][j]);
                    }
                }
    };
    constexpr int NMMA = TM * TN;
    // The same, with one DMA instruction of K step kt_i slipped in after every EVERY-th MFMA, starting with load i0:
    // 64 loads issued back to back fill the texture-address queue and stall the MFMA issue of every wavefront.
    constexpr int EVERY = T::DMA_EVERY > 0 ? T::DMA_EVERY : 1;
    constexpr bool SPREAD = T::DMA_EVERY > 0;
    auto mma_dma = [&](const v4i(&af)[TM], const v4i(&bf)[TN], int first, int last, bool on, int win, int slot_a, int slot_b, int i0,
                       bool restart = false) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int idx = i * TN + j;
                if (idx >= first && idx < last) {
                    if (W4 && restart) {
                        if (flush_group >= 0) flush_tile(i, j);
                        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                        if constexpr (!F16) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], zero, 0, 0, 0);
                    } else {
                        acc[i][j] = mfma_step<F16>(af[i], bf[j], acc[i][j]);
                    }
                    const int li = i0 + (idx - first) / EVERY;
                    if (SPREAD && (idx - first) % EVERY == EVERY - 1 && li < NA + NB) {
                        if (on) issue_win(win, slot_a, slot_b, li);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
    };
    constexpr int N_Q = (NMMA - 1) / EVERY;    // loads that fit behind the MFMAs of one quarter
    static_assert(!SPREAD || 3 * N_Q >= NA + NB, "the loads of a refill window must be issued within three quarters");

    // prologue: the first SA activation tiles and SB weight tiles, in K-step order.  A persistent workgroup requests
    // step 0 ahead of everything else (for its first tile here, for later tiles before the previous epilogue).
    auto issue_step0 = [&]() {
        if (0 < nk) {
#pragma unroll
            for (int i = 0; i < NA; ++i) issue_a(0, 0, i);
#pragma unroll
            for (int i = 0; i < NB; ++i) issue_b(0, 0, i);
        }
    };
    if (T::PERSIST) issue_step0();
    for (;;) {   // one pass per tile; a single pass unless the launch is persistent
    if (T::PERSIST) load_scales();
    clear_sums();
    flush_group = -1;
    if (!T::PERSIST) issue_step0();
#pragma unroll
    for (int st = 1; st < T::SMAX; ++st) {
        if (st < SA && st < nk) {
#pragma unroll
            for (int i = 0; i < NA; ++i) issue_a(st, st, i);
        }
        if (st < SB && st < nk) {
#pragma unroll
            for (int i = 0; i < NB; ++i) issue_b(st, st, i);
        }
    }
    QL_PHASE(1)
    v4i af0[TM], bf0[TN], af1[TM], bf1[TN];
    // K step 0 has landed once only the later steps of the prologue are outstanding
    if (nk >= T::SMAX) wait_vm(std::integral_constant<int, T::WAIT_START>{});
    else wait_vm(std::integral_constant<int, 0>{});
    __builtin_amdgcn_s_barrier();
    read_frags(0, 0, 0, af0, bf0);
    int sa = 0, sb = 0, pa = SA - 1, pb = SB - 1;   // ring slots of K step kt and of step kt-1
    for (int kt = 0; kt < nk; ++kt) {
        const int na = sa + 1 == SA ? 0 : sa + 1, nb = sb + 1 == SB ? 0 : sb + 1;
        const bool refill = kt > 0;   // refill window kt-1 is still being issued during quarters 0 and 1
        // quarter 0 (fragments 0) while reading quarter 1 (fragments 1)
        mma(af0, bf0, 0, 1, true);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(sa, sb, 1, af1, bf1);
        __builtin_amdgcn_sched_barrier(0);
        mma_dma(af0, bf0, 1, NMMA, refill, kt - 1, pa, pb, N_Q, true);
        flush_group = kt;
        __builtin_amdgcn_sched_barrier(0);
        // quarter 1 while reading quarter 2
        mma(af1, bf1, 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(sa, sb, 2, af0, bf0);
        __builtin_amdgcn_sched_barrier(0);
        mma_dma(af1, bf1, 1, NMMA, refill, kt - 1, pa, pb, 2 * N_Q);
        __builtin_amdgcn_sched_barrier(0);
        // quarter 2 while reading quarter 3
        mma(af0, bf0, 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(sa, sb, 3, af1, bf1);
        __builtin_amdgcn_sched_barrier(0);
        mma(af0, bf0, 1, NMMA);
        __builtin_amdgcn_sched_barrier(0);
        // quarter 3: its first MFMA needs the last fragments of this K step, so once it has issued every read of
        // this step's slots by this wavefront is complete.  Then hand over: step kt+1 must be in LDS (only loads
        // issued after its last one may still be in flight), and after the barrier this step's slots can be refilled.
        mma(af1, bf1, 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (kt + T::SMAX <= nk) wait_vm(std::integral_constant<int, T::WAIT_HAND>{});
        else wait_vm(std::integral_constant<int, 0>{});
        __builtin_amdgcn_s_barrier();
        if (!SPREAD) {
#pragma unroll
            for (int li = 0; li < NA + NB; ++li) issue_win(kt, sa, sb, li);
        }
        if (kt + 1 < nk) read_frags(na, nb, 0, af0, bf0);
        __builtin_amdgcn_sched_barrier(0);
        mma_dma(af1, bf1, 1, NMMA, true, kt, sa, sb, 0);
        __builtin_amdgcn_sched_barrier(0);
        pa = sa;
        pb = sb;
        sa = na;
        sb = nb;
    }
    if (W4) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) flush_tile(i, j);
    }
    QL_PHASE(2)
    __syncthreads();

    // the tile being written out; a persistent workgroup moves on to its next tile first and requests that tile's
    // first K step, so that it travels while the epilogue runs
    const int em0 = m0, en0 = n0;
    bool has_next = false;
    if (T::PERSIST) {
        in_xcd += slots_per_xcd;
        has_next = in_xcd < per_xcd && xcd_first + in_xcd < tiles_m * tiles_n;
        if (has_next) {
            set_tile(xcd_first + in_xcd);
            set_goff();
            issue_step0();
        }
    }
    float *sRow = reinterpret_cast<float *>(smem + T::EPI_OFF);
    if (tid < BM) sRow[tid] = sa_pre;
    __syncthreads();
    QL_PHASE(3)
    _Float16 *y = static_cast<_Float16 *>(a.y);
    const unsigned short *bias = static_cast<const unsigned short *>(a.bias);
    const bool full = (em0 + BM <= M) && (en0 + BN <= N);
    const bool glue_pieces = GLUE && (a.residual || a.gate);
    const bool glue_aligned = !glue_pieces || (((reinterpret_cast<uintptr_t>(a.residual) | reinterpret_cast<uintptr_t>(a.gate)) & 15) == 0);
    if (full && (N % 8) == 0 && (reinterpret_cast<uintptr_t>(a.y) & 15) == 0 && (W4 || !a.acc_out) && glue_aligned) {
        GluePieces gl;
        if (glue_pieces) {
            gl.gate = static_cast<const _Float16 *>(a.gate);
            gl.residual = static_cast<const _Float16 *>(a.residual);
            gl.gate_rows = a.gate_rows;
            gl.on = true;
        }
        if (GLUE) gl.rowmax = a.row_absmax;
        unsigned char *strip = smem + T::EPI_OFF + T::STRIP_OFF + wave * T::STRIP_BYTES;
        // the 16 row scales of each 32-row block of this lane (rows 8g + 4*frag_half + 0..3), read once as 4 x 16 bytes
        float sr[TM * 16];
        {
            const float *srow = sRow + wm * TM * 32 + 4 * frag_half;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const v4f t = *reinterpret_cast<const v4f *>(srow + i * 32 + 8 * g);
                    sr[i * 16 + 4 * g + 0] = t[0];
                    sr[i * 16 + 4 * g + 1] = t[1];
                    sr[i * 16 + 4 * g + 2] = t[2];
                    sr[i * 16 + 4 * g + 3] = t[3];
                }
        }
        // the activation is chosen once per kernel, not per element
        auto emit_fast = [&](auto act_tag) {
            constexpr bool ACT = decltype(act_tag)::value;
            auto act_of = [&](float u) { return ACT ? gelu_tanh_dev(u) : u; };
            if (F16)
                store_tile_staged<TM, TN, T::STAGED_STORE, T::STRIP_ROWS>(strip, lane, y, N, em0 + wm * TM * 32, en0 + wn * TN * 32, [&](int i, int j, int r) {
                    return act_of((float)acc[i][j][r] + bj[j]);
                }, gl);
            else if (W4 && bias)
                store_tile_staged<TM, TN, T::STAGED_STORE, T::STRIP_ROWS>(strip, lane, y, N, em0 + wm * TM * 32, en0 + wn * TN * 32, [&](int i, int j, int r) {
                    return act_of(__builtin_fmaf(fsum[W4 ? i : 0][W4 ? j : 0][r], sr[i * 16 + r], bj[j]));
                }, gl);
            else if (W4)
                store_tile_staged<TM, TN, T::STAGED_STORE, T::STRIP_ROWS>(strip, lane, y, N, em0 + wm * TM * 32, en0 + wn * TN * 32, [&](int i, int j, int r) {
                    return act_of(fsum[W4 ? i : 0][W4 ? j : 0][r] * sr[i * 16 + r]);
                }, gl);
            else if (bias)
                store_tile_staged<TM, TN, T::STAGED_STORE, T::STRIP_ROWS>(strip, lane, y, N, em0 + wm * TM * 32, en0 + wn * TN * 32, [&](int i, int j, int r) {
                    return act_of(__builtin_fmaf((float)acc[i][j][r] * sr[i * 16 + r], swt[j], bj[j]));
                }, gl);
            else
                store_tile_staged<TM, TN, T::STAGED_STORE, T::STRIP_ROWS>(strip, lane, y, N, em0 + wm * TM * 32, en0 + wn * TN * 32, [&](int i, int j, int r) {
                    return act_of((float)acc[i][j][r] * sr[i * 16 + r] * swt[j]);
                }, gl);
        };
        if (GLUE && a.act == 1) emit_fast(std::true_type{});
        else emit_fast(std::false_type{});
    } else {
        auto emit = [&](auto edge) {
            constexpr bool EDGE = decltype(edge)::value;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = en0 + wn * TN * 32 + j * 32 + frag_row;
                const bool n_ok = !EDGE || n < N;
                const float b = bj[j];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                        const int m = em0 + row;
                        if (!EDGE || (m < M && n_ok)) {
                            const unsigned off = (unsigned)(m * N + n);
                            float u;
                            if (F16) {
                                u = (float)acc[i][j][r] + b;
                            } else if (W4) {
                                const float f = fsum[W4 ? i : 0][W4 ? j : 0][r];
                                u = bias ? __builtin_fmaf(f, sRow[row], b) : f * sRow[row];
                            } else {
                                const float t = (float)acc[i][j][r] * sRow[row];
                                u = bias ? __builtin_fmaf(t, swt[j], b) : t * swt[j];
                                if (a.acc_out) a.acc_out[off] = (int)acc[i][j][r];
                            }
                            asm volatile("" : "+v"(u));   // keep the fp32 rounding before the fp16 one
                            if (GLUE) y[off] = glue_one(a, u, m, n, GateRows(a.gate, a.gate_rows, em0, BM).of(row));
                            else y[off] = (_Float16)u;
                        }
                    }
            }
        };
        if (full) emit(std::false_type{});
        else emit(std::true_type{});
    }
    QL_PHASE(4)
    if (!has_next) break;
    __syncthreads();   // the epilogue's scratch is free again: the rest of the next prologue may overwrite it
    }
}

template <class T, bool GLUE = false>
static hipError_t run_dma(const GemmArgs &a, hipStream_t s)
{
    // LDS above 64 KB needs an opt-in, once per kernel (initialised thread-safely on first use)
    static const hipError_t lds_opt_in = [] {
        if (T::LDS_BYTES <= 64 * 1024) return hipSuccess;
        return hipFuncSetAttribute(reinterpret_cast<const void *>(&qgemm_dma<T, GLUE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    }();
    if (lds_opt_in != hipSuccess) return lds_opt_in;
    const int tiles_m = (a.M + T::BM - 1) / T::BM, tiles_n = (a.N + T::BN - 1) / T::BN;
    const int nblk = tiles_m * tiles_n;
    const int padded = (nblk + XCDS - 1) / XCDS * XCDS;
    int grid = padded;
    if (T::PERSIST) {
        // as many workgroups as the chip holds at once (LDS decides), a multiple of the XCD count
        static const int resident = [] {
            int dev = 0, cus = 0;
            if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
                cus < XCDS)
                return 0;   // no guess: the launch fails instead
            const int per_cu = 160 * 1024 / T::LDS_BYTES > 0 ? 160 * 1024 / T::LDS_BYTES : 1;
            return cus / XCDS * XCDS * per_cu;
        }();
        if (resident <= 0) return hipErrorInvalidDevice;
        if (grid > resident) grid = resident;
    }
    hipLaunchKernelGGL((qgemm_dma<T, GLUE>), dim3(grid), dim3(T::NT), T::LDS_BYTES, s, a, tiles_m, tiles_n, padded, pick_group_m(T::BM));
    return hipGetLastError();
}

// Any shape, no alignment needs: one thread per output element.
__global__ __launch_bounds__(256) void qgemm_naive(GemmArgs a)
{
    const int n = blockIdx.y * 64 + (threadIdx.x & 63);
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= a.M || n >= a.N) return;
    const int K = a.K;
    const unsigned short *bias = static_cast<const unsigned short *>(a.bias);
    const float b = bias ? half_to_float_dev(bias[n]) : 0.0f;
    if (a.w_bits == 16) {
        // a layer left in FP16: a.q holds the binary16 activations, a.w the binary16 weights; fp32 running sum
        const unsigned short *xr = reinterpret_cast<const unsigned short *>(a.q) + (size_t)m * K;
        const unsigned short *wr = static_cast<const unsigned short *>(a.w) + (size_t)n * K;
        float s = 0.0f;
        for (int k = 0; k < K; ++k) s = __builtin_fmaf(half_to_float_dev(xr[k]), half_to_float_dev(wr[k]), s);
        const float u16 = s + b;
        static_cast<_Float16 *>(a.y)[(size_t)m * a.N + n] = has_glue(a) ? glue_one(a, u16, m, n, a.gate ? m / a.gate_rows : 0) : (_Float16)u16;
        return;
    }
    const float sa = a.s_ag ? 1.0f : a.s_a[m / a.R];
    const int8_t *q = a.q + (size_t)m * K;
    float u;
    if (a.w_bits == 8 && !a.w_grouped) {
        const int8_t *w = static_cast<const int8_t *>(a.w) + (size_t)n * K;
        int s = 0;
        for (int k = 0; k < K; ++k) s += (int)q[k] * (int)w[k];
        if (a.acc_out) a.acc_out[(size_t)m * a.N + n] = s;
        const float t = (float)s * sa;
        const float sw = static_cast<const float *>(a.s_w)[n];
        u = bias ? __builtin_fmaf(t, sw, b) : t * sw;
    } else {
        // group-wise weight scales: packed nibbles, or int8 codes of any width up to 8 bits
        const unsigned char *w = static_cast<const unsigned char *>(a.w) + (size_t)n * (a.w_grouped ? K : K / 2);
        const int gsz = a.group;
        const int G = K / gsz;
        float f = 0.0f;
        for (int g = 0; g < G; ++g) {
            int s = 0;
            for (int k = gsz * g; k < gsz * g + gsz; ++k) {
                int v;
                if (a.w_grouped) {
                    v = (int)(int8_t)w[k];
                } else {
                    const unsigned byte = w[4 * (k / 8) + (k % 4)];
                    v = (k % 8) >= 4 ? (int)(byte >> 4) : (int)(byte & 0xf);
                    v = v >= 8 ? v - 16 : v;
                }
                s += (int)q[k] * v;
            }
            if (a.acc_out) a.acc_out[((size_t)m * G + g) * a.N + n] = s;
            float c = half_to_float_dev(static_cast<const unsigned short *>(a.s_w)[(size_t)n * G + g]);
            if (a.s_ag) c = c * a.s_ag[(size_t)(m / a.R) * G + g];
            f = __builtin_fmaf((float)s, c, f);
        }
        u = bias ? __builtin_fmaf(f, sa, b) : f * sa;
    }
    static_cast<_Float16 *>(a.y)[(size_t)m * a.N + n] = has_glue(a) ? glue_one(a, u, m, n, a.gate ? m / a.gate_rows : 0) : (_Float16)u;
}

// ---- variants -----------------------------------------------------------------
template <class T, bool GLUE = false>
static hipError_t run_variant(const GemmArgs &a, hipStream_t s)
{
    static const hipError_t lds_opt_in = [] {
        if (T::LDS_BYTES <= 64 * 1024) return hipSuccess;
        return hipFuncSetAttribute(reinterpret_cast<const void *>(&qgemm_mfma<T, GLUE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    }();
    if (lds_opt_in != hipSuccess) return lds_opt_in;
    const int tiles_m = (a.M + T::BM - 1) / T::BM, tiles_n = (a.N + T::BN - 1) / T::BN;
    const int nblk = tiles_m * tiles_n;
    const int padded = (nblk + XCDS - 1) / XCDS * XCDS;
    hipLaunchKernelGGL((qgemm_mfma<T, GLUE>), dim3(padded), dim3(T::NT), T::LDS_BYTES, s, a, tiles_m, tiles_n, padded, pick_group_m(T::BM));
    return hipGetLastError();
}

struct Variant {
    const char *name;
    int w_bits, BM, BN, BK;   // BK: K must be a multiple of this
    hipError_t (*run)(const GemmArgs &, hipStream_t);
    hipError_t (*run_glue)(const GemmArgs &, hipStream_t) = nullptr;   // the same tile with block glue in the epilogue (shape-chosen variants only)
};

//                         TM TN WGM WGN BK  W4  WPS
using W8_128x128_k64 = Tile<2, 2, 2, 2, 64, false, 2>;
using W8_128x128_k128 = Tile<2, 2, 2, 2, 128, false, 2>;
using W8_256x128_k64 = Tile<4, 2, 2, 2, 64, false, 2>;
using W8_256x128_k128 = Tile<4, 2, 2, 2, 128, false, 2>;
using W8_128x192_k64 = Tile<2, 3, 2, 2, 64, false, 2>;
using W8_256x192_k64 = Tile<4, 3, 2, 2, 64, false, 1>;
using W8_256x256_8w = Tile<4, 2, 2, 4, 64, false, 2>;
using W8_64x64_k64 = Tile<1, 1, 2, 2, 64, false, 4>;
using W8_128x128_k64_o3 = Tile<2, 2, 2, 2, 64, false, 3>;
using W4_128x128_k128 = Tile<2, 2, 2, 2, 128, true, 2>;
using W4_64x128_k128 = Tile<1, 2, 2, 2, 128, true, 2>;
using W4_256x128_8w = Tile<2, 2, 4, 2, 128, true, 2>;
using W4_128x64_k128 = Tile<2, 1, 2, 2, 128, true, 3>;
using W4G_128x64_k128 = Tile<2, 1, 2, 2, 128, true, 3, true>;   // any group size that is a multiple of 32
using W4G_128x128_k128 = Tile<2, 2, 2, 2, 128, true, 2, true>;
using W4G_64x128_k128 = Tile<1, 2, 2, 2, 128, true, 3, true>;
using W4G_64x64_k128 = Tile<1, 1, 2, 2, 128, true, 4, true>;

//                          TM TN WGM WGN S WPS
using D8_128x128_s3 = TileD<2, 2, 2, 2, 3, 2>;
using D8_128x128_s2 = TileD<2, 2, 2, 2, 2, 2>;
using D8_128x192_s3 = TileD<2, 3, 2, 2, 3, 2>;
using D8_128x192_s2 = TileD<2, 3, 2, 2, 2, 2>;
using D8_256x128_s3 = TileD<4, 2, 2, 2, 3, 1>;
using D8_256x192_s2 = TileD<4, 3, 2, 2, 2, 1>;
using D8_256x256_8w = TileD<4, 2, 2, 4, 2, 2>;
using D8_256x192_8w = TileD<2, 3, 4, 2, 2, 2>;
using D8_256x192_8w_e1 = TileD<2, 3, 4, 2, 2, 2, true, 1>;
using D8_256x256_8w_e1 = TileD<4, 2, 2, 4, 2, 2, true, 1>;
using D8_256x256_8w_e2 = TileD<4, 2, 2, 4, 2, 2, true, 2>;
using D8_256x192_4w_e2 = TileD<4, 3, 2, 2, 2, 1, true, 2>;
using D8_64x64_s4 = TileD<1, 1, 2, 2, 4, 4>;
using D4_128x128_4w = TileD<2, 2, 2, 2, 2, 2, true, 0, true>;
//                                                       SA                  SB
using D8_256x192_8w_a3b2 = TileD<2, 3, 4, 2, 3, 2, true, 1, false, 2>;
using D8_256x192_8w_a2b3 = TileD<2, 3, 4, 2, 2, 2, true, 1, false, 3>;
using D8_256x256_8w_a3b2 = TileD<4, 2, 2, 4, 3, 2, true, 1, false, 2>;
using D8_128x128_a3b2 = TileD<2, 2, 2, 2, 3, 2, true, 0, false, 2>;
using D8_128x128_a3b2_e1 = TileD<2, 2, 2, 2, 3, 2, true, 1, false, 2>;
using D8_128x128_s2_e1 = TileD<2, 2, 2, 2, 2, 2, true, 1>;
//                                                                               persistent
using P8_128x128_a3b2 = TileD<2, 2, 2, 2, 3, 2, true, 1, false, 2, true>;
using P8_128x192_s2 = TileD<2, 3, 2, 2, 2, 2, true, 1, false, 2, true>;
//                                                                                      FP16 operands
using H_256x192_8w = TileD<2, 3, 4, 2, 3, 2, true, 1, false, 2, false, true>;
using H_128x128_4w = TileD<2, 2, 2, 2, 3, 2, true, 1, false, 2, false, true>;
using H_64x64_4w = TileD<1, 1, 2, 2, 4, 4, true, 0, false, 4, false, true>;
using H_p192 = TileD<2, 3, 2, 2, 2, 2, true, 1, false, 2, true, true>;
using H_p128 = TileD<2, 2, 2, 2, 3, 2, true, 1, false, 2, true, true>;

static const Variant VARIANTS[] = {
    {"w8 dma 64x64 s4 4w", 8, 64, 64, 128, run_dma<D8_64x64_s4>, run_dma<D8_64x64_s4, true>},
    {"w8 dma 256x192 a3b2 8w spread1", 8, 256, 192, 128, run_dma<D8_256x192_8w_a3b2>, run_dma<D8_256x192_8w_a3b2, true>},
    {"w8 dma 128x128 a3b2 4w", 8, 128, 128, 128, run_dma<D8_128x128_a3b2>, run_dma<D8_128x128_a3b2, true>},
    {"w8 dma 128x128 a3b2 4w spread1", 8, 128, 128, 128, run_dma<D8_128x128_a3b2_e1>, run_dma<D8_128x128_a3b2_e1, true>},
    {"w8 dma 128x128 a3b2 4w spread1 persistent", 8, 128, 128, 128, run_dma<P8_128x128_a3b2>},
    {"w8 dma 128x192 s2 4w spread1 persistent", 8, 128, 192, 128, run_dma<P8_128x192_s2>},
    {"f16 dma 256x192 a3b2 8w spread1", 16, 256, 192, 64, run_dma<H_256x192_8w>, run_dma<H_256x192_8w, true>},
    {"f16 dma 128x128 a3b2 4w spread1", 16, 128, 128, 64, run_dma<H_128x128_4w>, run_dma<H_128x128_4w, true>},
    {"f16 dma 64x64 s4 4w", 16, 64, 64, 64, run_dma<H_64x64_4w>, run_dma<H_64x64_4w, true>},
    {"f16 dma 128x192 s2 4w spread1 persistent", 16, 128, 192, 64, run_dma<H_p192>},
    {"w8 128x128 bk64 4w occ3", 8, 128, 128, 64, run_variant<W8_128x128_k64_o3>, run_variant<W8_128x128_k64_o3, true>},
    {"w4 any-group 64x64 bk128 4w occ4", 4, 64, 64, 128, run_variant<W4G_64x64_k128>, run_variant<W4G_64x64_k128, true>},
    {"w4 pipelined 128x128 a3b2 4w any-group", 4, 128, 128, 128, launch_qgemm_w4, launch_qgemm_w4},
#ifdef QL_SWEEP_VARIANTS   // the other tile shapes of the sweeps that chose the ones above
    {"w8 dma 128x128 s3 4w", 8, 128, 128, 128, run_dma<D8_128x128_s3>},
    {"w8 dma 128x128 s2 4w", 8, 128, 128, 128, run_dma<D8_128x128_s2>},
    {"w8 dma 128x192 s3 4w", 8, 128, 192, 128, run_dma<D8_128x192_s3>},
    {"w8 dma 128x192 s2 4w", 8, 128, 192, 128, run_dma<D8_128x192_s2>},
    {"w8 dma 256x128 s3 4w", 8, 256, 128, 128, run_dma<D8_256x128_s3>},
    {"w8 dma 256x192 s2 4w", 8, 256, 192, 128, run_dma<D8_256x192_s2>},
    {"w8 dma 256x256 s2 8w", 8, 256, 256, 128, run_dma<D8_256x256_8w>},
    {"w8 dma 256x192 s2 8w", 8, 256, 192, 128, run_dma<D8_256x192_8w>},
    {"w8 dma 256x192 s2 8w spread1", 8, 256, 192, 128, run_dma<D8_256x192_8w_e1>},
    {"w8 dma 256x256 s2 8w spread1", 8, 256, 256, 128, run_dma<D8_256x256_8w_e1>},
    {"w8 dma 256x256 s2 8w spread2", 8, 256, 256, 128, run_dma<D8_256x256_8w_e2>},
    {"w8 dma 256x192 s2 4w spread2", 8, 256, 192, 128, run_dma<D8_256x192_4w_e2>},
    {"w4 dma 128x128 s2 4w", 4, 128, 128, 128, run_dma<D4_128x128_4w>},
    {"w8 dma 256x192 a2b3 8w spread1", 8, 256, 192, 128, run_dma<D8_256x192_8w_a2b3>},
    {"w8 dma 256x256 a3b2 8w spread1", 8, 256, 256, 128, run_dma<D8_256x256_8w_a3b2>},
    {"w8 dma 128x128 s2 4w spread1", 8, 128, 128, 128, run_dma<D8_128x128_s2_e1>},
    {"f16 dma 128x128 a3b2 4w spread1 persistent", 16, 128, 128, 64, run_dma<H_p128>},
    {"w8 128x128 bk64 4w occ2", 8, 128, 128, 64, run_variant<W8_128x128_k64>},
    {"w8 128x128 bk128 4w occ2", 8, 128, 128, 128, run_variant<W8_128x128_k128>},
    {"w8 256x128 bk64 4w occ2", 8, 256, 128, 64, run_variant<W8_256x128_k64>},
    {"w8 256x128 bk128 4w occ2", 8, 256, 128, 128, run_variant<W8_256x128_k128>},
    {"w8 128x192 bk64 4w occ2", 8, 128, 192, 64, run_variant<W8_128x192_k64>},
    {"w8 256x192 bk64 4w occ1", 8, 256, 192, 64, run_variant<W8_256x192_k64>},
    {"w8 256x256 bk64 8w occ2", 8, 256, 256, 64, run_variant<W8_256x256_8w>},
    {"w8 64x64 bk64 4w occ4", 8, 64, 64, 64, run_variant<W8_64x64_k64>},
    {"w4 128x128 bk128 4w occ2", 4, 128, 128, 128, run_variant<W4_128x128_k128>},
    {"w4 64x128 bk128 4w occ2", 4, 64, 128, 128, run_variant<W4_64x128_k128>},
    {"w4 256x128 bk128 8w occ2", 4, 256, 128, 128, run_variant<W4_256x128_8w>},
    {"w4 128x64 bk128 4w occ3", 4, 128, 64, 128, run_variant<W4_128x64_k128>},
    {"w4 any-group 128x64 bk128 4w occ3", 4, 128, 64, 128, run_variant<W4G_128x64_k128>, run_variant<W4G_128x64_k128, true>},
    {"w4 any-group 128x128 bk128 4w occ2", 4, 128, 128, 128, run_variant<W4G_128x128_k128>},
    {"w4 any-group 64x128 bk128 4w occ3", 4, 64, 128, 128, run_variant<W4G_64x128_k128>},
#endif
};
constexpr int NUM_VARIANTS = sizeof(VARIANTS) / sizeof(VARIANTS[0]);

int num_gemm_variants() { return NUM_VARIANTS; }
const char *gemm_variant_name(int v) { return (v >= 0 && v < NUM_VARIANTS) ? VARIANTS[v].name : "naive (any shape)"; }

static int find_variant(const char *name)
{
    for (int v = 0; v < NUM_VARIANTS; ++v)
        if (__builtin_strcmp(VARIANTS[v].name, name) == 0) return v;
    return 0;
}

// Tile choice by shape, from sweeps over the DiT-XL/2 layer shapes on MI355X (256 CUs).
static int choose_variant(const GemmArgs &a)
{
    static const int w8_small = find_variant("w8 dma 64x64 s4 4w"),
                     w8_mid = find_variant("w8 dma 128x128 a3b2 4w spread1"),
                     w8_mid_deep = find_variant("w8 dma 128x128 a3b2 4w"),
                     w8_p128 = find_variant("w8 dma 128x128 a3b2 4w spread1 persistent"),
                     w8_p192 = find_variant("w8 dma 128x192 s2 4w spread1 persistent"),
                     w8_big = find_variant("w8 dma 256x192 a3b2 8w spread1"),
                     w8_k64 = find_variant("w8 128x128 bk64 4w occ3"), w4_any = find_variant("w4 any-group 64x64 bk128 4w occ4");
    // the register-staged kernel hides the per-group VALU work best at high occupancy (64x64 tiles, 5 workgroups per CU);
    // its any-group form, whose four K slices share one copy of the loop body, is also the fastest at group 128
    if (a.w_bits == 16) {
        static const int h_small = find_variant("f16 dma 64x64 s4 4w"), h_mid = find_variant("f16 dma 128x128 a3b2 4w spread1"),
                         h_big = find_variant("f16 dma 256x192 a3b2 8w spread1"),
                         h_p192 = find_variant("f16 dma 128x192 s2 4w spread1 persistent");
        if (a.M <= 512) return h_small;
        if ((long)((a.M + 255) / 256) * ((a.N + 191) / 192) < 192) return h_mid;
        return (a.M >= 4096 && a.N < 4096) ? h_p192 : h_big;
    }
    // 4-bit weights: the pipelined kernel where the tile's group scales fit its LDS table and the rows fill tiles
    if (a.w_bits == 4) {
        static const int w4_pipe = find_variant("w4 pipelined 128x128 a3b2 4w any-group");
        return (qgemm_w4_takes(a) && a.M > 256) ? w4_pipe : w4_any;
    }
    if (a.K % 128 != 0) return w8_k64;
    if (a.M <= 512) return w8_small;
    const long tiles_big = (long)((a.M + 255) / 256) * ((a.N + 191) / 192);
    if (tiles_big >= 192) {                                   // enough work for every CU
        // Several tiles per CU: two resident 4-wavefront workgroups per CU that walk their tiles and fetch the next
        // tile's first K step under the epilogue.  128x192 tiles move less data per MAC; 128x128 tiles balance better
        // when the tiles per CU are few and N is wide.
        if (a.M >= 4096) return (a.K >= 2304 || a.N <= 1536 || a.M >= 12288) ? w8_p192 : w8_p128;
        return w8_big;
    }
    return a.K >= 2304 ? w8_mid_deep : w8_mid;
}

static bool is_any_group(int v) { return __builtin_strstr(VARIANTS[v].name, "any-group") != nullptr; }

hipError_t launch_qgemm(const GemmArgs &a, int variant, hipStream_t stream)
{
    if (a.w_grouped || a.s_ag) {
        // plan-space generality: the pipelined grouped kernel where it takes the shape, else one thread per element
        if (variant < NUM_VARIANTS && qgemm_w4_takes(a) && !(a.act != 0 || a.residual != nullptr || a.gate != nullptr || a.row_absmax != nullptr))
            return launch_qgemm_w4(a, stream);
        hipLaunchKernelGGL(qgemm_naive, dim3((a.M + 3) / 4, (a.N + 63) / 64), dim3(256), 0, stream, a);
        return hipGetLastError();
    }
    // MFMA tiles need 16-byte loads along K and a whole number of K steps
    const bool fast = (a.K % 64 == 0) && ((uintptr_t)a.q % 16 == 0) && ((uintptr_t)a.w % 16 == 0) &&
                      (a.w_bits != 4 || (a.K % 128 == 0 && a.group % 32 == 0));
    if (!fast || variant >= NUM_VARIANTS) {
        hipLaunchKernelGGL(qgemm_naive, dim3((a.M + 3) / 4, (a.N + 63) / 64), dim3(256), 0, stream, a);
        return hipGetLastError();
    }
    int v = variant;
    if (v < 0 || VARIANTS[v].w_bits != a.w_bits || a.K % VARIANTS[v].BK != 0) v = choose_variant(a);
    if (a.w_bits == 4) {
        // group sizes other than 128 run on the variants that end a group at any 32-wide K slice
        static const int any_group = find_variant("w4 any-group 64x64 bk128 4w occ4");
        if (a.group != 128 && !is_any_group(v)) v = any_group;
        if (__builtin_strstr(VARIANTS[v].name, "w4 pipelined") && !qgemm_w4_takes(a)) v = any_group;
        // the pipelined 4-bit kernel keeps the group scales of a tile in LDS: at most 40 groups (K <= 5120)
        if (a.K > 128 * 40 && __builtin_strncmp(VARIANTS[v].name, "w4 dma", 6) == 0)
            v = find_variant("w4 128x64 bk128 4w occ3");
    }
    if (a.act != 0 || a.residual != nullptr || a.gate != nullptr || a.row_absmax != nullptr) {
        // block glue in the epilogue: only the shape-chosen tiles carry it
        if (!VARIANTS[v].run_glue) v = choose_variant(a);
        // the prefetched gate and residual pieces need registers the persistent tiles do not have left
        // (256x192 and two resident 128x128 workgroups per CU measure alike here: 495 and 491 us for a block at M = 16384)
        static const int big = find_variant("w8 dma 256x192 a3b2 8w spread1"), hbig = find_variant("f16 dma 256x192 a3b2 8w spread1");
        if (__builtin_strstr(VARIANTS[v].name, "persistent")) v = a.w_bits == 16 ? hbig : big;
        return VARIANTS[v].run_glue(a, stream);
    }
    return VARIANTS[v].run(a, stream);
}

}  // namespace ql
