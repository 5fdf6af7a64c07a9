// INT8 x INT4 -> INT32 GEMM with group-wise weight scales for gfx950 (CDNA4): the 4-bit layers of the bit plan
// (Step 2: integer weights with one scale per group of input channels; Algorithm 2 Phase B runs them with 8-bit
// dynamic activations).
//
//   P[m,g,n] = sum_{k in group g} q[m,k] * w4[n,k]              v_mfma_i32_32x32x32_i8, nibbles fed as value * 16
//   f        = fma(float(P[m,g,n]), s_w[n,g], f)                 g ascending, fp32
//   y[m,n]   = fp16(fma(f, alpha[m/R], bias[n]))
//
// A workgroup owns a 128x128 (4 wavefronts) or 256x128 (8 wavefronts) tile; every wavefront a 64x64 block of it as
// 2x2 MFMA tiles.  Both operands go global -> LDS by DMA (global_load_lds_dwordx4) through rings of their own: one
// K step is 128 k = 128 bytes per activation row and 64 bytes per packed weight row.  The launch is persistent: as
// many workgroups as the chip holds walk their XCD's tiles, and the first K step of the next tile is requested before
// the epilogue of the current one.
//
// The per-group work is what bounds this kernel: 16 conversions and 16 multiply-adds per 32x32 tile and group on the
// vector ALU against group/32 MFMAs on the matrix cores.  It is placed where the matrix cores stay busy: the partial
// sums of tile (i,j) are folded right before that tile's first MFMA of the next group, which then starts from a zero
// C operand (no clearing pass), while the MFMAs of the other tiles and of the SIMD's second wavefront execute.  The
// nibble unpacking (6 ALU operations per 16-byte operand) is done once per pair of MFMAs, directly before them, on
// words that were read from LDS one quarter of a K step earlier.
#include "qgemm_common.h"

namespace ql {

typedef __attribute__((address_space(3))) void lds_void_w4;

// WGM_: wavefront rows of the workgroup (2: 128x128 tile, 4: 256x128); SA_/SB_: ring depths of the two operands
// B8_: the weight operand is int8 codes (128 bytes per row and K step) instead of packed nibbles
// MAXG_: weight groups along K whose scales the tile keeps in LDS (40: two workgroups per CU; more: one)
template <int WGM_, int SA_, int SB_, bool B8_ = false, int MAXG_ = 40>
struct TileW4 {
    static constexpr bool B8 = B8_;
    static constexpr int TM = 2, TN = 2, WGM = WGM_, WGN = 2;
    static constexpr int NW = WGM * WGN, NT = NW * 64;
    static constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    static constexpr int SA = SA_, SB = SB_;
    // 1024-byte DMA groups per K step: 8 activation rows x 128 B, 16 packed weight rows x 64 B
    static constexpr int A_GROUPS = BM / 8, B_GROUPS = B8 ? BN / 8 : BN / 16;
    static constexpr int NA = A_GROUPS / NW, NB = B_GROUPS / NW;
    static constexpr int A_BYTES = A_GROUPS * 1024, B_BYTES = B_GROUPS * 1024;
    static constexpr int B_RING = SA * A_BYTES;
    static constexpr int RINGS = SA * A_BYTES + SB * B_BYTES;
    // the epilogue's scratch (row scales, one 32-row strip per wavefront) lives beside stage 0 of the activation ring,
    // which by then receives the next tile's first K step
    static constexpr int EPI_OFF = A_BYTES;
    static constexpr int STRIP_OFF = (BM * 4 + 255) / 256 * 256;
    static constexpr int STRIP_BYTES = 32 * (TN * 64 + 16);
    static constexpr int EPI_BYTES = STRIP_OFF + NW * STRIP_BYTES;
    // group scales of the tile's columns, [column][group] fp16 as in global memory
    static constexpr int MAX_GROUPS = MAXG_;
    static constexpr int SCALE_OFF = RINGS;
    static constexpr int LDS_BYTES = RINGS + BN * MAX_GROUPS * 2;
    static constexpr int SMAX = SA > SB ? SA : SB;
    // loads that may still be in flight when K step 0 is first read, and at the hand-over from step kt to kt+1
    static constexpr int WAIT_START = (SA - 1) * NA + (SB - 1) * NB;
    static constexpr int WAIT_HAND = SA > SB ? NA + (SB - 2) * (NA + NB) : SA < SB ? NB + (SA - 2) * (NA + NB) : (SA - 2) * (NA + NB);
    static_assert(A_GROUPS % NW == 0 && B_GROUPS % NW == 0, "every wavefront issues the same number of DMA instructions");
    static_assert(SA >= 2 && SB >= 2 && (SA - SB) * (SA - SB) <= 1, "ring depths differ by at most one");
    static_assert((SA - 1) * A_BYTES >= EPI_BYTES, "epilogue scratch beside stage 0");
    static_assert(NA + NB <= 9, "the loads of a refill window are issued behind the MFMAs of three quarters");
    static_assert(WAIT_START <= 63, "vmcnt is a 6-bit counter");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
    static_assert(BM <= NT, "one row scale per thread");
};

// One DMA instruction, buffer form: 64 lanes x 16 bytes from base + lane_off + step_off to the 1024 bytes at lds.  The
// descriptor and the K-step offset live in scalar registers and the lane's fixed offset in one vector register, so that
// issuing a load costs no vector ALU work; reads past `bytes` return zero.
__device__ __forceinline__ void dma16_w4(const void *base, int bytes, unsigned char *lds, unsigned lane_off, int step_off)
{
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_w4 *)lds, 16, lane_off, step_off, 0, 0);
}

// int8 value * 16 of the 16 nibbles of two packed words: byte b of a word holds k = b (low nibble) and k = 4 + b (high)
__device__ __forceinline__ v4i unpack_w4(v2i p)
{
    return v4i{(int)(((unsigned)p[0] << 4) & 0xf0f0f0f0u), (int)((unsigned)p[0] & 0xf0f0f0f0u),
               (int)(((unsigned)p[1] << 4) & 0xf0f0f0f0u), (int)((unsigned)p[1] & 0xf0f0f0f0u)};
}

template <class F, int... S>
__device__ __forceinline__ void unrolled_steps(F &f, int kt, std::integer_sequence<int, S...>)
{
    (f(std::integral_constant<int, S>{}, kt + S), ...);
}

// QGF: 32-wide K slices per weight group when fixed at compile time (4 = groups of 128, 9 = groups of 288, ...): the quarters
// that open a group are then known statically over a period of lcm(QGF, 4) slices, which is unrolled; 0 = read from the
// arguments, one uniform branch per MFMA
// EXPORT: the int32 group partial sums are also written to a.acc_out
template <class T, int QGF, bool EXPORT, bool GLUE>
__global__ __launch_bounds__(T::NT, 2) void qgemm_w4(GemmArgs a, int tiles_m, int tiles_n, int nblk_padded, int group_m)
{
    constexpr int TM = T::TM, TN = T::TN, BM = T::BM, BN = T::BN, NT = T::NT, NW = T::NW;
    constexpr int SA = T::SA, SB = T::SB, NA = T::NA, NB = T::NB;
    constexpr bool B8 = T::B8;
    typedef typename std::conditional<B8, v4i, v2i>::type bfrag_t;   // a lane's weight fragment as read from LDS
    extern __shared__ __align__(1024) unsigned char smem[];

    // Workgroup ids go round-robin over the XCDs; each XCD owns per_xcd consecutive logical tiles and its resident
    // workgroups take them in order, gridDim.x / XCDS at a time.
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
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / T::WGN, wn = wave % T::WGN;
    const int M = a.M, N = a.N, K = a.K;
    const int nk = K / 128;
    const int QG = QGF ? QGF : a.group / 32;   // K slices per weight group
    const int G = K / (32 * QG);
    const unsigned short *gsw = static_cast<const unsigned short *>(a.s_w);
    unsigned short *sScale = reinterpret_cast<unsigned short *>(smem + T::SCALE_OFF);

    // DMA addressing: lane l of a wavefront fills bytes [16 l, 16 l + 16) of a 1024-byte group.  Activations: row l/8,
    // slot l%8, chunk c of row r kept at slot c ^ ((r >> 1) & 7).  Packed weights: row l/4, slot l%4, chunk c of row r
    // at slot c ^ ((r >> 2) & 3).  Wavefront w takes groups w, w+NW, ... of both operands.
    unsigned goffA[NA], goffB[NB];
    auto set_goff = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int row = 8 * (wave + i * NW) + (lane >> 3);
            const int c = (lane & 7) ^ ((row >> 1) & 7);
            goffA[i] = (unsigned)(min(m0 + row, M - 1) * K + 16 * c);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if (B8) {
                const int row = 8 * (wave + i * NW) + (lane >> 3);
                const int c = (lane & 7) ^ ((row >> 1) & 7);
                goffB[i] = (unsigned)(min(n0 + row, N - 1) * K + 16 * c);
            } else {
                const int row = 16 * (wave + i * NW) + (lane >> 2);
                const int c = (lane & 3) ^ ((row >> 2) & 3);
                goffB[i] = (unsigned)(min(n0 + row, N - 1) * (K / 2) + 16 * c);
            }
        }
    };
    set_goff();
    auto issue_a = [&](int kt, int slot, int i) {
        dma16_w4(a.q, M * K, smem + slot * T::A_BYTES + (wave + i * NW) * 1024, goffA[i], kt * 128);
    };
    auto issue_b = [&](int kt, int slot, int i) {
        dma16_w4(a.w, B8 ? N * K : N * (K / 2), smem + T::B_RING + slot * T::B_BYTES + (wave + i * NW) * 1024, goffB[i], kt * (B8 ? 128 : 64));
    };
    // Refill window j = the loads issued after the hand-over barrier of K step j, into the slots that step used:
    // weight tile of step j+SB and activation tile of step j+SA; the operand with the shallower ring goes first.
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
    auto issue_step0 = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) issue_a(0, 0, i);
#pragma unroll
        for (int i = 0; i < NB; ++i) issue_b(0, 0, i);
    };

    // fragment of a lane: row (lane & 31) of a 32-row tile, 16 k starting at 32 * quarter + 16 * (lane >> 5)
    const int frag_row = lane & 31, frag_half = lane >> 5;
    const int key = (lane >> 1) & 7, key4 = (lane >> 2) & 3;
    const int a_off = (wm * TM * 32 + frag_row) * 128;
    const int b_off = B8 ? T::B_RING + (wn * TN * 32 + frag_row) * 128 : T::B_RING + (wn * TN * 32 + frag_row) * 64 + frag_half * 8;
    auto read_frags = [&](int sl_a, int sl_b, int quarter, v4i(&af)[TM], bfrag_t(&bp)[TN]) {
        const unsigned char *st = smem + sl_a * T::A_BYTES + a_off + ((2 * quarter + frag_half) ^ key) * 16;
        const unsigned char *stb = smem + sl_b * T::B_BYTES + b_off + (B8 ? ((2 * quarter + frag_half) ^ key) : (quarter ^ key4)) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const v4i *>(st + i * 32 * 128);
#pragma unroll
        for (int j = 0; j < TN; ++j) bp[j] = *reinterpret_cast<const bfrag_t *>(stb + j * 32 * (B8 ? 128 : 64));
    };
    // the MFMA operand of a fragment: int8 codes as they are, nibbles as value * 16
    auto operand = [&](const bfrag_t &p) {
        if constexpr (B8) return p;
        else return unpack_w4(p);
    };

    v16i acc[TM][TN];
    float fsum[TM][TN][16];
    float s16[TN];        // scale / 16 of the group whose partial sums are in acc (the nibbles are used as value * 16)
    int grp_acc, grp_next, qs;   // group in acc (-1: none yet), next group to start, K slice inside the current group

    // one tile's partial sums of the finished group -> fp32 sum
    auto fold_tile = [&](int i, int j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (EXPORT) {
                const int m = m0 + wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                const int n = n0 + wn * TN * 32 + j * 32 + frag_row;
                if (grp_acc >= 0 && m < M && n < N) a.acc_out[(unsigned)((m * G + grp_acc) * N + n)] = B8 ? acc[i][j][r] : acc[i][j][r] >> 4;
            }
            fsum[i][j][r] = __builtin_fmaf((float)acc[i][j][r], s16[j], fsum[i][j][r]);
        }
    };
    // MFMA number idx of a quarter: tiles in the order (0,0) (1,0) (0,1) (1,1), so that two consecutive MFMAs share one
    // unpacked weight operand.      // restart: a compile-time tag (groups of 128: every K step opens one) or a wavefront-uniform flag.
    auto mma_one = [&](auto restart, const v4i(&af)[TM], const v4i &bf, int idx) {
        const int i = idx & 1, j = idx >> 1;
        if (restart) {
            // The fold must be complete before the MFMA overwrites the tile's accumulators in place.  Left to itself the
            // compiler sinks the fold to the end of the K step and starts the MFMAs into a second set of 64 registers,
            // which the budget does not have: the empty statement below makes the MFMA's operand depend on the folded sums.
            fold_tile(i, j);
            v4i a_dep = af[i];
            float(&f)[16] = fsum[i][j];
            asm volatile("" : "+v"(a_dep), "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]),
                         "+v"(f[8]), "+v"(f[9]), "+v"(f[10]), "+v"(f[11]), "+v"(f[12]), "+v"(f[13]), "+v"(f[14]), "+v"(f[15]));
            const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a_dep, bf, zero, 0, 0, 0);
        } else {
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf, acc[i][j], 0, 0, 0);
        }
    };
    // first MFMA of a quarter (the reads of the next quarter's fragments follow it)
    auto quarter_head = [&](auto restart_tag, const v4i(&af)[TM], const bfrag_t(&bp)[TN], v4i &bf0) {
        bf0 = operand(bp[0]);
        mma_one(restart_tag, af, bf0, 0);
    };
    // MFMAs 1..3 of a quarter, one DMA instruction of refill window `win` behind each (loads i0, i0+1, i0+2)
    auto quarter_tail = [&](auto restart_tag, const v4i(&af)[TM], const bfrag_t(&bp)[TN], const v4i &bf0, bool on, int win, int slot_a,
                            int slot_b, int i0) {
        const v4i bf1 = operand(bp[1]);
#pragma unroll
        for (int idx = 1; idx < 4; ++idx) {
            mma_one(restart_tag, af, idx < 2 ? bf0 : bf1, idx);
            const int li = i0 + idx - 1;
            if (li < NA + NB) {
                if (on) issue_win(win, slot_a, slot_b, li);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // bookkeeping of a quarter that opens a group: the scale of the new group is requested from LDS (needed at the next fold)
    auto open_group = [&]() {
        grp_acc = grp_next;
#pragma unroll
        for (int j = 0; j < TN; ++j) s16[j] = half_to_float_dev(sScale[(wn * TN * 32 + j * 32 + frag_row) * G + grp_next]) * (B8 ? 1.0f : 0.0625f);
        if (a.s_ag) {
            // one activation scale per scale block and channel group (eq. (4)): the tile lies inside one scale block
            // (the dispatcher sends R % BM == 0 only), so the scale is wavefront-uniform and joins the group's weight scale
            const float alpha_g = a.s_ag[(size_t)(m0 / a.R) * G + grp_next];
#pragma unroll
            for (int j = 0; j < TN; ++j) s16[j] *= alpha_g;
        }
        ++grp_next;
    };

    // does quarter Q of step S of the period open a weight group?  (compile-time group sizes only)
    auto restart_at = [](auto s_tag, auto q_tag) {
        return std::integral_constant<bool, QGF != 0 && (4 * decltype(s_tag)::value + decltype(q_tag)::value) % (QGF ? QGF : 1) == 0>{};
    };

    float sa_pre, bj[TN];
    issue_step0();
    for (;;) {   // one pass per tile
        // ---- per tile: row scale of one tile row per thread, bias of this lane's columns, group scales of the tile's columns
        sa_pre = (tid < BM && !a.s_ag) ? a.s_a[min(m0 + tid, M - 1) / a.R] : 1.0f;
        {
            const unsigned short *bias_h = static_cast<const unsigned short *>(a.bias);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bj[j] = bias_h ? half_to_float_dev(bias_h[min(n0 + wn * TN * 32 + j * 32 + frag_row, N - 1)]) : 0.0f;
        }
        if (n0 + BN <= N && ((reinterpret_cast<uintptr_t>(gsw) + (size_t)n0 * G * 2) & 15) == 0) {
            // the tile's columns are one contiguous run of BN * G scales: BN * G / 8 pieces of 16 bytes
            const v4i *src = reinterpret_cast<const v4i *>(gsw + (size_t)n0 * G);
            for (int idx = tid; idx < BN * G / 8; idx += NT) reinterpret_cast<v4i_alias *>(sScale)[idx] = src[idx];
        } else {
            for (int n = tid % BN, g = tid / BN; g < G; g += NT / BN) sScale[n * G + g] = gsw[(size_t)min(n0 + n, N - 1) * G + g];
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    acc[i][j][r] = 0;
                    fsum[i][j][r] = 0.0f;
                }
#pragma unroll
        for (int j = 0; j < TN; ++j) s16[j] = 0.0f;
        grp_acc = -1;
        grp_next = 0;
        qs = 0;
        // ---- prologue: the later stages of both rings, in K-step order (step 0 is already on its way)
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
        v4i af0[TM], af1[TM], bfa;
        bfrag_t bp0[TN], bp1[TN];
        if (nk >= T::SMAX) wait_vm(std::integral_constant<int, T::WAIT_START>{});
        else wait_vm(std::integral_constant<int, 0>{});
        __syncthreads();   // K step 0 and the group scales are in LDS
        read_frags(0, 0, 0, af0, bp0);
        int sa = 0, sb = 0, pa = SA - 1, pb = SB - 1;   // ring slots of K step kt and of step kt-1
        // one K step; with a compile-time group size s_tag is the step's index inside the period of the restart pattern
        auto kstep = [&](auto s_tag, int kt) {
            const int na = sa + 1 == SA ? 0 : sa + 1, nb = sb + 1 == SB ? 0 : sb + 1;
            const bool refill = kt > 0;   // refill window kt-1 is still being issued during quarter 0
            // One quarter of the K step on fragments (afc, bpc): first MFMA, [hand-over], the reads of the next quarter's
            // fragments, then the other three MFMAs with the DMA instructions li = i0, i0+1, i0+2 of window `win` behind them.
            auto quarter = [&](auto restart_tag, const v4i(&afc)[TM], const bfrag_t(&bpc)[TN], auto next_read, auto hand_tag, bool on, int win,
                               int slot_a, int slot_b, int i0) {
                quarter_head(restart_tag, afc, bpc, bfa);
                __builtin_amdgcn_sched_barrier(0);
                if (decltype(hand_tag)::value) {
                    // every LDS read of this K step's slots was issued at least a quarter ago; make that explicit, then
                    // wait for step kt+1 (only loads issued after its last one may still be in flight)
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    if (kt + T::SMAX <= nk) wait_vm(std::integral_constant<int, T::WAIT_HAND>{});
                    else wait_vm(std::integral_constant<int, 0>{});
                    __builtin_amdgcn_s_barrier();
                }
                next_read();
                __builtin_amdgcn_sched_barrier(0);
                quarter_tail(restart_tag, afc, bpc, bfa, on, win, slot_a, slot_b, i0);
                __builtin_amdgcn_sched_barrier(0);
            };
            // the same with the group bookkeeping: a quarter that opens a weight group folds the finished one first
            auto step = [&](auto first_tag, const v4i(&afc)[TM], const bfrag_t(&bpc)[TN], auto next_read, auto hand_tag, bool on, int win,
                            int slot_a, int slot_b, int i0) {
                if constexpr (QGF > 0) {
                    quarter(first_tag, afc, bpc, next_read, hand_tag, on, win, slot_a, slot_b, i0);
                    if (decltype(first_tag)::value) open_group();
                } else {
                    const bool restart = qs == 0;
                    quarter(restart, afc, bpc, next_read, hand_tag, on, win, slot_a, slot_b, i0);
                    if (restart) open_group();
                    qs = qs + 1 == QG ? 0 : qs + 1;
                }
            };
            // quarter 0 (fragments 0) while reading quarter 1; the rest of refill window kt-1 goes behind its MFMAs
            step(restart_at(s_tag, std::integral_constant<int, 0>{}), af0, bp0, [&]() { read_frags(sa, sb, 1, af1, bp1); }, std::false_type{}, refill, kt - 1, pa, pb, 3);
            // quarter 1 while reading quarter 2
            step(restart_at(s_tag, std::integral_constant<int, 1>{}), af1, bp1, [&]() { read_frags(sa, sb, 2, af0, bp0); }, std::false_type{}, refill, kt - 1, pa, pb, 6);
            // quarter 2 while reading quarter 3
            step(restart_at(s_tag, std::integral_constant<int, 2>{}), af0, bp0, [&]() { read_frags(sa, sb, 3, af1, bp1); }, std::false_type{}, false, 0, 0, 0, NA + NB);
            // quarter 3: after its first MFMA the hand-over (step kt+1 must be in LDS; after the barrier this step's slots
            // can be refilled), the first fragments of step kt+1, and the first three loads of refill window kt
            step(restart_at(s_tag, std::integral_constant<int, 3>{}), af1, bp1, [&]() { if (kt + 1 < nk) read_frags(na, nb, 0, af0, bp0); }, std::true_type{}, true, kt, sa, sb, 0);
            pa = sa;
            pb = sb;
            sa = na;
            sb = nb;
        };
        if constexpr (QGF > 0) {
            // the restart pattern repeats every PERIOD K steps (lcm(QGF, 4) slices); the dispatcher sends nk % PERIOD == 0 only
            constexpr int PERIOD = QGF % 4 == 0 ? QGF / 4 : QGF % 2 == 0 ? QGF / 2 : QGF;
            for (int kt = 0; kt < nk; kt += PERIOD) unrolled_steps(kstep, kt, std::make_integer_sequence<int, PERIOD>{});
        } else {
            for (int kt = 0; kt < nk; ++kt) kstep(std::integral_constant<int, 0>{}, kt);
        }
        // the last group's partial sums
#pragma unroll
        for (int idx = 0; idx < 4; ++idx) fold_tile(idx & 1, idx >> 1);
        __syncthreads();

        // ---- the tile being written out; the workgroup moves on to its next tile first and requests that tile's first
        // K step, so that it travels while the epilogue runs
        const int em0 = m0, en0 = n0;
        in_xcd += slots_per_xcd;
        const bool has_next = in_xcd < per_xcd && xcd_first + in_xcd < tiles_m * tiles_n;
        if (has_next) {
            set_tile(xcd_first + in_xcd);
            set_goff();
            issue_step0();
        }
        float *sRow = reinterpret_cast<float *>(smem + T::EPI_OFF);
        if (tid < BM) sRow[tid] = sa_pre;
        __syncthreads();
        _Float16 *y = static_cast<_Float16 *>(a.y);
        const bool full = (em0 + BM <= M) && (en0 + BN <= N);
        const bool glue_pieces = GLUE && (a.residual || a.gate);
        const bool glue_aligned = !glue_pieces || (((reinterpret_cast<uintptr_t>(a.residual) | reinterpret_cast<uintptr_t>(a.gate)) & 15) == 0);
        if (full && (N % 8) == 0 && (reinterpret_cast<uintptr_t>(a.y) & 15) == 0 && glue_aligned) {
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
            auto emit_fast = [&](auto act_tag) {
                constexpr bool ACT = decltype(act_tag)::value;
                auto act_of = [&](float u) { return ACT ? gelu_tanh_dev(u) : u; };
                if (a.bias)
                    store_tile_staged<TM, TN, true, 32>(strip, lane, y, N, em0 + wm * TM * 32, en0 + wn * TN * 32, [&](int i, int j, int r) {
                        return act_of(__builtin_fmaf(fsum[i][j][r], sr[i * 16 + r], bj[j]));
                    }, gl);
                else
                    store_tile_staged<TM, TN, true, 32>(strip, lane, y, N, em0 + wm * TM * 32, en0 + wn * TN * 32, [&](int i, int j, int r) {
                        return act_of(fsum[i][j][r] * sr[i * 16 + r]);
                    }, gl);
            };
            if (GLUE && a.act == 1) emit_fast(std::true_type{});
            else emit_fast(std::false_type{});
        } else {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = en0 + wn * TN * 32 + j * 32 + frag_row;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = wm * TM * 32 + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                        const int m = em0 + row;
                        if (m < M && n < N) {
                            const float f = fsum[i][j][r];
                            float u = a.bias ? __builtin_fmaf(f, sRow[row], bj[j]) : f * sRow[row];
                            asm volatile("" : "+v"(u));   // keep the fp32 rounding before the fp16 one
                            const unsigned off = (unsigned)(m * N + n);
                            if (GLUE) y[off] = glue_one(a, u, m, n, GateRows(a.gate, a.gate_rows, em0, BM).of(row));
                            else y[off] = (_Float16)u;
                        }
                    }
            }
        }
        if (!has_next) break;
        __syncthreads();   // the epilogue's scratch is free again: the rest of the next prologue may overwrite it
    }
}

template <class T, int QGF, bool EXPORT, bool GLUE>
static hipError_t run_w4(const GemmArgs &a, hipStream_t s)
{
    static const hipError_t lds_opt_in = hipFuncSetAttribute(reinterpret_cast<const void *>(&qgemm_w4<T, QGF, EXPORT, GLUE>),
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (lds_opt_in != hipSuccess) return lds_opt_in;
    const int tiles_m = (a.M + T::BM - 1) / T::BM, tiles_n = (a.N + T::BN - 1) / T::BN;
    const int nblk = tiles_m * tiles_n;
    const int padded = (nblk + XCDS - 1) / XCDS * XCDS;
    // as many workgroups as the chip holds at once (LDS decides), a multiple of the XCD count
    static const int resident = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < XCDS)
            return 0;
        const int per_cu = 160 * 1024 / T::LDS_BYTES > 0 ? 160 * 1024 / T::LDS_BYTES : 1;
        return cus / XCDS * XCDS * per_cu;
    }();
    if (resident <= 0) return hipErrorInvalidDevice;
    const int grid = padded < resident ? padded : resident;
    hipLaunchKernelGGL((qgemm_w4<T, QGF, EXPORT, GLUE>), dim3(grid), dim3(T::NT), T::LDS_BYTES, s, a, tiles_m, tiles_n, padded,
                       pick_group_m(T::BM));
    return hipGetLastError();
}

// more than 40 groups (K = 4608 with groups of 32 or 64): a table of up to 144 groups, one workgroup per CU
constexpr int W4_MANY_GROUPS = 144;

bool qgemm_w4_takes(const GemmArgs &a)
{
    if (a.s_ag && (a.R % 128 != 0 || a.M % a.R != 0)) return false;   // channel-group activation scales: tiles inside one scale block
    if (a.w_grouped)
        return a.w_bits == 8 && a.K % 128 == 0 && a.group % 32 == 0 && a.K % a.group == 0 && a.K / a.group <= TileW4<2, 3, 2>::MAX_GROUPS &&
               (uintptr_t)a.q % 16 == 0 && (uintptr_t)a.w % 16 == 0;
    return a.w_bits == 4 && a.K % 128 == 0 && a.group % 32 == 0 && a.K % a.group == 0 && a.K / a.group <= W4_MANY_GROUPS &&
           (uintptr_t)a.q % 16 == 0 && (uintptr_t)a.w % 16 == 0;
}

hipError_t launch_qgemm_w4(const GemmArgs &a, hipStream_t stream)
{
    using T = TileW4<2, 3, 2>;
    const bool glue = a.act != 0 || a.residual != nullptr || a.gate != nullptr || a.row_absmax != nullptr;
    if (a.w_grouped) {
        // int8 codes with group scales: one workgroup per CU (the weight ring is twice as large)
        using T8 = TileW4<2, 3, 2, true>;
        if (glue) return hipErrorInvalidValue;
        return a.acc_out ? run_w4<T8, 0, true, false>(a, stream) : run_w4<T8, 0, false, false>(a, stream);
    }
    if (a.K / a.group > T::MAX_GROUPS) {
        using TG = TileW4<2, 3, 2, false, W4_MANY_GROUPS>;
        if (a.acc_out) return run_w4<TG, 0, true, true>(a, stream);
        if (glue) return run_w4<TG, 0, false, true>(a, stream);
        if (a.group == 32) return run_w4<TG, 1, false, false>(a, stream);
        if (a.group == 64) return run_w4<TG, 2, false, false>(a, stream);
        return run_w4<TG, 0, false, false>(a, stream);
    }
    if (a.acc_out) return run_w4<T, 0, true, true>(a, stream);   // verification: group partial sums exported
    if (glue) return a.group == 128 ? run_w4<T, 4, false, true>(a, stream) : run_w4<T, 0, false, true>(a, stream);
    // the group set of Algorithm 1 (32, 64, 128, 192, 288) with the restart pattern unrolled, when K holds whole periods of it
    const int nk = a.K / 128;
    switch (a.group) {
    case 32: return run_w4<T, 1, false, false>(a, stream);
    case 64: return run_w4<T, 2, false, false>(a, stream);
    case 128: return run_w4<T, 4, false, false>(a, stream);
    case 192: if (nk % 3 == 0) return run_w4<T, 6, false, false>(a, stream); break;
    case 288: if (nk % 9 == 0) return run_w4<T, 9, false, false>(a, stream); break;
    default: break;
    }
    return run_w4<T, 0, false, false>(a, stream);
}

// Pair order (byte i of a row: k = 2i low nibble, k = 2i+1 high nibble) -> the storage order unpack_w4 reads (byte j of a
// 4-byte block: k = 8b+j low, k = 8b+4+j high).  One thread per 4-byte block; `blocks` = N*K/8.
__global__ __launch_bounds__(256) void prepack_w4_pairs(const unsigned *__restrict__ pairs, unsigned *__restrict__ packed, long long blocks)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= blocks) return;
    const unsigned s = pairs[i];                       // nibble t (bits 4t..4t+3) holds k = 8b+t
    unsigned d = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) d |= (((s >> (4 * j)) & 0xfu) | (((s >> (4 * (4 + j))) & 0xfu) << 4)) << (8 * j);
    packed[i] = d;
}

hipError_t launch_prepack_w4(const void *pairs, void *packed, long long blocks, hipStream_t stream)
{
    hipLaunchKernelGGL(prepack_w4_pairs, dim3((unsigned)((blocks + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const unsigned *>(pairs), static_cast<unsigned *>(packed), blocks);
    return hipGetLastError();
}

}  // namespace ql
