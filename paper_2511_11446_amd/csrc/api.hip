// Host side of the C ABI declared in include/diffpro_qlinear.h: argument
// validation (always before the first HIP call), workspace carving, kernel
// dispatch, and the plan runner (Algorithm 2, Phase B restricted to the
// quantized linears).
#include "../../include/diffpro_qlinear.h"
#include "ql_internal.h"

#include <atomic>
#include <new>
#include <vector>

// Scratch of the allocation-free entry point (qlinear_w8a8_noalloc): one array per GPU the library runs on, held until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address it yields is
// what kernels and launches receive.
#define QL_NOALLOC_SCRATCH_BYTES (24u << 20)
static __device__ __align__(256) unsigned char scratch[QL_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local int g_last_device_error = 0;
std::atomic<int> g_gemm_variant{-1};

constexpr int64_t K_MAX = 133143;          // 133143 * 127 * 127 < 2^31
constexpr int64_t ELEMS_MAX = 2147483647;  // int32 indexing inside the kernels
constexpr int64_t W4_GROUP_MAX = 132096;   // largest multiple of 32 with 127 * 8 * 16 * group < 2^31

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int device_status(hipError_t e)
{
    if (e == hipSuccess) return QL_OK;
    g_last_device_error = (int)e;
    return QL_ERR_DEVICE;
}

int check_shape(int64_t M, int64_t K, int64_t R, int64_t N)
{
    if (M < 1 || K < 1 || N < 1 || R < 1) return QL_ERR_SHAPE;
    if (K > K_MAX || M % R != 0) return QL_ERR_SHAPE;
    if (M > ELEMS_MAX / K || M > ELEMS_MAX / N || N > ELEMS_MAX / K) return QL_ERR_SHAPE;
    return QL_OK;
}

inline bool misaligned(const void *p, size_t a) { return p && ((uintptr_t)p % a) != 0; }

// DAQ scratch for R > 1.  Absmax: [block maxima M/R][partial maxima (M/R) * parts]; percentile: [tau patterns M/R]
// [selection histograms (M/R) * DAQ_ROBUST_WORDS].  One size covers both, so a workspace serves either mode.
size_t daq_scratch_bytes(int64_t M, int64_t K, int64_t R)
{
    if (M < 1 || R <= 1 || M % R != 0) return 0;
    const size_t nblk = (size_t)(M / R);
    const size_t plain = align_up(nblk * ql::daq_parts_per_block(K, R) * 4, 256);
    const size_t robust = align_up(nblk * ql::DAQ_ROBUST_WORDS * 4, 256);
    return align_up(nblk * 4, 256) + (plain > robust ? plain : robust);
}

// eq. (4): rank from the top of the nearest-rank percentile, c = n - ceil(n p) + 1 with n = R*K values per scale block
int robust_args(const ql_daq_params *dp, int64_t K, int64_t R, ql::DaqArgs &d)
{
    if (dp->p_ppm < 1 || dp->p_ppm > 1000000 || dp->a_bits < 2 || dp->a_bits > 8) return QL_ERR_UNSUPPORTED;
    const int64_t n = R * K;
    if (n > (int64_t)1 << 31) return QL_ERR_SHAPE;
    int64_t k = (n * (int64_t)dp->p_ppm + 999999) / 1000000;
    if (k < 1) k = 1;
    if (k > n) k = n;
    d.top_rank = (unsigned)(n - k + 1);
    d.qmax = (1 << (dp->a_bits - 1)) - 1;
    return QL_OK;
}

// workspace layout of one layer: [codes M*K][scales M/R][DAQ scratch (R > 1)]
struct LayerWs {
    size_t q_off, s_off, bm_off, total;
};

LayerWs layer_ws(int64_t M, int64_t K, int64_t R)
{
    LayerWs w;
    w.q_off = 0;
    w.s_off = align_up((size_t)(M * K), 256);
    w.bm_off = w.s_off + align_up((size_t)(M / R) * 4, 256);
    w.total = w.bm_off + daq_scratch_bytes(M, K, R);
    return w;
}

int check_workspace(void *ws, size_t have, size_t need)
{
    if (need == 0) return QL_OK;
    if (!ws || have < need) return QL_ERR_WORKSPACE;
    if ((uintptr_t)ws % 256 != 0) return QL_ERR_ALIGN;
    return QL_OK;
}

// 4-bit weight groups: a multiple of 32 that divides K (Step 2 / Algorithm 1 choose the size per layer)
int check_group(int64_t K, int64_t group)
{
    if (group < 32 || group % 32 != 0) return QL_ERR_UNSUPPORTED;
    if (K % group != 0 || K % 8 != 0) return QL_ERR_SHAPE;
    // the kernels multiply nibbles as value * 16: a group's sum of 127 * 128 * group must stay below 2^31
    if (group > W4_GROUP_MAX) return QL_ERR_SHAPE;
    return QL_OK;
}

// DAQ then GEMM for one layer; all arguments already validated
int run_layer(const void *x, int64_t M, int64_t K, int64_t R, int w_bits, const void *w, const void *w_scale,
              const void *bias, int64_t N, void *y, const ql_debug *dbg, void *workspace, hipStream_t stream,
              const ql_daq_params *dp = nullptr, int64_t group = 128, const ql_fusion *fu = nullptr)
{
    if (w_bits == 16) {
        // a layer the plan leaves in FP16: no quantization, both operands binary16
        ql::GemmArgs g{};
        g.q = static_cast<const int8_t *>(x);
        g.w = w;
        g.bias = bias;
        g.y = y;
        g.M = (int)M;
        g.N = (int)N;
        g.K = (int)K;
        g.R = 1;
        g.w_bits = 16;
        g.group = 128;
        if (fu) {
            g.act = fu->act;
            g.residual = fu->residual;
            g.gate = fu->gate;
            g.gate_rows = (int)fu->gate_rows;
            g.row_absmax = static_cast<unsigned *>(fu->row_absmax);
        }
        if (g.row_absmax) {
            const int rc = device_status(ql::launch_fill_u32(g.row_absmax, (int)M, 0u, stream));
            if (rc) return rc;
        }
        return device_status(ql::launch_qgemm(g, g_gemm_variant.load(), stream));
    }
    const LayerWs lw = layer_ws(M, K, R);
    unsigned char *base = static_cast<unsigned char *>(workspace);
    ql::DaqArgs d{};
    d.x = x;
    d.q = (dbg && dbg->q) ? static_cast<int8_t *>(dbg->q) : reinterpret_cast<int8_t *>(base + lw.q_off);
    d.scales = (dbg && dbg->a_scales) ? static_cast<float *>(dbg->a_scales) : reinterpret_cast<float *>(base + lw.s_off);
    d.blockmax = R > 1 ? reinterpret_cast<unsigned *>(base + lw.bm_off) : nullptr;
    d.partmax = R > 1 ? reinterpret_cast<unsigned *>(base + lw.bm_off + align_up((size_t)(M / R) * 4, 256)) : nullptr;
    d.hist = d.partmax;
    d.M = (int)M;
    d.K = (int)K;
    d.R = (int)R;
    int rc;
    if (dp) {
        rc = robust_args(dp, K, R, d);
        if (rc) return rc;
        rc = device_status(ql::launch_daq_robust(d, stream));
    } else {
        rc = device_status(ql::launch_daq(d, stream));
    }
    if (rc) return rc;
    ql::GemmArgs g{};
    g.q = d.q;
    g.s_a = d.scales;
    g.w = w;
    g.s_w = w_scale;
    g.bias = bias;
    g.y = y;
    g.acc_out = dbg ? static_cast<int32_t *>(dbg->acc) : nullptr;
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    g.R = (int)R;
    g.w_bits = w_bits;
    g.group = (int)group;
    if (fu) {
        g.act = fu->act;
        g.residual = fu->residual;
        g.gate = fu->gate;
        g.gate_rows = (int)fu->gate_rows;
        g.row_absmax = static_cast<unsigned *>(fu->row_absmax);
    }
    if (g.row_absmax) {
        rc = device_status(ql::launch_fill_u32(g.row_absmax, (int)M, 0u, stream));
        if (rc) return rc;
    }
    return device_status(ql::launch_qgemm(g, g_gemm_variant.load(), stream));
}

// device address of `scratch` on the current device, looked up once per device
constexpr int NOALLOC_MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[NOALLOC_MAX_DEVICES];

int noalloc_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return device_status(e);
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return QL_ERR_UNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return device_status(e);
        if (!p) return QL_ERR_DEVICE;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return QL_OK;
}

int check_fusion(const ql_fusion *fu, int64_t M)
{
    if (!fu) return QL_OK;
    if (fu->act != QL_ACT_NONE && fu->act != QL_ACT_GELU_TANH) return QL_ERR_UNSUPPORTED;
    if (misaligned(fu->residual, 2) || misaligned(fu->gate, 2) || misaligned(fu->row_absmax, 4)) return QL_ERR_ALIGN;
    if (fu->gate && (fu->gate_rows < 1 || M % fu->gate_rows != 0)) return QL_ERR_SHAPE;
    return QL_OK;
}

int check_layer_ptrs(const void *x, const void *w, const void *w_scale, const void *bias, const void *y,
                     const ql_debug *dbg, int w_bits)
{
    if (!x || !w || !w_scale || !y) return QL_ERR_NULL;
    if (misaligned(x, 2) || misaligned(y, 2) || misaligned(bias, 2)) return QL_ERR_ALIGN;
    if (misaligned(w_scale, w_bits == 8 ? 4 : 2)) return QL_ERR_ALIGN;
    if (dbg && (misaligned(dbg->a_scales, 4) || misaligned(dbg->acc, 4))) return QL_ERR_ALIGN;
    return QL_OK;
}

int qlinear_any(int w_bits, const void *x, int64_t M, int64_t K, int64_t R, const void *w, const void *w_scale,
                const void *bias, int64_t N, void *y, const ql_debug *dbg, void *workspace, size_t workspace_bytes,
                void *stream, int64_t group = 128, const ql_fusion *fu = nullptr)
{
    int rc = check_layer_ptrs(x, w, w_scale, bias, y, dbg, w_bits);
    if (rc) return rc;
    rc = check_shape(M, K, R, N);
    if (rc) return rc;
    rc = check_fusion(fu, M);
    if (rc) return rc;
    if (w_bits == 4) {
        rc = check_group(K, group);
        if (rc) return rc;
        if (M > ELEMS_MAX / N / (K / group) && dbg && dbg->acc) return QL_ERR_SHAPE;
    }
    rc = check_workspace(workspace, workspace_bytes, layer_ws(M, K, R).total);
    if (rc) return rc;
    return run_layer(x, M, K, R, w_bits, w, w_scale, bias, N, y, dbg, workspace, static_cast<hipStream_t>(stream), nullptr,
                     group, fu);
}

int qgemm_any(int w_bits, const void *q, const void *a_scales, int64_t M, int64_t K, int64_t R, const void *w,
              const void *w_scale, const void *bias, int64_t N, void *y, void *acc, void *stream, int64_t group = 128)
{
    if (!q || !a_scales || !w || !w_scale || !y) return QL_ERR_NULL;
    if (misaligned(a_scales, 4) || misaligned(y, 2) || misaligned(bias, 2) || misaligned(acc, 4) ||
        misaligned(w_scale, w_bits == 8 ? 4 : 2))
        return QL_ERR_ALIGN;
    int rc = check_shape(M, K, R, N);
    if (rc) return rc;
    if (w_bits == 4) {
        rc = check_group(K, group);
        if (rc) return rc;
        if (acc && M > ELEMS_MAX / N / (K / group)) return QL_ERR_SHAPE;
    }
    ql::GemmArgs g{};
    g.q = static_cast<const int8_t *>(q);
    g.s_a = static_cast<const float *>(a_scales);
    g.w = w;
    g.s_w = w_scale;
    g.bias = bias;
    g.y = y;
    g.acc_out = static_cast<int32_t *>(acc);
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    g.R = (int)R;
    g.w_bits = w_bits;
    g.group = (int)group;
    return device_status(ql::launch_qgemm(g, g_gemm_variant.load(), static_cast<hipStream_t>(stream)));
}

}  // namespace

struct ql_plan {
    std::vector<ql_layer_desc> layers;
    int64_t M_max;
    int64_t K_widest;
};

extern "C" {

const char *ql_status_string(int status)
{
    switch (status) {
        case QL_OK: return "QL_OK";
        case QL_ERR_NULL: return "QL_ERR_NULL";
        case QL_ERR_SHAPE: return "QL_ERR_SHAPE";
        case QL_ERR_ALIGN: return "QL_ERR_ALIGN";
        case QL_ERR_UNSUPPORTED: return "QL_ERR_UNSUPPORTED";
        case QL_ERR_WORKSPACE: return "QL_ERR_WORKSPACE";
        case QL_ERR_DEVICE: return "QL_ERR_DEVICE";
        default: return "QL_ERR_?";
    }
}

int ql_last_device_error(void) { return g_last_device_error; }

int ql_version(void) { return 1000; }

size_t daq_workspace_bytes(int64_t M, int64_t K, int64_t R)
{
    return daq_scratch_bytes(M, K, R);
}

static int daq_any(const void *x, int64_t M, int64_t K, int64_t R, const ql_daq_params *dp, void *q, void *scales,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !q || !scales) return QL_ERR_NULL;
    if (misaligned(x, 2) || misaligned(scales, 4)) return QL_ERR_ALIGN;
    int rc = check_shape(M, K, R, 1);
    if (rc) return rc;
    ql::DaqArgs d{};
    if (dp) {
        rc = robust_args(dp, K, R, d);
        if (rc) return rc;
    }
    rc = check_workspace(workspace, workspace_bytes, daq_workspace_bytes(M, K, R));
    if (rc) return rc;
    d.x = x;
    d.q = static_cast<int8_t *>(q);
    d.scales = static_cast<float *>(scales);
    d.blockmax = R > 1 ? static_cast<unsigned *>(workspace) : nullptr;
    d.partmax = R > 1 ? reinterpret_cast<unsigned *>(static_cast<unsigned char *>(workspace) + align_up((size_t)(M / R) * 4, 256))
                      : nullptr;
    d.hist = d.partmax;
    d.M = (int)M;
    d.K = (int)K;
    d.R = (int)R;
    return device_status(dp ? ql::launch_daq_robust(d, static_cast<hipStream_t>(stream))
                            : ql::launch_daq(d, static_cast<hipStream_t>(stream)));
}

int daq_quantize(const void *x, int64_t M, int64_t K, int64_t R, void *q, void *scales, void *workspace,
                 size_t workspace_bytes, void *stream)
{
    return daq_any(x, M, K, R, nullptr, q, scales, workspace, workspace_bytes, stream);
}

int daq_quantize_robust(const void *x, int64_t M, int64_t K, int64_t R, const ql_daq_params *params, void *q, void *scales,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    if (!params) return QL_ERR_NULL;
    return daq_any(x, M, K, R, params, q, scales, workspace, workspace_bytes, stream);
}

int daq_quantize_rowmax(const void *x, int64_t M, int64_t K, int64_t R, const void *row_absmax, void *q, void *scales,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !q || !scales || !row_absmax) return QL_ERR_NULL;
    if (misaligned(x, 2) || misaligned(scales, 4) || misaligned(row_absmax, 4)) return QL_ERR_ALIGN;
    int rc = check_shape(M, K, R, 1);
    if (rc) return rc;
    rc = check_workspace(workspace, workspace_bytes, daq_workspace_bytes(M, K, R));
    if (rc) return rc;
    ql::DaqArgs d{};
    d.x = x;
    d.q = static_cast<int8_t *>(q);
    d.scales = static_cast<float *>(scales);
    d.blockmax = R > 1 ? static_cast<unsigned *>(workspace) : nullptr;
    d.M = (int)M;
    d.K = (int)K;
    d.R = (int)R;
    return device_status(ql::launch_daq_from_rowmax(d, static_cast<const unsigned *>(row_absmax), static_cast<hipStream_t>(stream)));
}

// ---- plan-space generality: channel-group activation scales, int8-held codes of any width with group scales ----------
static int check_act_group(int64_t K, int64_t ag)
{
    if (ag < 8 || ag % 8 != 0) return QL_ERR_UNSUPPORTED;
    if (K % 8 != 0 || K % ag != 0 || K / ag > 1024) return QL_ERR_SHAPE;
    return QL_OK;
}

size_t daq_cg_workspace_bytes(int64_t M, int64_t K, int64_t R, int64_t act_group)
{
    if (M < 1 || K < 1 || R < 1 || M % R != 0 || act_group < 1 || K % act_group != 0) return 0;
    return align_up((size_t)(M / R) * (size_t)(K / act_group) * 4, 256);
}

int daq_quantize_cg(const void *x, int64_t M, int64_t K, int64_t R, int64_t act_group, void *q, void *scales, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    if (!x || !q || !scales) return QL_ERR_NULL;
    if (misaligned(x, 16) || misaligned(q, 8) || misaligned(scales, 4)) return QL_ERR_ALIGN;
    int rc = check_shape(M, K, R, 1);
    if (rc) return rc;
    rc = check_act_group(K, act_group);
    if (rc) return rc;
    rc = check_workspace(workspace, workspace_bytes, daq_cg_workspace_bytes(M, K, R, act_group));
    if (rc) return rc;
    ql::DaqArgs d{};
    d.x = x;
    d.q = static_cast<int8_t *>(q);
    d.scales = static_cast<float *>(scales);
    d.blockmax = static_cast<unsigned *>(workspace);
    d.M = (int)M;
    d.K = (int)K;
    d.R = (int)R;
    return device_status(ql::launch_daq_cg(d, (int)act_group, static_cast<hipStream_t>(stream)));
}

size_t qlinear_grouped_workspace_bytes(int64_t M, int64_t K, int64_t R, int64_t act_group)
{
    if (M < 1 || K < 1 || R < 1 || M % R != 0) return 0;
    if (act_group <= 0) return layer_ws(M, K, R).total;
    if (K % act_group != 0) return 0;
    return align_up((size_t)(M * K), 256) + 2 * daq_cg_workspace_bytes(M, K, R, act_group);
}

int qlinear_grouped(const void *x, int64_t M, int64_t K, int64_t R, int64_t act_group, const void *w, int32_t w_storage,
                    const void *w_scale, int64_t group, const void *bias, int64_t N, void *y, const ql_debug *dbg,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    if (w_storage != 4 && w_storage != 8) return QL_ERR_UNSUPPORTED;
    int rc = check_layer_ptrs(x, w, w_scale, bias, y, dbg, 4);
    if (rc) return rc;
    rc = check_shape(M, K, R, N);
    if (rc) return rc;
    rc = check_group(K, group);
    if (rc) return rc;
    if (act_group != 0 && act_group != group) return QL_ERR_UNSUPPORTED;   // the channel groups are the weight groups
    if (act_group != 0) {
        rc = check_act_group(K, act_group);
        if (rc) return rc;
        if (misaligned(x, 16)) return QL_ERR_ALIGN;
    }
    if (dbg && dbg->acc && M > ELEMS_MAX / N / (K / group)) return QL_ERR_SHAPE;
    rc = check_workspace(workspace, workspace_bytes, qlinear_grouped_workspace_bytes(M, K, R, act_group));
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned char *base = static_cast<unsigned char *>(workspace);
    ql::GemmArgs g{};
    if (act_group == 0) {
        const LayerWs lw = layer_ws(M, K, R);
        ql::DaqArgs d{};
        d.x = x;
        d.q = (dbg && dbg->q) ? static_cast<int8_t *>(dbg->q) : reinterpret_cast<int8_t *>(base + lw.q_off);
        d.scales = (dbg && dbg->a_scales) ? static_cast<float *>(dbg->a_scales) : reinterpret_cast<float *>(base + lw.s_off);
        d.blockmax = R > 1 ? reinterpret_cast<unsigned *>(base + lw.bm_off) : nullptr;
        d.partmax = R > 1 ? reinterpret_cast<unsigned *>(base + lw.bm_off + align_up((size_t)(M / R) * 4, 256)) : nullptr;
        d.M = (int)M;
        d.K = (int)K;
        d.R = (int)R;
        rc = device_status(ql::launch_daq(d, s));
        if (rc) return rc;
        g.q = d.q;
        g.s_a = d.scales;
    } else {
        const size_t cgb = daq_cg_workspace_bytes(M, K, R, act_group);
        ql::DaqArgs d{};
        d.x = x;
        d.q = (dbg && dbg->q) ? static_cast<int8_t *>(dbg->q) : reinterpret_cast<int8_t *>(base);
        d.scales = (dbg && dbg->a_scales) ? static_cast<float *>(dbg->a_scales) : reinterpret_cast<float *>(base + align_up((size_t)(M * K), 256));
        d.blockmax = reinterpret_cast<unsigned *>(base + align_up((size_t)(M * K), 256) + cgb);
        d.M = (int)M;
        d.K = (int)K;
        d.R = (int)R;
        rc = device_status(ql::launch_daq_cg(d, (int)act_group, s));
        if (rc) return rc;
        g.q = d.q;
        g.s_ag = d.scales;
    }
    g.w = w;
    g.s_w = w_scale;
    g.bias = bias;
    g.y = y;
    g.acc_out = dbg ? static_cast<int32_t *>(dbg->acc) : nullptr;
    g.M = (int)M;
    g.N = (int)N;
    g.K = (int)K;
    g.R = (int)R;
    g.w_bits = w_storage;
    g.w_grouped = w_storage == 8 ? 1 : 0;
    g.group = (int)group;
    return device_status(ql::launch_qgemm(g, g_gemm_variant.load(), s));
}

int ql_pack_bits_host(const int8_t *codes, int64_t N, int64_t K, int32_t bits, uint8_t *packed)
{
    if (!codes || !packed) return QL_ERR_NULL;
    if (bits < 2 || bits > 7) return QL_ERR_UNSUPPORTED;
    if (N < 1 || K < 1 || (K * bits) % 8 != 0) return QL_ERR_SHAPE;
    const int64_t row_bytes = K * bits / 8;
    const int lo = -(1 << (bits - 1)), hi = (1 << (bits - 1)) - 1;
    for (int64_t n = 0; n < N; ++n) {
        uint8_t *dst = packed + n * row_bytes;
        for (int64_t i = 0; i < row_bytes; ++i) dst[i] = 0;
        for (int64_t k = 0; k < K; ++k) {
            const int c = codes[n * K + k];
            if (c < lo || c > hi) return QL_ERR_SHAPE;
            const unsigned u = (unsigned)c & ((1u << bits) - 1);
            for (int b = 0; b < bits; ++b)
                if (u >> b & 1) dst[(k * bits + b) / 8] |= (uint8_t)(1u << ((k * bits + b) % 8));
        }
    }
    return QL_OK;
}

int ql_unpack_bits_host(const uint8_t *packed, int64_t N, int64_t K, int32_t bits, int8_t *codes)
{
    if (!codes || !packed) return QL_ERR_NULL;
    if (bits < 2 || bits > 7) return QL_ERR_UNSUPPORTED;
    if (N < 1 || K < 1 || (K * bits) % 8 != 0) return QL_ERR_SHAPE;
    const int64_t row_bytes = K * bits / 8;
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *src = packed + n * row_bytes;
        for (int64_t k = 0; k < K; ++k) {
            int u = 0;
            for (int b = 0; b < bits; ++b) u |= ((src[(k * bits + b) / 8] >> ((k * bits + b) % 8)) & 1) << b;
            codes[n * K + k] = (int8_t)(u >= (1 << (bits - 1)) ? u - (1 << bits) : u);
        }
    }
    return QL_OK;
}

int ql_zero_point_fold_host(const int8_t *codes, const int32_t *zeros, int64_t N, int64_t K, int64_t group, int8_t *out)
{
    if (!codes || !zeros || !out) return QL_ERR_NULL;
    if (N < 1 || K < 1 || group < 1 || K % group != 0) return QL_ERR_SHAPE;
    const int64_t G = K / group;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const int d = (int)codes[n * K + k] - zeros[n * G + k / group];
            if (d < -127 || d > 127) return QL_ERR_UNSUPPORTED;   // 8-bit codes with a zero point do not fit
            out[n * K + k] = (int8_t)d;
        }
    return QL_OK;
}

int daq_quantize_ln(const void *x, int64_t M, int64_t K, int64_t R, const void *shift, const void *scale, int64_t rows_per_mod,
                    float eps, void *h, void *q, void *scales, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || (!q && !h) || (q && !scales)) return QL_ERR_NULL;
    if (misaligned(x, 16) || misaligned(shift, 16) || misaligned(scale, 16) || misaligned(h, 16) || misaligned(q, 8) ||
        misaligned(scales, 4))
        return QL_ERR_ALIGN;
    int rc = check_shape(M, K, R, 1);
    if (rc) return rc;
    if (K % 8 != 0 || K > 4608 || !(eps >= 0.0f)) return QL_ERR_SHAPE;
    if ((shift || scale) && (rows_per_mod < 1 || M % rows_per_mod != 0)) return QL_ERR_SHAPE;
    if (R > 1 && q && !h) return QL_ERR_NULL;    // several rows per scale: the normalised rows are staged in h
    if (R > 1 && q) {
        rc = check_workspace(workspace, workspace_bytes, daq_workspace_bytes(M, K, R));
        if (rc) return rc;
    }
    ql::LnDaqArgs a{};
    a.x = x;
    a.shift = shift;
    a.scale = scale;
    a.h = h;
    a.q = R == 1 ? static_cast<int8_t *>(q) : nullptr;
    a.scales = static_cast<float *>(scales);
    a.M = (int)M;
    a.K = (int)K;
    a.rows_per_mod = (shift || scale) ? (int)rows_per_mod : 1;
    a.eps = eps;
    rc = device_status(ql::launch_daq_ln(a, static_cast<hipStream_t>(stream)));
    if (rc || R == 1 || !q) return rc;
    return daq_any(h, M, K, R, nullptr, q, scales, workspace, workspace_bytes, stream);
}

int ql_time_bin(int64_t step, int64_t num_steps)
{
    if (num_steps < 1 || step < 0 || step >= num_steps) return -1;
    return (int)(step * 3 / num_steps);
}

size_t qlinear_workspace_bytes(int64_t M, int64_t K, int64_t R)
{
    if (M < 1 || K < 1 || R < 1 || M % R != 0) return 0;
    return layer_ws(M, K, R).total;
}

int qlinear_w8a8(const void *x, int64_t M, int64_t K, int64_t R, const void *w, const void *w_scale,
                 const void *bias, int64_t N, void *y, const ql_debug *dbg, void *workspace, size_t workspace_bytes,
                 void *stream)
{
    return qlinear_any(8, x, M, K, R, w, w_scale, bias, N, y, dbg, workspace, workspace_bytes, stream);
}

size_t qlinear_noalloc_max_bytes(void) { return QL_NOALLOC_SCRATCH_BYTES; }

int qlinear_w8a8_noalloc(const void *x, int64_t M, int64_t K, int64_t R, const void *w, const void *w_scale,
                         const void *bias, int64_t N, void *y, void *stream)
{
    int rc = check_layer_ptrs(x, w, w_scale, bias, y, nullptr, 8);
    if (rc) return rc;
    rc = check_shape(M, K, R, N);
    if (rc) return rc;
    if (layer_ws(M, K, R).total > QL_NOALLOC_SCRATCH_BYTES) return QL_ERR_WORKSPACE;
    void *ws = nullptr;
    rc = noalloc_scratch(&ws);
    if (rc) return rc;
    // nothing in the scratch has to start at zero: codes, scales and partial maxima are written before they are read
    // (the atomic-maximum fallback of the DAQ pass clears its block maxima with a fill kernel of its own)
    return run_layer(x, M, K, R, 8, w, w_scale, bias, N, y, nullptr, ws, static_cast<hipStream_t>(stream));
}

int qlinear_w4a8(const void *x, int64_t M, int64_t K, int64_t R, const void *w4, const void *w_scale,
                 const void *bias, int64_t N, void *y, const ql_debug *dbg, void *workspace, size_t workspace_bytes,
                 void *stream)
{
    return qlinear_any(4, x, M, K, R, w4, w_scale, bias, N, y, dbg, workspace, workspace_bytes, stream);
}

int qlinear_w4a8_g(const void *x, int64_t M, int64_t K, int64_t R, const void *w4, const void *w_scale, int64_t group,
                   const void *bias, int64_t N, void *y, const ql_debug *dbg, void *workspace, size_t workspace_bytes,
                   void *stream)
{
    return qlinear_any(4, x, M, K, R, w4, w_scale, bias, N, y, dbg, workspace, workspace_bytes, stream, group);
}

int qlinear_w8a8_fused(const void *x, int64_t M, int64_t K, int64_t R, const void *w, const void *w_scale, const void *bias,
                       int64_t N, const ql_fusion *fusion, void *y, void *workspace, size_t workspace_bytes, void *stream)
{
    return qlinear_any(8, x, M, K, R, w, w_scale, bias, N, y, nullptr, workspace, workspace_bytes, stream, 128, fusion);
}

int qlinear_w4a8_fused(const void *x, int64_t M, int64_t K, int64_t R, const void *w4, const void *w_scale, int64_t group,
                       const void *bias, int64_t N, const ql_fusion *fusion, void *y, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    return qlinear_any(4, x, M, K, R, w4, w_scale, bias, N, y, nullptr, workspace, workspace_bytes, stream, group, fusion);
}

int qlinear_f16(const void *x, int64_t M, int64_t K, const void *w, const void *bias, int64_t N, const ql_fusion *fusion,
                void *y, void *stream)
{
    if (!x || !w || !y) return QL_ERR_NULL;
    if (misaligned(x, 2) || misaligned(w, 2) || misaligned(y, 2) || misaligned(bias, 2)) return QL_ERR_ALIGN;
    int rc = check_shape(M, K, 1, N);
    if (rc) return rc;
    rc = check_fusion(fusion, M);
    if (rc) return rc;
    return run_layer(x, M, K, 1, 16, w, nullptr, bias, N, y, nullptr, nullptr, static_cast<hipStream_t>(stream), nullptr, 128,
                     fusion);
}

int qgemm_w4a8_g(const void *q, const void *a_scales, int64_t M, int64_t K, int64_t R, const void *w4,
                 const void *w_scale, int64_t group, const void *bias, int64_t N, void *y, void *acc, void *stream)
{
    return qgemm_any(4, q, a_scales, M, K, R, w4, w_scale, bias, N, y, acc, stream, group);
}

int qgemm_w8a8(const void *q, const void *a_scales, int64_t M, int64_t K, int64_t R, const void *w,
               const void *w_scale, const void *bias, int64_t N, void *y, void *acc, void *stream)
{
    return qgemm_any(8, q, a_scales, M, K, R, w, w_scale, bias, N, y, acc, stream);
}

int qgemm_w4a8(const void *q, const void *a_scales, int64_t M, int64_t K, int64_t R, const void *w4,
               const void *w_scale, const void *bias, int64_t N, void *y, void *acc, void *stream)
{
    return qgemm_any(4, q, a_scales, M, K, R, w4, w_scale, bias, N, y, acc, stream);
}

int ql_pack_w4_host(const int8_t *codes, int64_t N, int64_t K, uint8_t *packed)
{
    if (!codes || !packed) return QL_ERR_NULL;
    if (N < 1 || K < 1 || K % 8 != 0) return QL_ERR_SHAPE;
    for (int64_t n = 0; n < N; ++n) {
        const int8_t *src = codes + n * K;
        uint8_t *dst = packed + n * (K / 2);
        for (int64_t blk = 0; blk < K / 8; ++blk)
            for (int j = 0; j < 4; ++j) {
                const int lo = src[8 * blk + j], hi = src[8 * blk + 4 + j];
                if (lo < -8 || lo > 7 || hi < -8 || hi > 7) return QL_ERR_SHAPE;
                dst[4 * blk + j] = (uint8_t)((lo & 0xf) | ((hi & 0xf) << 4));
            }
    }
    return QL_OK;
}

int ql_repack_w4_pairs_host(const uint8_t *pairs, int64_t N, int64_t K, uint8_t *packed)
{
    if (!pairs || !packed) return QL_ERR_NULL;
    if (pairs == packed) return QL_ERR_UNSUPPORTED;
    if (N < 1 || K < 1 || K % 8 != 0) return QL_ERR_SHAPE;
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *src = pairs + n * (K / 2);   // byte i: k = 2i in the low nibble, k = 2i+1 in the high nibble
        uint8_t *dst = packed + n * (K / 2);
        auto nib = [&](int64_t k) { return (uint8_t)((k & 1) ? (src[k / 2] >> 4) : (src[k / 2] & 0xf)); };
        for (int64_t blk = 0; blk < K / 8; ++blk)
            for (int j = 0; j < 4; ++j) dst[4 * blk + j] = (uint8_t)(nib(8 * blk + j) | (nib(8 * blk + 4 + j) << 4));
    }
    return QL_OK;
}

int ql_prepack_w4(const void *pairs, int64_t N, int64_t K, void *packed, void *stream)
{
    if (!pairs || !packed) return QL_ERR_NULL;
    if (pairs == packed) return QL_ERR_UNSUPPORTED;
    if (N < 1 || K < 1 || K % 8 != 0 || N * K / 8 > ((int64_t)1 << 31) * 256 - 256) return QL_ERR_SHAPE;
    if (misaligned(pairs, 4) || misaligned(packed, 4)) return QL_ERR_ALIGN;
    return device_status(ql::launch_prepack_w4(pairs, packed, N * K / 8, static_cast<hipStream_t>(stream)));
}

int ql_plan_create(const ql_layer_desc *layers, int32_t n_layers, int64_t M_max, ql_plan **plan_out)
{
    if (!layers || !plan_out) return QL_ERR_NULL;
    *plan_out = nullptr;
    if (n_layers < 1 || M_max < 1) return QL_ERR_SHAPE;
    int64_t widest = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        const ql_layer_desc &d = layers[l];
        if (d.w_bits != 8 && d.w_bits != 4 && d.w_bits != 16) return QL_ERR_UNSUPPORTED;
        if (d.w_bits != 4 && d.group != 0) return QL_ERR_UNSUPPORTED;
        if (!d.w || (!d.w_scale && d.w_bits != 16)) return QL_ERR_NULL;
        if (d.w_bits == 16 && misaligned(d.w, 2)) return QL_ERR_ALIGN;
        int rc = check_shape(M_max, d.K, 1, d.N);
        if (rc) return rc;
        if (d.w_bits == 4) {
            rc = check_group(d.K, d.group);
            if (rc) return rc;
        }
        if ((d.w_bits != 16 && misaligned(d.w_scale, d.w_bits == 8 ? 4 : 2)) || misaligned(d.bias, 2)) return QL_ERR_ALIGN;
        widest = d.K > widest ? d.K : widest;
    }
    ql_plan *p = new (std::nothrow) ql_plan;
    if (!p) return QL_ERR_WORKSPACE;
    p->layers.assign(layers, layers + n_layers);
    p->M_max = M_max;
    p->K_widest = widest;
    *plan_out = p;
    return QL_OK;
}

void ql_plan_destroy(ql_plan *plan) { delete plan; }

int32_t ql_plan_num_layers(const ql_plan *plan) { return plan ? (int32_t)plan->layers.size() : 0; }

size_t ql_plan_workspace_bytes(const ql_plan *plan, int64_t M, int64_t R)
{
    if (!plan || M < 1 || R < 1 || M % R != 0 || M > plan->M_max) return 0;
    return layer_ws(M, plan->K_widest, R).total;
}

static int plan_run_any(const ql_plan *plan, const void *const *x_in, void *const *y_out, int64_t M, int64_t R,
                        const ql_daq_params *dp, void *workspace, size_t workspace_bytes, void *stream,
                        const ql_fusion *const *fusion = nullptr)
{
    if (!plan || !x_in || !y_out) return QL_ERR_NULL;
    if (M < 1 || R < 1 || M % R != 0 || M > plan->M_max) return QL_ERR_SHAPE;
    if (dp && (dp->p_ppm < 1 || dp->p_ppm > 1000000 || dp->a_bits < 2 || dp->a_bits > 8)) return QL_ERR_UNSUPPORTED;
    for (size_t l = 0; l < plan->layers.size(); ++l) {
        if (!x_in[l] || !y_out[l]) return QL_ERR_NULL;
        if (misaligned(x_in[l], 2) || misaligned(y_out[l], 2)) return QL_ERR_ALIGN;
    }
    int rc = check_workspace(workspace, workspace_bytes, ql_plan_workspace_bytes(plan, M, R));
    if (rc) return rc;
    if (fusion)
        for (size_t l = 0; l < plan->layers.size(); ++l) {
            rc = check_fusion(fusion[l], M);
            if (rc) return rc;
        }
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (size_t l = 0; l < plan->layers.size(); ++l) {
        const ql_layer_desc &d = plan->layers[l];
        rc = run_layer(x_in[l], M, d.K, R, d.w_bits, d.w, d.w_scale, d.bias, d.N, y_out[l], nullptr, workspace, s, dp,
                       d.w_bits == 4 ? d.group : 128, fusion ? fusion[l] : nullptr);
        if (rc) return rc;
    }
    return QL_OK;
}

int qlinear_plan_run(const ql_plan *plan, const void *const *x_in, void *const *y_out, int64_t M, int64_t R,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    return plan_run_any(plan, x_in, y_out, M, R, nullptr, workspace, workspace_bytes, stream);
}

int qlinear_plan_run_ex(const ql_plan *plan, const void *const *x_in, void *const *y_out, int64_t M, int64_t R,
                        const ql_daq_params *params, const ql_fusion *const *fusion, void *workspace, size_t workspace_bytes,
                        void *stream)
{
    return plan_run_any(plan, x_in, y_out, M, R, params, workspace, workspace_bytes, stream, fusion);
}

int qlinear_plan_run_robust(const ql_plan *plan, const void *const *x_in, void *const *y_out, int64_t M, int64_t R,
                            const ql_daq_params *params, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!params) return QL_ERR_NULL;
    return plan_run_any(plan, x_in, y_out, M, R, params, workspace, workspace_bytes, stream);
}

int ql_set_gemm_variant(int variant)
{
    if (variant < -1 || variant > ql::num_gemm_variants()) return QL_ERR_UNSUPPORTED;
    g_gemm_variant.store(variant);
    return QL_OK;
}

int ql_num_gemm_variants(void) { return ql::num_gemm_variants(); }

const char *ql_gemm_variant_name(int variant) { return ql::gemm_variant_name(variant); }

}  // extern "C"
