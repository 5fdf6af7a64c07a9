// Host side of the method's offline stages, behind the C ABI of include/diffpro_qlinear.h: which timesteps to keep
// (Step 4, eqs. (5)-(6)), the budgeted greedy planner over weight widths and timesteps (Algorithm 2, Phase A; fed
// with per-layer latencies measured through this library), and the GPTQ weight packer (Step 2) whose integer codes
// go to ql_pack_w4_host / the int8 weight layout.  Plain C++ on host memory, no device call.
#include "../../include/diffpro_qlinear.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <queue>
#include <vector>

namespace {

inline bool rho_ok(int32_t rho_ppm) { return rho_ppm >= 0 && rho_ppm <= 1000000; }

// binary16 rounding (nearest, ties to even) of a positive double, returned as a double; subnormal results are kept
double round_to_half(double v)
{
    if (!(v > 0.0)) return 0.0;
    if (v >= 65520.0) return 65504.0;                 // saturate instead of overflowing to infinity
    int e;
    std::frexp(v, &e);                                // v = f * 2^e, f in [0.5, 1)
    int ulp_exp = (e - 1) - 10;                       // 11 significant bits
    if (ulp_exp < -24) ulp_exp = -24;                 // subnormal spacing
    const double scaled = std::ldexp(v, -ulp_exp);
    return std::ldexp(std::nearbyint(scaled), ulp_exp);   // default rounding mode: ties to even
}

struct Grid {
    double scale;
    int zero, qmin, qmax;
};

void code_range(int bits, bool symmetric, int &qmin, int &qmax)
{
    if (symmetric) {
        qmax = (1 << (bits - 1)) - 1;
        qmin = bits == 8 ? -qmax : -(1 << (bits - 1));
    } else {
        qmin = 0;
        qmax = (1 << bits) - 1;
    }
}

// scale and zero point of one group of one row, from the row's current weights (Step 2: per-group scale and zero point)
Grid make_grid(const double *w, int64_t n, int bits, bool symmetric, bool scale_fp16)
{
    Grid g;
    code_range(bits, symmetric, g.qmin, g.qmax);
    double lo = 0.0, hi = 0.0, amax = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        lo = std::min(lo, w[i]);
        hi = std::max(hi, w[i]);
        amax = std::max(amax, std::fabs(w[i]));
    }
    double s;
    if (symmetric) s = amax > 0.0 ? amax / g.qmax : 1.0;
    else s = hi > lo ? (hi - lo) / g.qmax : 1.0;
    if (scale_fp16) {
        s = round_to_half(s);
        if (!(s > 0.0)) s = std::ldexp(1.0, -24);
    } else {
        s = (double)(float)s;
    }
    g.scale = s;
    g.zero = symmetric ? 0 : (int)std::nearbyint(-lo / s);
    return g;
}

}  // namespace

extern "C" {

int ql_schedule_topk(const double *delta, const int32_t *candidates, int32_t n_candidates, int32_t T, int32_t rho_ppm,
                     int32_t k, int32_t *kept_out)
{
    if (!delta || !candidates || !kept_out) return QL_ERR_NULL;
    if (T < 1 || n_candidates < 1 || k < 0 || !rho_ok(rho_ppm)) return QL_ERR_SHAPE;
    std::vector<int32_t> cand(candidates, candidates + n_candidates);
    for (int32_t t : cand)
        if (t < 0 || t >= T) return QL_ERR_SHAPE;
    std::sort(cand.begin(), cand.end());
    cand.erase(std::unique(cand.begin(), cand.end()), cand.end());
    // T_tail = { t in C : t / T >= 1 - rho }, decided in integers
    std::vector<int32_t> tail, rest;
    for (int32_t t : cand) {
        if ((int64_t)t * 1000000 >= (int64_t)T * (1000000 - rho_ppm)) tail.push_back(t);
        else rest.push_back(t);
    }
    const int64_t m = (int64_t)k - (int64_t)tail.size();
    if (m < 0 || k > (int32_t)cand.size()) return QL_ERR_SHAPE;
    // TopK: the m largest delta, the earlier step first among equals
    std::stable_sort(rest.begin(), rest.end(), [&](int32_t x, int32_t y) { return delta[x] > delta[y]; });
    std::vector<int32_t> kept(tail);
    kept.insert(kept.end(), rest.begin(), rest.begin() + m);
    std::sort(kept.begin(), kept.end());
    std::copy(kept.begin(), kept.end(), kept_out);
    return QL_OK;
}

int ql_plan_greedy(const double *drift, const double *c_step, int32_t T, const ql_planner_layer *layers, int32_t L,
                   double B_lat, double B_mem, int32_t rho_ppm, double eps, int32_t *bits_out, uint8_t *kept_out,
                   double *C_lat_out, double *C_mem_out, int32_t *feasible_out)
{
    if (!drift || !c_step || !layers || !bits_out || !kept_out) return QL_ERR_NULL;
    if (T < 1 || L < 1 || !rho_ok(rho_ppm) || !(eps >= 0.0)) return QL_ERR_SHAPE;
    for (int32_t l = 0; l < L; ++l) {
        if (layers[l].n_options < 1) return QL_ERR_SHAPE;
        if (!layers[l].bits || !layers[l].c_lat || !layers[l].c_mem) return QL_ERR_NULL;
    }
    // every layer's options by decreasing width; the plan starts at the widest
    std::vector<std::vector<int>> order(L);
    std::vector<int> pos(L, 0);
    for (int32_t l = 0; l < L; ++l) {
        order[l].resize(layers[l].n_options);
        for (int i = 0; i < layers[l].n_options; ++i) order[l][i] = i;
        std::stable_sort(order[l].begin(), order[l].end(), [&](int x, int y) { return layers[l].bits[x] > layers[l].bits[y]; });
        for (int i = 1; i < layers[l].n_options; ++i)
            if (layers[l].bits[order[l][i]] == layers[l].bits[order[l][i - 1]]) return QL_ERR_SHAPE;   // a width listed twice
    }
    const int32_t n_tail = (int32_t)((int64_t)rho_ppm * T / 1000000);   // Tail = the last floor(rho |T|) indices
    double C_lat = 0.0, C_mem = 0.0;
    for (int32_t t = 0; t < T; ++t) {
        C_lat += c_step[t];
        kept_out[t] = 1;
    }
    for (int32_t l = 0; l < L; ++l) {
        C_lat += layers[l].c_lat[order[l][0]];
        C_mem += layers[l].c_mem[order[l][0]];
    }
    // prunable steps by increasing drift (the earlier step first among equals)
    std::vector<int32_t> R;
    for (int32_t t = 0; t < T - n_tail; ++t) R.push_back(t);
    std::stable_sort(R.begin(), R.end(), [&](int32_t x, int32_t y) { return drift[x] < drift[y]; });
    size_t r_head = 0;
    // max-heap of the next move of every layer, scored S_bit = delta c_lat / (eps + s_M); smaller layer index first among equals
    struct Move {
        double score;
        int32_t layer;
    };
    auto worse = [](const Move &x, const Move &y) { return x.score < y.score || (x.score == y.score && x.layer > y.layer); };
    std::priority_queue<Move, std::vector<Move>, decltype(worse)> heap(worse);
    auto push = [&](int32_t l) {
        if (pos[l] + 1 < layers[l].n_options) {
            const double d = layers[l].c_lat[order[l][pos[l]]] - layers[l].c_lat[order[l][pos[l] + 1]];
            heap.push(Move{d / (eps + layers[l].sensitivity), l});
        }
    };
    for (int32_t l = 0; l < L; ++l) push(l);
    int32_t feasible = 1;
    while (C_lat > B_lat || C_mem > B_mem) {
        const bool step_ok = r_head < R.size() && C_lat > B_lat;   // removing a step frees no memory
        const bool bit_ok = !heap.empty();
        if (!step_ok && !bit_ok) {
            feasible = 0;
            break;
        }
        const double S_step = step_ok ? c_step[R[r_head]] / (eps + drift[R[r_head]]) : 0.0;
        if (step_ok && (!bit_ok || S_step > heap.top().score)) {
            const int32_t t = R[r_head++];
            kept_out[t] = 0;
            C_lat -= c_step[t];
        } else {
            const int32_t l = heap.top().layer;
            heap.pop();
            const int from = order[l][pos[l]], to = order[l][pos[l] + 1];
            C_lat -= layers[l].c_lat[from] - layers[l].c_lat[to];
            C_mem -= layers[l].c_mem[from] - layers[l].c_mem[to];
            ++pos[l];
            push(l);
        }
    }
    for (int32_t l = 0; l < L; ++l) bits_out[l] = layers[l].bits[order[l][pos[l]]];
    if (C_lat_out) *C_lat_out = C_lat;
    if (C_mem_out) *C_mem_out = C_mem;
    if (feasible_out) *feasible_out = feasible;
    return QL_OK;
}

int ql_gptq_quantize_host(const float *W_in, int64_t N, int64_t K, const double *H_in, int32_t bits, int64_t group,
                          int32_t symmetric, double damp, int32_t scale_fp16, int8_t *codes, float *scales, int32_t *zeros)
{
    if (!W_in || !H_in || !codes || !scales) return QL_ERR_NULL;
    if (!symmetric && !zeros) return QL_ERR_NULL;
    if (N < 1 || K < 1 || group < 1 || K % group != 0 || K > 16384) return QL_ERR_SHAPE;
    if (bits < 2 || bits > 8 || !(damp >= 0.0)) return QL_ERR_UNSUPPORTED;
    const int64_t G = K / group;
    std::vector<double> H(H_in, H_in + K * K), W((size_t)N * K);
    for (int64_t i = 0; i < N * K; ++i) W[i] = W_in[i];
    // 1. inputs that never fire: unit diagonal, weight column dropped; then the damping term on the diagonal
    double mean_diag = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        if (H[k * K + k] == 0.0) {
            H[k * K + k] = 1.0;
            for (int64_t n = 0; n < N; ++n) W[n * K + k] = 0.0;
        }
        mean_diag += H[k * K + k];
    }
    mean_diag /= (double)K;
    for (int64_t k = 0; k < K; ++k) H[k * K + k] += damp * mean_diag;
    // 2. H = L L^T (column Cholesky, in place in the lower triangle)
    for (int64_t j = 0; j < K; ++j) {
        double d = H[j * K + j];
        for (int64_t p = 0; p < j; ++p) d -= H[j * K + p] * H[j * K + p];
        if (!(d > 0.0)) return QL_ERR_UNSUPPORTED;   // not positive definite: more damping needed
        const double ljj = std::sqrt(d);
        H[j * K + j] = ljj;
        for (int64_t i = j + 1; i < K; ++i) {
            double v = H[i * K + j];
            for (int64_t p = 0; p < j; ++p) v -= H[i * K + p] * H[j * K + p];
            H[i * K + j] = v / ljj;
        }
    }
    //    Li = L^-1 (lower), then H^-1 = Li^T Li
    std::vector<double> Li((size_t)K * K, 0.0);
    for (int64_t c = 0; c < K; ++c) {   // column c of Li: forward substitution on e_c
        for (int64_t i = c; i < K; ++i) {
            double v = i == c ? 1.0 : 0.0;
            for (int64_t p = c; p < i; ++p) v -= H[i * K + p] * Li[p * K + c];
            Li[i * K + c] = v / H[i * K + i];
        }
    }
    std::vector<double> Hinv((size_t)K * K, 0.0);
    for (int64_t i = 0; i < K; ++i)
        for (int64_t j = 0; j <= i; ++j) {
            double v = 0.0;
            for (int64_t p = i; p < K; ++p) v += Li[p * K + i] * Li[p * K + j];
            Hinv[i * K + j] = v;
            Hinv[j * K + i] = v;
        }
    //    H^-1 = U^T U with U upper triangular: the lower Cholesky factor of H^-1 is U^T; kept as U[k][j] = C[j][k]
    std::vector<double> &C = Hinv;   // factor in place, lower triangle
    for (int64_t j = 0; j < K; ++j) {
        double d = C[j * K + j];
        for (int64_t p = 0; p < j; ++p) d -= C[j * K + p] * C[j * K + p];
        if (!(d > 0.0)) return QL_ERR_UNSUPPORTED;
        const double cjj = std::sqrt(d);
        C[j * K + j] = cjj;
        for (int64_t i = j + 1; i < K; ++i) {
            double v = C[i * K + j];
            for (int64_t p = 0; p < j; ++p) v -= C[i * K + p] * C[j * K + p];
            C[i * K + j] = v / cjj;
        }
    }
    //    row-major copy of U, so that the update below walks memory in order
    std::vector<double> U((size_t)K * K, 0.0);
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = k; j < K; ++j) U[k * K + j] = C[j * K + k];
    // 3. column by column: quantize, push the rounding error onto the columns still to come.  Rows are independent.
    const bool sym = symmetric != 0;
    const int shift = sym ? 0 : (1 << (bits - 1));   // asymmetric codes 0 .. 2^b - 1 are stored shifted into int8
    for (int64_t n = 0; n < N; ++n) {
        double *w = &W[n * K];
        Grid g{1.0, 0, 0, 0};
        for (int64_t k = 0; k < K; ++k) {
            if (k % group == 0) {
                g = make_grid(w + k, group, bits, sym, scale_fp16 != 0);
                scales[n * G + k / group] = (float)g.scale;
                if (zeros) zeros[n * G + k / group] = g.zero - shift;
            }
            double q = std::nearbyint(w[k] / g.scale) + g.zero;
            q = std::min(std::max(q, (double)g.qmin), (double)g.qmax);
            codes[n * K + k] = (int8_t)((int)q - shift);
            const double err = (w[k] - (q - g.zero) * g.scale) / U[k * K + k];
            const double *u = &U[k * K];
            for (int64_t j = k + 1; j < K; ++j) w[j] -= err * u[j];
        }
    }
    return QL_OK;
}

}  // extern "C"
