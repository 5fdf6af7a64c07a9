/*
 * CPU oracle for the quantized DiT linear layer of DiffPro (arXiv 2511.11446).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * scalar restatement of what the deployed layer computes, written to be
 * checked against the paper by eye.  Only the test-suite, the smoke check and
 * the benchmark's "cpu_baseline" leg may call it.  It shares no code, header,
 * table or constant with the HIP path.
 *
 * What it follows:
 *   - Step 3, eq. (4): symmetric activation quantizer, zero-point 0, b = 8,
 *     alpha = tau / (2^(b-1) - 1), code = round(clip(v, +-tau) / alpha).
 *     tau is read as the block's absolute maximum (percentile p -> 100, the
 *     "min max scales" of Section 2.3), so the clip never changes a value.
 *   - Step 3 / Step 5 / Section 6: every linear is an INT8 x INT8 -> INT32
 *     GEMM with per-output-channel (or per-group) weight scales, followed by
 *     dequantization.
 *   - Step 2: weights are integer codes with per-group scales; the symmetric
 *     form (zero-point 0) of the ablation section is used.  Group sizes other
 *     than 128 (Algorithm 1) and layers left in FP16: orc_gemm_w4g, orc_linear_f16.
 *   - eq. (4) as printed (percentile clipping) with the activation width of
 *     Step 6: orc_daq_robust.  Residual additions and the MLP activation folded
 *     into the epilogue (Section 6 counts them in the latency): orc_block_glue.
 *
 * Every function is pinned by the CPU tests against something other than itself
 * (hand-worked cases, invariants, brute force, numpy routines): none is
 * "parity unpinned".
 *
 * Conventions the paper leaves open (every one is listed in the design notes):
 *   round = round-half-to-even; an all-zero block gets scale 1; the quotient
 *   v / alpha is one correctly rounded binary32 division; codes are clamped
 *   to [-127, 127]; the epilogue is evaluated in binary32 in the order
 *   written below, where fmaf(a, b, c) is a*b+c with a single rounding and
 *   every other operation rounds once.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC.
 * Rows are independent, so the only parallelism is an OpenMP loop over rows
 * (nthreads <= 1 means serial).
 */
#include <math.h>
#include <stdlib.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* IEEE binary16 <-> binary32, written out on the bit fields.          */
/* ------------------------------------------------------------------ */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* Exact widening: every binary16 value is a binary32 value. */
float orc_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu;
    uint32_t m = h & 0x3ffu;
    if (e == 0) {
        /* zero or subnormal: m * 2^-24, exact in binary32 */
        float v = (float)m * bits_to_f32(0x33800000u); /* 2^-24 */
        return sign ? -v : v;
    }
    if (e == 31) return bits_to_f32(sign | 0x7f800000u | (m << 13));
    return bits_to_f32(sign | ((e + 112u) << 23) | (m << 13));
}

/* Narrowing with round-to-nearest, ties-to-even; overflow gives infinity. */
uint16_t orc_float_to_half(float f)
{
    uint32_t u = f32_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);   /* NaN */
    if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);  /* >= 65520 -> inf */
    if (a < 0x38800000u) {
        /* below 2^-14: the result is k * 2^-24 with k = rne(|f| * 2^24) */
        float scaled = bits_to_f32(a) * bits_to_f32(0x4b800000u); /* 2^24, exact */
        uint32_t k = (uint32_t)nearbyintf(scaled); /* 0..1024; 1024 is the smallest normal */
        return (uint16_t)(sign | k);
    }
    uint32_t keep = (a >> 13) - (112u << 10);  /* exponent re-biased, 10 mantissa bits */
    uint32_t drop = a & 0x1fffu;               /* the 13 bits that do not fit */
    if (drop > 0x1000u || (drop == 0x1000u && (keep & 1u))) keep += 1; /* carry may bump the exponent */
    return (uint16_t)(sign | keep);
}

void orc_half_to_float_array(const uint16_t *h, float *f, int64_t n)
{ for (int64_t i = 0; i < n; ++i) f[i] = orc_half_to_float(h[i]); }

void orc_float_to_half_array(const float *f, uint16_t *h, int64_t n)
{ for (int64_t i = 0; i < n; ++i) h[i] = orc_float_to_half(f[i]); }

/* ------------------------------------------------------------------ */
/* Step 3, eq. (4): dynamic activation quantization.                   */
/*   x      [M,K] binary16, row-major                                  */
/*   R      rows per scale block (1 = per token, tokens-per-image =    */
/*          per sample, M = per tensor); M % R == 0                    */
/*   q      [M,K] int8 codes, out                                      */
/*   scale  [M/R] binary32 alpha, out                                  */
/* ------------------------------------------------------------------ */
int orc_daq(const uint16_t *x, int64_t M, int64_t K, int64_t R,
            int8_t *q, float *scale, int nthreads)
{
    if (M < 0 || K < 0 || R <= 0 || (M % R) != 0) return 1;
    int64_t nblk = M / R;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int64_t b = 0; b < nblk; ++b) {
        const uint16_t *xb = x + b * R * K;
        /* tau: largest magnitude of the block (eq. 4 line 1 with p = 100) */
        float tau = 0.0f;
        for (int64_t i = 0; i < R * K; ++i) {
            float v = fabsf(orc_half_to_float(xb[i]));
            if (v > tau) tau = v;
        }
        /* alpha = tau / (2^(b-1) - 1), b = 8 (eq. 4 line 2) */
        float alpha = (tau == 0.0f) ? 1.0f : tau / 127.0f;
        scale[b] = alpha;
        /* code = round(clip(v, -tau, tau) / alpha) (eq. 4 line 3, before the
         * multiplication back by alpha, which the GEMM epilogue performs) */
        for (int64_t i = 0; i < R * K; ++i) {
            float v = orc_half_to_float(xb[i]);
            if (v > tau) v = tau;
            if (v < -tau) v = -tau;
            float t = v / alpha;
            float r = nearbyintf(t);           /* ties to even */
            if (r > 127.0f) r = 127.0f;
            if (r < -127.0f) r = -127.0f;
            q[b * R * K + i] = (int8_t)r;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Step 3, eq. (4) as printed: percentile clipping, and the activation */
/* width b that Step 6 / Algorithm 2 Phase B set per time bin.         */
/*   tau   = Percentile(|v|, p) over the scale block, nearest rank:    */
/*           the k-th smallest magnitude, k = ceil(n * p_ppm / 10^6)   */
/*           (p given in parts per million of 1, 999000 = the paper's  */
/*           p = 99.9; k clamped to [1, n]; integer arithmetic)        */
/*   alpha = tau / (2^(b-1) - 1)      (1 if tau = 0)                   */
/*   code  = round(clip(v, -tau, tau) / alpha), ties to even           */
/*   a_bits b in [2, 8]; codes are stored as int8                      */
/* p_ppm = 10^6 and b = 8 is orc_daq().                                */
/* ------------------------------------------------------------------ */
static int cmp_u16(const void *a, const void *b)
{
    uint16_t x = *(const uint16_t *)a, y = *(const uint16_t *)b;
    return (x > y) - (x < y);
}

int orc_daq_robust(const uint16_t *x, int64_t M, int64_t K, int64_t R, int64_t p_ppm, int a_bits,
                   int8_t *q, float *scale, int nthreads)
{
    if (M < 0 || K < 0 || R <= 0 || (M % R) != 0) return 1;
    if (p_ppm < 1 || p_ppm > 1000000 || a_bits < 2 || a_bits > 8) return 1;
    int64_t nblk = M / R, n = R * K;
    const float qmax = (float)((1 << (a_bits - 1)) - 1);
    int fail = 0;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int64_t b = 0; b < nblk; ++b) {
        const uint16_t *xb = x + b * n;
        if (n == 0) continue;
        /* magnitudes as binary16 bit patterns with the sign cleared: for finite values their integer order is the
         * numeric order, so sorting the patterns sorts the magnitudes */
        uint16_t *mag = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)n);
        if (!mag) { fail = 1; continue; }
        for (int64_t i = 0; i < n; ++i) mag[i] = (uint16_t)(xb[i] & 0x7fffu);
        qsort(mag, (size_t)n, sizeof(uint16_t), cmp_u16);
        int64_t k = (n * p_ppm + 999999) / 1000000;   /* ceil(n p) */
        if (k < 1) k = 1;
        if (k > n) k = n;
        float tau = orc_half_to_float(mag[k - 1]);
        free(mag);
        float alpha = (tau == 0.0f) ? 1.0f : tau / qmax;
        scale[b] = alpha;
        for (int64_t i = 0; i < n; ++i) {
            float v = orc_half_to_float(xb[i]);
            if (v > tau) v = tau;
            if (v < -tau) v = -tau;
            float t = v / alpha;
            float r = nearbyintf(t);
            if (r > qmax) r = qmax;
            if (r < -qmax) r = -qmax;
            q[b * n + i] = (int8_t)r;
        }
    }
    return fail ? 3 : 0;
}

/* ------------------------------------------------------------------ */
/* INT8 x INT8 -> INT32 GEMM (Step 3, Section 6).                      */
/*   acc[m,n] = sum_k q[m,k] * w[n,k]     q [M,K], w [N,K], acc [M,N]  */
/* ------------------------------------------------------------------ */
int orc_gemm_i8(const int8_t *q, const int8_t *w, int64_t M, int64_t N, int64_t K,
                int32_t *acc, int nthreads)
{
    if (M < 0 || N < 0 || K < 0) return 1;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int32_t)q[m * K + k] * (int32_t)w[n * K + k];
            acc[m * N + n] = s;
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* 4-bit weight storage.  Codes are two's-complement nibbles in        */
/* [-8, 7], two per byte, K/2 bytes per output channel.  Inside every  */
/* run of 8 consecutive k (4 bytes), byte j (j = 0..3) carries         */
/* k = 8b + j in its low nibble and k = 8b + 4 + j in its high nibble. */
/* (The paper says only that weights are packed; this order is the     */
/* library's documented storage format.)                               */
/* ------------------------------------------------------------------ */
static int64_t w4_byte_of(int64_t k) { return 4 * (k / 8) + (k % 4); }
static int w4_is_high(int64_t k) { return (k % 8) >= 4; }

int orc_pack_w4(const int8_t *w, int64_t N, int64_t K, uint8_t *packed)
{
    if (N < 0 || K < 0 || (K % 8) != 0) return 1;
    memset(packed, 0, (size_t)(N * (K / 2)));
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int v = w[n * K + k];
            if (v < -8 || v > 7) return 2;
            uint8_t nib = (uint8_t)(v & 0xF);
            uint8_t *p = &packed[n * (K / 2) + w4_byte_of(k)];
            *p |= w4_is_high(k) ? (uint8_t)(nib << 4) : nib;
        }
    return 0;
}

int orc_unpack_w4(const uint8_t *packed, int64_t N, int64_t K, int8_t *w)
{
    if (N < 0 || K < 0 || (K % 8) != 0) return 1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            uint8_t byte = packed[n * (K / 2) + w4_byte_of(k)];
            int v = w4_is_high(k) ? (byte >> 4) : (byte & 0xF);
            w[n * K + k] = (int8_t)(v >= 8 ? v - 16 : v);
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* INT8 x INT4 GEMM with one int32 partial per group of 128 k          */
/* (Step 2: group-wise weight scales need the sum split per group).    */
/*   P[m,g,n] = sum_{k in [128g,128g+128)} q[m,k] * w4[n,k]            */
/*   P is [M, K/128, N]                                                */
/* ------------------------------------------------------------------ */
int orc_gemm_w4g128(const int8_t *q, const uint8_t *w4, int64_t M, int64_t N, int64_t K,
                    int32_t *P, int nthreads)
{
    if (M < 0 || N < 0 || K < 0 || (K % 128) != 0) return 1;
    int64_t G = K / 128;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t g = 0; g < G; ++g) {
                int32_t s = 0;
                for (int64_t k = 128 * g; k < 128 * g + 128; ++k) {
                    uint8_t byte = w4[n * (K / 2) + w4_byte_of(k)];
                    int v = w4_is_high(k) ? (byte >> 4) : (byte & 0xF);
                    if (v >= 8) v -= 16;
                    s += (int32_t)q[m * K + k] * v;
                }
                P[(m * G + g) * N + n] = s;
            }
    return 0;
}

/* ------------------------------------------------------------------ */
/* The same with weight groups of `group` consecutive k (Step 2 and    */
/* Algorithm 1 choose the group size per layer; Step 2's final plan    */
/* uses 32, 64, 128, 192 and 288):                               */
/*   P[m,g,n] = sum_{k in [group*g, group*g+group)} q[m,k] * w4[n,k]   */
/*   P is [M, K/group, N];  K % group == 0                             */
/* ------------------------------------------------------------------ */
int orc_gemm_w4g(const int8_t *q, const uint8_t *w4, int64_t M, int64_t N, int64_t K, int64_t group,
                 int32_t *P, int nthreads)
{
    if (M < 0 || N < 0 || K < 0 || group <= 0 || (K % group) != 0 || (K % 8) != 0) return 1;
    int64_t G = K / group;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t g = 0; g < G; ++g) {
                int32_t s = 0;
                for (int64_t k = group * g; k < group * g + group; ++k) {
                    uint8_t byte = w4[n * (K / 2) + w4_byte_of(k)];
                    int v = w4_is_high(k) ? (byte >> 4) : (byte & 0xF);
                    if (v >= 8) v -= 16;
                    s += (int32_t)q[m * K + k] * v;
                }
                P[(m * G + g) * N + n] = s;
            }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Integer codes of any width up to 8 bits held as int8 (W3, W6, W8 with */
/* group scales, or asymmetric codes stored as code - zero; Step 2,      */
/* Algorithm 1), with weight groups of `group` consecutive k:            */
/*   P[m,g,n] = sum_{k in group g} q[m,k] * w[n,k],  P is [M, K/group, N] */
/* ------------------------------------------------------------------ */
int orc_gemm_i8g(const int8_t *q, const int8_t *w, int64_t M, int64_t N, int64_t K, int64_t group,
                 int32_t *P, int nthreads)
{
    if (M < 0 || N < 0 || K < 0 || group <= 0 || (K % group) != 0) return 1;
    int64_t G = K / group;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            for (int64_t g = 0; g < G; ++g) {
                int32_t s = 0;
                for (int64_t k = group * g; k < group * g + group; ++k) s += (int32_t)q[m * K + k] * (int32_t)w[n * K + k];
                P[(m * G + g) * N + n] = s;
            }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Dequantization when the activation scales are per scale block AND    */
/* per channel group (Step 3, eq. (4): one scale per sample, timestep   */
/* and group of channels), the channel groups being the weight groups:  */
/*   c = s_w[n,g] * alpha[m/R, g]                (binary32 product)      */
/*   f = fma(float(P[m,g,n]), c, f)              g ascending, f from 0   */
/*   y = f16(f + bias[n])                        (f without a bias)      */
/* alpha is [M/R, G] binary32, s_w [N, G] binary16.                      */
/* ------------------------------------------------------------------ */
int orc_epilogue_cg(const int32_t *P, const float *alpha, int64_t R, const uint16_t *s_w,
                    const uint16_t *bias, int64_t M, int64_t N, int64_t G, uint16_t *y)
{
    if (M < 0 || N < 0 || G < 0 || R <= 0 || (M % R) != 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float f = 0.0f;
            for (int64_t g = 0; g < G; ++g) {
                float c = orc_half_to_float(s_w[n * G + g]) * alpha[(m / R) * G + g];
                f = fmaf((float)P[(m * G + g) * N + n], c, f);
            }
            float u = bias ? f + orc_half_to_float(bias[n]) : f;
            y[m * N + n] = orc_float_to_half(u);
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Dequantization epilogues (Section 6: "dequantization"; Step 5:      */
/* per-output-channel weight scales).  binary32, one rounding per      */
/* operation, in the order written; fma = fused multiply-add.          */
/*   W8:  t = float(acc) * s_a[m/R]                                     */
/*        y = f16( fma(t, s_w[n], bias[n]) )      [t * s_w[n] if no bias] */
/*   W4:  f = 0; for g ascending: f = fma(float(P[g]), s_w[n,g], f)      */
/*        y = f16( fma(f, s_a[m/R], bias[n]) )    [f * s_a if no bias]   */
/*   bias == NULL means no bias term.                                  */
/* ------------------------------------------------------------------ */
int orc_epilogue_w8(const int32_t *acc, const float *s_a, int64_t R, const float *s_w,
                    const uint16_t *bias, int64_t M, int64_t N, uint16_t *y)
{
    if (M < 0 || N < 0 || R <= 0 || (M % R) != 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float t = (float)acc[m * N + n] * s_a[m / R];
            float u = bias ? fmaf(t, s_w[n], orc_half_to_float(bias[n])) : t * s_w[n];
            y[m * N + n] = orc_float_to_half(u);
        }
    return 0;
}

int orc_epilogue_w4(const int32_t *P, const float *s_a, int64_t R, const uint16_t *s_w,
                    const uint16_t *bias, int64_t M, int64_t N, int64_t G, uint16_t *y)
{
    if (M < 0 || N < 0 || G < 0 || R <= 0 || (M % R) != 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float f = 0.0f;
            for (int64_t g = 0; g < G; ++g)
                f = fmaf((float)P[(m * G + g) * N + n], orc_half_to_float(s_w[n * G + g]), f);
            float u = bias ? fmaf(f, s_a[m / R], orc_half_to_float(bias[n])) : f * s_a[m / R];
            y[m * N + n] = orc_float_to_half(u);
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Block glue folded into the layer's epilogue (Section 6 counts the   */
/* residual additions in the latency; Step 3 keeps residual adds in    */
/* higher precision; the MLP's activation sits between its two         */
/* quantized linears).                                                  */
/*   u  = the dequantized binary32 value of the layer, as above, before */
/*        its rounding to binary16 (orc_dequant_w8 / _w4)               */
/*   h  = f16( act(u) )     act = identity, or GELU in its tanh form    */
/*        gelu(u) = u * sigmoid(2 z), z = sqrt(2/pi) (u + 0.044715 u^3) */
/*        (= 0.5 u (1 + tanh z)), evaluated in binary64, rounded to     */
/*        binary32 and then to binary16                                 */
/*   y  = h                                   without gate and residual */
/*   y  = f16( fma(g, float(h), r) )          g = gate[m / gate_rows, n] (1 if none), r = residual[m, n] (0 if none) */
/* ------------------------------------------------------------------ */
int orc_dequant_w8(const int32_t *acc, const float *s_a, int64_t R, const float *s_w,
                   const uint16_t *bias, int64_t M, int64_t N, float *u)
{
    if (M < 0 || N < 0 || R <= 0 || (M % R) != 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float t = (float)acc[m * N + n] * s_a[m / R];
            u[m * N + n] = bias ? fmaf(t, s_w[n], orc_half_to_float(bias[n])) : t * s_w[n];
        }
    return 0;
}

int orc_dequant_w4(const int32_t *P, const float *s_a, int64_t R, const uint16_t *s_w,
                   const uint16_t *bias, int64_t M, int64_t N, int64_t G, float *u)
{
    if (M < 0 || N < 0 || G < 0 || R <= 0 || (M % R) != 0) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float f = 0.0f;
            for (int64_t g = 0; g < G; ++g)
                f = fmaf((float)P[(m * G + g) * N + n], orc_half_to_float(s_w[n * G + g]), f);
            u[m * N + n] = bias ? fmaf(f, s_a[m / R], orc_half_to_float(bias[n])) : f * s_a[m / R];
        }
    return 0;
}

int orc_block_glue(const float *u, int64_t M, int64_t N, int act, const uint16_t *residual,
                   const uint16_t *gate, int64_t gate_rows, uint16_t *y)
{
    if (M < 0 || N < 0 || (act != 0 && act != 1)) return 1;
    if (gate && (gate_rows <= 0 || (M % gate_rows) != 0)) return 1;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float v = u[m * N + n];
            if (act == 1) {
                double x = (double)v;
                double z = 0.7978845608028654 * (x + 0.044715 * x * x * x);   /* sqrt(2/pi) */
                v = (float)(x / (1.0 + exp(-2.0 * z)));
            }
            uint16_t h = orc_float_to_half(v);
            if (gate || residual) {
                float g = gate ? orc_half_to_float(gate[(m / gate_rows) * N + n]) : 1.0f;
                float r = residual ? orc_half_to_float(residual[m * N + n]) : 0.0f;
                h = orc_float_to_half(fmaf(g, orc_half_to_float(h), r));
            }
            y[m * N + n] = h;
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* A layer the plan leaves in FP16 (Step 2 freezes the most sensitive   */
/* layers; its final plan keeps 22 of 113 layers in FP16):              */
/*   y[m,n] = f16( sum_k x[m,k] * w[n,k] + bias[n] )                    */
/* x [M,K], w [N,K], bias [N] binary16.  The sum is taken in binary64   */
/* (every product of two binary16 values is exact there), the bias is   */
/* added in binary64, and the result is rounded to binary32 and then to */
/* binary16.                                                            */
/* ------------------------------------------------------------------ */
int orc_linear_f16(const uint16_t *x, const uint16_t *w, const uint16_t *bias,
                   int64_t M, int64_t N, int64_t K, uint16_t *y, int nthreads)
{
    if (M < 0 || N < 0 || K < 0) return 1;
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 1 ? nthreads : 1)
#endif
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += (double)orc_half_to_float(x[m * K + k]) * (double)orc_half_to_float(w[n * K + k]);
            if (bias) s += (double)orc_half_to_float(bias[n]);
            y[m * N + n] = orc_float_to_half((float)s);
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* The whole layer: DAQ -> GEMM -> epilogue.  Optional outputs         */
/* (q, s_a, acc / P) may be NULL; scratch is then taken from the heap. */
/* ------------------------------------------------------------------ */
#include <stdlib.h>

int orc_qlinear_w8a8(const uint16_t *x, int64_t M, int64_t K, int64_t R,
                     const int8_t *w, const float *s_w, const uint16_t *bias, int64_t N,
                     uint16_t *y, int8_t *q_out, float *s_a_out, int32_t *acc_out, int nthreads)
{
    if (M <= 0 || K <= 0 || N <= 0 || R <= 0 || (M % R) != 0) return 1;
    int8_t *q = q_out ? q_out : (int8_t *)malloc((size_t)(M * K));
    float *s_a = s_a_out ? s_a_out : (float *)malloc(sizeof(float) * (size_t)(M / R));
    int32_t *acc = acc_out ? acc_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(M * N));
    int rc = (!q || !s_a || !acc) ? 3 : 0;
    if (!rc) rc = orc_daq(x, M, K, R, q, s_a, nthreads);
    if (!rc) rc = orc_gemm_i8(q, w, M, N, K, acc, nthreads);
    if (!rc) rc = orc_epilogue_w8(acc, s_a, R, s_w, bias, M, N, y);
    if (!q_out) free(q);
    if (!s_a_out) free(s_a);
    if (!acc_out) free(acc);
    return rc;
}

int orc_qlinear_w4a8(const uint16_t *x, int64_t M, int64_t K, int64_t R,
                     const uint8_t *w4, const uint16_t *s_w, const uint16_t *bias, int64_t N,
                     uint16_t *y, int8_t *q_out, float *s_a_out, int32_t *P_out, int nthreads)
{
    if (M <= 0 || K <= 0 || N <= 0 || R <= 0 || (M % R) != 0 || (K % 128) != 0) return 1;
    int64_t G = K / 128;
    int8_t *q = q_out ? q_out : (int8_t *)malloc((size_t)(M * K));
    float *s_a = s_a_out ? s_a_out : (float *)malloc(sizeof(float) * (size_t)(M / R));
    int32_t *P = P_out ? P_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(M * G * N));
    int rc = (!q || !s_a || !P) ? 3 : 0;
    if (!rc) rc = orc_daq(x, M, K, R, q, s_a, nthreads);
    if (!rc) rc = orc_gemm_w4g128(q, w4, M, N, K, P, nthreads);
    if (!rc) rc = orc_epilogue_w4(P, s_a, R, s_w, bias, M, N, G, y);
    if (!q_out) free(q);
    if (!s_a_out) free(s_a);
    if (!P_out) free(P);
    return rc;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
