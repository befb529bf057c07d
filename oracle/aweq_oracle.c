/*
 * AWEQ CPU oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, literal implementation of the per-linear-layer calibration and
 * quantization path of AWEQ (arXiv 2311.01305), written from the paper's equations.
 * It exists only to check the GPU library; it shares no source, header, table or
 * helper with the HIP path and nothing in the product imports or links it.  Only
 * the tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * Conventions
 *   X[T x K]  calibration activations, row-major, K contiguous (channel = column k)
 *   W[N x K]  linear weight, row-major, K contiguous (PyTorch Linear.weight layout);
 *             the paper writes Y = X W with W as K x N (Sec. 3.1, Eq. 3), so the
 *             paper's "channel i" is our column index k of both X and W.
 *   dtype 0 = IEEE binary32, 1 = IEEE binary16 (raw uint16 bit patterns)
 *   Every element-wise fp32 step is ONE binary32 operation (this file is compiled
 *   with -ffp-contract=off and without fast-math); every sum is fp64 or an exact
 *   integer.  Loops are in the order the equations are written; no blocking.
 *
 * Readings of points the paper leaves open (each is listed again in the design notes):
 *   - codes are unsigned, q_min = 0, q_max = 2^b - 1, asymmetric with zero point
 *     (Eq. 1-2 use x_max - x_min and Z);
 *   - Z = -rint(x_min / Step): x_min maps to code 0;
 *   - round-to-nearest resolves ties to even (IEEE default, what PyTorch's round does);
 *   - x / Step is a true binary32 division;
 *   - order is round, add Z, clamp (Eq. 1 as printed);
 *   - a slice whose Eq. 2 Step is not a positive finite number gets Step = 1;
 *   - Eq. 10 is evaluated on raw (un-normalised) channel ranges in fp64;
 *     channels with r_x < 1e-5 or r_w < 1e-5 get s = 1, and s is clamped to [1e-4, 1e4].
 *
 * Pins: see tests/test_oracle_*.py (hand-worked examples under tests/golden/,
 * closed forms, invariants, brute force, numpy/library special cases).
 * "parity unpinned": the choices in the list above are not fixed by any value the
 * paper prints; they are pinned only to the stated reading through worked examples.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_F16 = 1 };

/* status bits (numeric conditions met while computing) */
enum {
    ORC_ST_DEGENERATE = 1u, /* Eq. 2 gave a non-positive / non-finite Step; Step := 1 */
    ORC_ST_NONFINITE  = 2u, /* a NaN or Inf was seen in the input */
    ORC_ST_BIGQUOT    = 4u, /* |x / Step| >= 2^24 : quotient saturated / not exact */
    ORC_ST_SCALEGUARD = 8u  /* Eq. 10 guard: s forced to 1 or clamped */
};

/* ---------------------------------------------------------------- binary16 <-> binary32 */

float orc_h2f(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? (double)NAN : (double)INFINITY;
    else
        v = ldexp((double)(1024 + m), e - 25); /* (1 + m/1024) * 2^(e-15) */
    return (float)(sign ? -v : v); /* exact: every binary16 value is a binary32 value */
}

uint16_t orc_f2h(float f)
{
    uint16_t sign = signbit(f) ? 0x8000u : 0u;
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (isinf(f)) return (uint16_t)(sign | 0x7c00u);
    double a = fabs((double)f);
    int e;
    (void)frexp(a, &e); /* 2^(e-1) <= a < 2^e */
    int E = e - 1;
    if (E < -14) E = -14; /* below the smallest normal the spacing stays 2^-24 */
    double quantum = ldexp(1.0, E - 10);
    double n = nearbyint(a / quantum); /* default rounding mode: ties to even */
    if (n == 2048.0) { E += 1; n = 1024.0; }
    if (E > 15) return (uint16_t)(sign | 0x7c00u);
    if (n < 1024.0) return (uint16_t)(sign | (uint16_t)n); /* zero / subnormal */
    return (uint16_t)(sign | ((E + 15) << 10) | ((int)n - 1024));
}

static inline float ld_elt(const void* M, int dt, int64_t idx)
{
    if (dt == ORC_F16) return orc_h2f(((const uint16_t*)M)[idx]);
    return ((const float*)M)[idx];
}

static inline void st_elt(void* M, int dt, int64_t idx, float v)
{
    if (dt == ORC_F16) ((uint16_t*)M)[idx] = orc_f2h(v);
    else ((float*)M)[idx] = v;
}

void orc_h2f_array(const uint16_t* h, float* f, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) f[i] = orc_h2f(h[i]);
}

void orc_f2h_array(const float* f, uint16_t* h, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) h[i] = orc_f2h(f[i]);
}

/* ------------------------------------------------------------------ stage 1: statistics */

/* Per-column minimum, maximum and sum of a row-major [rows x K] matrix: the channel
 * range of Sec. 3.2 is "maximum minus minimum of the channel", and E[x] of Sec. 3.3 is
 * collected in the same pass.  accumulate = 0 starts from (+inf, -inf, 0, 0);
 * accumulate = 1 continues from what the buffers hold (more calibration batches, or a
 * second weight that shares the same input).  csum / count may be NULL.
 * OpenMP splits the COLUMNS between threads; each column is still visited in row order. */
void orc_col_stats(const void* M, int dt, int64_t rows, int64_t K, int64_t ld,
                   float* cmin, float* cmax, double* csum, uint64_t* count,
                   int accumulate, uint32_t* status)
{
    uint32_t st = 0;
#pragma omp parallel for schedule(static) reduction(| : st)
    for (int64_t k = 0; k < K; ++k) {
        float mn = accumulate ? cmin[k] : INFINITY;
        float mx = accumulate ? cmax[k] : -INFINITY;
        double sm = (accumulate && csum) ? csum[k] : 0.0;
        for (int64_t t = 0; t < rows; ++t) {
            float v = ld_elt(M, dt, t * ld + k);
            if (!isfinite(v)) st |= ORC_ST_NONFINITE;
            if (v < mn) mn = v;
            if (v > mx) mx = v;
            sm += (double)v;
        }
        cmin[k] = mn;
        cmax[k] = mx;
        if (csum) csum[k] = sm;
    }
    if (count) *count = (accumulate ? *count : 0) + (uint64_t)rows;
    if (status) *status |= st;
}

/* Channel range r_i, tensor range R and difficulty p_i = r_i / R (Sec. 3.2, Eq. 4).
 * R is the tensor's maximum minus the tensor's minimum ("for all channel"). */
void orc_ranges(const float* cmin, const float* cmax, int64_t K, float* r, float* R, float* p)
{
    float gmin = INFINITY, gmax = -INFINITY;
    for (int64_t k = 0; k < K; ++k) {
        if (cmin[k] < gmin) gmin = cmin[k];
        if (cmax[k] > gmax) gmax = cmax[k];
        r[k] = cmax[k] - cmin[k];
    }
    float RR = gmax - gmin;
    *R = RR;
    if (p)
        for (int64_t k = 0; k < K; ++k) p[k] = r[k] / RR;
}

/* ----------------------------------------------------------------- stage 2: equalization */

/* Eq. 10: s_i = sqrt(r_i^X r_i^W) / r_i^W, on raw channel ranges, in fp64, stored fp32.
 * enable_awe = 0 gives s = 1 (ablation switch of Sec. 4.4). */
void orc_scales(const float* r_x, const float* r_w, int64_t K, int enable_awe,
                float* s, float* inv_s, uint32_t* status)
{
    uint32_t st = 0;
    for (int64_t k = 0; k < K; ++k) {
        float sk = 1.0f;
        if (enable_awe) {
            if (!(r_x[k] >= 1e-5f) || !(r_w[k] >= 1e-5f)) {
                st |= ORC_ST_SCALEGUARD;
            } else {
                double rx = (double)r_x[k], rw = (double)r_w[k];
                sk = (float)(sqrt(rx * rw) / rw);
                if (sk < 1e-4f) { sk = 1e-4f; st |= ORC_ST_SCALEGUARD; }
                if (sk > 1e4f) { sk = 1e4f; st |= ORC_ST_SCALEGUARD; }
            }
        }
        s[k] = sk;
        inv_s[k] = 1.0f / sk;
    }
    if (status) *status |= st;
}

/* The per-channel quantity of the difficulty definition the method replaces (Sec. 1 and Sec. 3.2:
 * difficulty measured by the largest magnitude of a channel, for activations and weights alike): m_i = max_t |x[t,i]| = max(|min_i|, |max_i|).
 * orc_scales applied to (m^X, m^W) instead of (r^X, r^W) gives that variant's scale in Eq. 10's form. */
void orc_channel_absmax(const float* cmin, const float* cmax, int64_t K, float* m)
{
    for (int64_t k = 0; k < K; ++k) {
        float a = fabsf(cmin[k]), b = fabsf(cmax[k]);
        m[k] = a > b ? a : b;
    }
}

/* Eq. 3, weight side: W_hat = diag(s) W, i.e. W_hat[n,k] = W[n,k] * s[k]; the product is
 * one binary32 multiply, then rounded (to nearest even) to the layer's storage type. */
void orc_fold_weight(const void* W, int dt, int64_t N, int64_t K, int64_t ldw,
                     const float* s, void* W_hat, int64_t ldo)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            float w = ld_elt(W, dt, n * ldw + k);
            float wh = w * s[k];
            st_elt(W_hat, dt, n * ldo + k, wh);
        }
}

/* Eq. 3, activation side: X_hat[t,k] = X[t,k] * inv_s[k] (binary32, never stored by the
 * GPU path).  Materialised here for brute-force tests on small shapes. */
void orc_fold_act(const void* X, int dt, int64_t T, int64_t K, int64_t ldx,
                  const float* inv_s, float* X_hat)
{
    for (int64_t t = 0; t < T; ++t)
        for (int64_t k = 0; k < K; ++k)
            X_hat[t * K + k] = ld_elt(X, dt, t * ldx + k) * inv_s[k];
}

/* Range and mean of the equalised activation from the per-column statistics of X:
 * min_t X_hat[t,k] = xmin[k] * inv_s[k] because a correctly rounded multiply by a
 * positive constant is monotone (checked against orc_fold_act by brute force).
 * mu_xhat[k] = (xsum[k] / count) * inv_s[k] in fp64, stored fp32 (Sec. 3.3: E[x] is
 * estimated alongside the equalization factors). */
void orc_xhat_stats(const float* xmin, const float* xmax, const double* xsum, uint64_t count,
                    const float* inv_s, int64_t K, float* xhat_min, float* xhat_max,
                    float* mu_xhat)
{
    float mn = INFINITY, mx = -INFINITY;
    for (int64_t k = 0; k < K; ++k) {
        float a = xmin[k] * inv_s[k];
        float b = xmax[k] * inv_s[k];
        if (a < mn) mn = a;
        if (b > mx) mx = b;
        if (mu_xhat && xsum)
            mu_xhat[k] = (float)((xsum[k] / (double)count) * (double)inv_s[k]);
    }
    *xhat_min = mn;
    *xhat_max = mx;
}

/* -------------------------------------------------------------------- stage 3: quantizer */

/* round-half-even to int32, saturated at +-2^30 (only reachable for values far outside
 * the slice's own range; flagged). */
static inline int32_t rint_sat(float q, uint32_t* st)
{
    float r = rintf(q); /* default rounding mode: ties to even */
    if (!(fabsf(r) < 16777216.0f)) *st |= ORC_ST_BIGQUOT;
    if (!(r < 1073741824.0f)) return r != r ? 0 : 1073741824;
    if (r < -1073741824.0f) return -1073741824;
    return (int32_t)r;
}

/* Eq. 2 and the zero point: Step = (x_max - x_min) / (2^b - 1); Z = -rint(x_min / Step). */
void orc_qparams(float lo, float hi, int bits, float* step, int32_t* zero, uint32_t* status)
{
    uint32_t st = 0;
    float range = hi - lo;
    float levels = (float)((1 << bits) - 1);
    float sp = range / levels;
    if (!(sp > 0.0f) || isinf(sp)) { sp = 1.0f; st |= ORC_ST_DEGENERATE; }
    float zq = lo / sp;
    *step = sp;
    *zero = -rint_sat(zq, &st);
    if (status) *status |= st;
}

/* Eq. 1: x_q = clamp(round(x / Step) + Z; 0, 2^b - 1). */
static inline int32_t quant_one(float x, float step, int32_t zero, int32_t qmax, uint32_t* st)
{
    float q = x / step;
    int32_t u = rint_sat(q, st) + zero;
    if (u < 0) u = 0;
    if (u > qmax) u = qmax;
    return u;
}

void orc_quant_values(const float* x, int64_t n, float step, int32_t zero, int bits,
                      int32_t* u, uint32_t* status)
{
    uint32_t st = 0;
    for (int64_t i = 0; i < n; ++i) u[i] = quant_one(x[i], step, zero, (1 << bits) - 1, &st);
    if (status) *status |= st;
}

/* De-quantised value: (u - Z) * Step, one binary32 multiply of an exact integer. */
void orc_dequant_values(const int32_t* u, int64_t n, float step, int32_t zero, float* x)
{
    for (int64_t i = 0; i < n; ++i) x[i] = (float)(u[i] - zero) * step;
}

/* Weight quantizer.  group = 0: one (Step, Z) per output row n; group = g > 0: one per g
 * consecutive k inside a row (K % g == 0), stored [N x K/g]; group = -1: one for the tensor.
 * codes_u holds the UNSIGNED codes u in [0, 2^b - 1], one byte each (packing is separate).
 * rowsum_w[n] = sum_k (u - 128) is produced for bits == 8 when the pointer is non-NULL. */
void orc_quant_weight(const void* W_hat, int dt, int64_t N, int64_t K, int64_t ldw,
                      int bits, int64_t group, uint8_t* codes_u, float* step, int32_t* zero,
                      int32_t* rowsum_w, uint32_t* status)
{
    uint32_t st = 0;
    const int32_t qmax = (1 << bits) - 1;
    if (group < 0) { /* per tensor */
        float lo = INFINITY, hi = -INFINITY;
        for (int64_t n = 0; n < N; ++n)
            for (int64_t k = 0; k < K; ++k) {
                float v = ld_elt(W_hat, dt, n * ldw + k);
                if (v < lo) lo = v;
                if (v > hi) hi = v;
            }
        orc_qparams(lo, hi, bits, step, zero, &st);
    }
    const int64_t g = group > 0 ? group : K;
    const int64_t ng = K / g;
#pragma omp parallel for schedule(static) reduction(| : st)
    for (int64_t n = 0; n < N; ++n) {
        int64_t rs = 0;
        for (int64_t j = 0; j < ng; ++j) {
            float sp;
            int32_t z;
            if (group < 0) {
                sp = step[0];
                z = zero[0];
            } else {
                float lo = INFINITY, hi = -INFINITY;
                for (int64_t k = j * g; k < (j + 1) * g; ++k) {
                    float v = ld_elt(W_hat, dt, n * ldw + k);
                    if (v < lo) lo = v;
                    if (v > hi) hi = v;
                }
                orc_qparams(lo, hi, bits, &sp, &z, &st);
                step[n * ng + j] = sp;
                zero[n * ng + j] = z;
            }
            for (int64_t k = j * g; k < (j + 1) * g; ++k) {
                float v = ld_elt(W_hat, dt, n * ldw + k);
                int32_t u = quant_one(v, sp, z, qmax, &st);
                codes_u[n * K + k] = (uint8_t)u;
                rs += u - 128;
            }
        }
        if (rowsum_w && bits == 8) rowsum_w[n] = (int32_t)rs;
    }
    if (status) *status |= st;
}

/* Storage formats of the codes of one [N x K] tensor.
 *   bits 8: int8, q = u - 128, N*K bytes
 *   bits 4: two codes per byte, even k in the low nibble, N*K/2 bytes
 *   bits 3: per row a little-endian bit stream, code k in bits [3k, 3k+3), N*3K/8 bytes */
void orc_pack_codes(const uint8_t* codes_u, int64_t N, int64_t K, int bits, uint8_t* out)
{
    if (bits == 8) {
        for (int64_t i = 0; i < N * K; ++i) out[i] = (uint8_t)(int8_t)((int)codes_u[i] - 128);
    } else if (bits == 4) {
        for (int64_t i = 0; i < N * K / 2; ++i)
            out[i] = (uint8_t)((codes_u[2 * i] & 15) | ((codes_u[2 * i + 1] & 15) << 4));
    } else {
        const int64_t rb = 3 * K / 8;
        memset(out, 0, (size_t)(N * rb));
        for (int64_t n = 0; n < N; ++n)
            for (int64_t k = 0; k < K; ++k)
                for (int b = 0; b < 3; ++b) {
                    int64_t bit = 3 * k + b;
                    if ((codes_u[n * K + k] >> b) & 1) out[n * rb + bit / 8] |= (uint8_t)(1u << (bit % 8));
                }
    }
}

void orc_unpack_codes(const uint8_t* in, int64_t N, int64_t K, int bits, uint8_t* codes_u)
{
    if (bits == 8) {
        for (int64_t i = 0; i < N * K; ++i) codes_u[i] = (uint8_t)((int)(int8_t)in[i] + 128);
    } else if (bits == 4) {
        for (int64_t i = 0; i < N * K / 2; ++i) {
            codes_u[2 * i] = in[i] & 15;
            codes_u[2 * i + 1] = in[i] >> 4;
        }
    } else {
        const int64_t rb = 3 * K / 8;
        for (int64_t n = 0; n < N; ++n)
            for (int64_t k = 0; k < K; ++k) {
                int v = 0;
                for (int b = 0; b < 3; ++b) {
                    int64_t bit = 3 * k + b;
                    v |= ((in[n * rb + bit / 8] >> (bit % 8)) & 1) << b;
                }
                codes_u[n * K + k] = (uint8_t)v;
            }
    }
}

/* Weight after quantise -> de-quantise (the W-tilde of Sec. 3.3), binary32. */
void orc_dequant_weight(const uint8_t* codes_u, int64_t N, int64_t K, int64_t group,
                        const float* step, const int32_t* zero, float* W_tilde)
{
    const int64_t g = group > 0 ? group : K;
    const int64_t ng = K / g;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int64_t pi = group < 0 ? 0 : n * ng + k / g;
            W_tilde[n * K + k] = (float)((int32_t)codes_u[n * K + k] - zero[pi]) * step[pi];
        }
}

/* The same W-tilde as the binary16 operand a half-precision matrix unit consumes in the
 * weight-only forward (Sec. 4.2: INT3 / INT4 weights, FP16 activations): Step is first
 * rounded to binary16, the product (u - Z) * Step_h is one binary32 multiplication and the
 * result is rounded to binary16.  (For |u - Z| <= 2048 the product is exact in binary32,
 * so this is the correctly rounded binary16 value of (u - Z) * Step_h.) */
void orc_dequant_weight_h(const uint8_t* codes_u, int64_t N, int64_t K, int64_t group,
                          const float* step, const int32_t* zero, uint16_t* W_tilde_h)
{
    const int64_t g = group > 0 ? group : K;
    const int64_t ng = K / g;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            int64_t pi = group < 0 ? 0 : (group == 0 ? n : n * ng + k / g);
            float step_h = orc_h2f(orc_f2h(step[pi]));
            float w = (float)((int32_t)codes_u[n * K + k] - zero[pi]) * step_h;
            W_tilde_h[n * K + k] = orc_f2h(w);
        }
}

/* Weight-only forward: y[t,n] = sum_k x_hat[t,k] w~_h[n,k] + b[n] with binary16 operands,
 * summed here in fp64 in the order of k; abs_y[t,n] = sum_k |x_hat w~_h| (+ |b|) is the
 * magnitude a floating-point accumulation error bound scales with.  bias / abs_y nullable. */
void orc_wonly_forward(const uint16_t* X_hat_h, int64_t T, int64_t K, int64_t ldx,
                       const uint16_t* W_tilde_h, int64_t N, const float* bias,
                       double* y, double* abs_y)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, mag = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = (double)orc_h2f(X_hat_h[t * ldx + k]) * (double)orc_h2f(W_tilde_h[n * K + k]);
                acc += p;
                mag += fabs(p);
            }
            if (bias) { acc += (double)bias[n]; mag += fabs((double)bias[n]); }
            y[t * N + n] = acc;
            if (abs_y) abs_y[t * N + n] = mag;
        }
}

/* ------------------------------------------------------- stage 4: W8A8 activation + GEMM */

/* Static per-tensor int8 activation quantizer applied to X_hat = X * inv_s (Eq. 1 with
 * b = 8, Step/Z from the calibrated range of X_hat).  Stored as q = u - 128.
 * rowsum_x[t] = sum_k q[t,k] (int32), colsum_xq[k] = sum_t q[t,k] (int64). */
void orc_quant_act(const void* X, int dt, int64_t T, int64_t K, int64_t ldx,
                   const float* inv_s, float step_x, int32_t zero_x,
                   int8_t* xq, int32_t* rowsum_x, int64_t* colsum_xq, uint32_t* status)
{
    uint32_t st = 0;
#pragma omp parallel for schedule(static) reduction(| : st)
    for (int64_t t = 0; t < T; ++t) {
        int32_t rs = 0;
        for (int64_t k = 0; k < K; ++k) {
            float xh = ld_elt(X, dt, t * ldx + k) * inv_s[k];
            int32_t u = quant_one(xh, step_x, zero_x, 255, &st);
            xq[t * K + k] = (int8_t)(u - 128);
            rs += u - 128;
        }
        if (rowsum_x) rowsum_x[t] = rs;
    }
    if (colsum_xq)
#pragma omp parallel for schedule(static)
        for (int64_t k = 0; k < K; ++k) {
            int64_t cs = 0;
            for (int64_t t = 0; t < T; ++t) cs += xq[t * K + k];
            colsum_xq[k] = cs;
        }
    if (status) *status |= st;
}

/* acc[t,n] = sum_k xq[t,k] * wq[n,k], signed 8-bit operands, 32-bit accumulation
 * (|acc| <= 128*128*K < 2^31 for every K used here). */
void orc_gemm_i8(const int8_t* xq, const int8_t* wq, int64_t T, int64_t N, int64_t K,
                 int32_t* acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < N; ++n) {
            int32_t a = 0;
            for (int64_t k = 0; k < K; ++k) a += (int32_t)xq[t * K + k] * (int32_t)wq[n * K + k];
            acc[t * N + n] = a;
        }
}

/* One row of acc only (sampled checks at full size). */
void orc_gemm_i8_rows(const int8_t* xq_rows, const int8_t* wq, int64_t n_rows, int64_t N,
                      int64_t K, int32_t* acc)
{
    orc_gemm_i8(xq_rows, wq, n_rows, N, K, acc);
}

/* De-quantised output, direct form: y~[t,n] = Step_x Step_w[n] sum_k (xq - Z'x)(wq - Z'w[n])
 * + bias[n], with Z' = Z - 128 the zero point of the stored signed code.  fp64. */
void orc_w8a8_output_direct(const int8_t* xq, const int8_t* wq, int64_t T, int64_t N, int64_t K,
                            float step_x, int32_t zero_x, const float* step_w,
                            const int32_t* zero_w, const float* bias, double* out)
{
    const int64_t zx = (int64_t)zero_x - 128;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < N; ++n) {
            const int64_t zw = (int64_t)zero_w[n] - 128;
            int64_t a = 0;
            for (int64_t k = 0; k < K; ++k)
                a += ((int64_t)xq[t * K + k] - zx) * ((int64_t)wq[n * K + k] - zw);
            out[t * N + n] = (double)step_x * (double)step_w[n] * (double)a + (bias ? (double)bias[n] : 0.0);
        }
}

/* Same output from the raw accumulator and the row sums (the form a GEMM epilogue uses):
 * sum (xq-Z'x)(wq-Z'w) = acc - Z'x rowsum_w[n] - Z'w[n] rowsum_x[t] + K Z'x Z'w[n].
 * Also returns the integer so a test can assert exact agreement with the direct form. */
void orc_w8a8_output_expanded(const int32_t* acc, const int32_t* rowsum_x, const int32_t* rowsum_w,
                              int64_t T, int64_t N, int64_t K, float step_x, int32_t zero_x,
                              const float* step_w, const int32_t* zero_w, const float* bias,
                              double* out, int64_t* integer_out)
{
    const int64_t zx = (int64_t)zero_x - 128;
    for (int64_t t = 0; t < T; ++t)
        for (int64_t n = 0; n < N; ++n) {
            const int64_t zw = (int64_t)zero_w[n] - 128;
            int64_t a = (int64_t)acc[t * N + n] - zx * (int64_t)rowsum_w[n] - zw * (int64_t)rowsum_x[t] + K * zx * zw;
            if (integer_out) integer_out[t * N + n] = a;
            out[t * N + n] = (double)step_x * (double)step_w[n] * (double)a + (bias ? (double)bias[n] : 0.0);
        }
}

/* ------------------------------------------------------------- stage 5: bias correction */

/* Eq. 11, literal, W8A8: for every calibration token the FP output of the equalised layer
 * y[t,n] = sum_k X_hat[t,k] W_hat[n,k] and the output of the int8 path y~[t,n] (no bias)
 * are formed, both are averaged over the tokens, delta = mean(y) - mean(y~) and the
 * corrected bias is b' = b - E[y~ - y] = b + delta (Sec. 3.3). */
void orc_bias_literal_w8a8(const void* X, int dt, int64_t T, int64_t K, int64_t ldx,
                           const float* inv_s, const void* W_hat, int64_t N, int64_t ldw,
                           const int8_t* xq, const int8_t* wq, float step_x, int32_t zero_x,
                           const float* step_w, const int32_t* zero_w,
                           const float* bias_in, double* delta, float* bias_out)
{
    const int64_t zx = (int64_t)zero_x - 128;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const int64_t zw = (int64_t)zero_w[n] - 128;
        double sum_y = 0.0, sum_yq = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double y = 0.0;
            int64_t a = 0;
            for (int64_t k = 0; k < K; ++k) {
                float xh = ld_elt(X, dt, t * ldx + k) * inv_s[k];
                y += (double)xh * (double)ld_elt(W_hat, dt, n * ldw + k);
                a += ((int64_t)xq[t * K + k] - zx) * ((int64_t)wq[n * K + k] - zw);
            }
            sum_y += y;
            sum_yq += (double)step_x * (double)step_w[n] * (double)a;
        }
        double d = sum_y / (double)T - sum_yq / (double)T;
        delta[n] = d;
        if (bias_out) bias_out[n] = (float)((bias_in ? (double)bias_in[n] : 0.0) + d);
    }
}

/* Eq. 11, literal, weight-only: y~[t,n] = sum_k X_hat[t,k] W~[n,k] with W~ the
 * de-quantised weight and FP activations. */
void orc_bias_literal_wonly(const void* X, int dt, int64_t T, int64_t K, int64_t ldx,
                            const float* inv_s, const void* W_hat, int64_t N, int64_t ldw,
                            const float* W_tilde, const float* bias_in, double* delta, float* bias_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double sum_y = 0.0, sum_yq = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double y = 0.0, yq = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                float xh = ld_elt(X, dt, t * ldx + k) * inv_s[k];
                y += (double)xh * (double)ld_elt(W_hat, dt, n * ldw + k);
                yq += (double)xh * (double)W_tilde[n * K + k];
            }
            sum_y += y;
            sum_yq += yq;
        }
        double d = sum_y / (double)T - sum_yq / (double)T;
        delta[n] = d;
        if (bias_out) bias_out[n] = (float)((bias_in ? (double)bias_in[n] : 0.0) + d);
    }
}

/* W8A8 bias error through the linearity identities (used at sizes where the literal
 * form is out of reach; asserted against it on small shapes):
 *   mean_t y[t,n]  = sum_k W_hat[n,k] mu_xhat[k]
 *   sum_t  y~[t,n] = Step_x Step_w[n] (colsum_acc[n] - T Z'x rowsum_w[n]
 *                                      - Z'w[n] sum_k colsum_xq[k] + T K Z'x Z'w[n]).
 * enable_bc = 0 returns delta but leaves the bias unchanged (ablation switch). */
void orc_bias_w8a8(const void* W_hat, int dt, int64_t N, int64_t K, int64_t ldw,
                   const float* mu_xhat, uint64_t count, const int64_t* colsum_acc,
                   const int64_t* colsum_xq, const int32_t* rowsum_w, float step_x, int32_t zero_x,
                   const float* step_w, const int32_t* zero_w, const float* bias_in,
                   int enable_bc, double* delta, float* bias_out)
{
    const int64_t zx = (int64_t)zero_x - 128;
    const int64_t T = (int64_t)count;
    int64_t total_xq = 0;
    for (int64_t k = 0; k < K; ++k) total_xq += colsum_xq[k];
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const int64_t zw = (int64_t)zero_w[n] - 128;
        double ybar = 0.0;
        for (int64_t k = 0; k < K; ++k) ybar += (double)ld_elt(W_hat, dt, n * ldw + k) * (double)mu_xhat[k];
        int64_t a = colsum_acc[n] - T * zx * (int64_t)rowsum_w[n] - zw * total_xq + T * K * zx * zw;
        double yqbar = (double)step_x * (double)step_w[n] * (double)a / (double)T;
        double d = ybar - yqbar;
        delta[n] = d;
        if (bias_out) bias_out[n] = (float)((bias_in ? (double)bias_in[n] : 0.0) + (enable_bc ? d : 0.0));
    }
}

/* Weight-only bias error, Eq. 12-15: E[y~ - y] = eps E[x] with eps = W~ - W_hat, so
 * delta[n] = -sum_k (W~[n,k] - W_hat[n,k]) mu_xhat[k]. */
void orc_bias_wonly(const void* W_hat, int dt, int64_t N, int64_t K, int64_t ldw,
                    const float* mu_xhat, const uint8_t* codes_u, int64_t group,
                    const float* step_w, const int32_t* zero_w, const float* bias_in,
                    int enable_bc, double* delta, float* bias_out)
{
    const int64_t g = group > 0 ? group : K;
    const int64_t ng = K / g;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double e = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            int64_t pi = group < 0 ? 0 : n * ng + k / g;
            float wt = (float)((int32_t)codes_u[n * K + k] - zero_w[pi]) * step_w[pi];
            double eps = (double)wt - (double)ld_elt(W_hat, dt, n * ldw + k);
            e += eps * (double)mu_xhat[k];
        }
        delta[n] = -e;
        if (bias_out) bias_out[n] = (float)((bias_in ? (double)bias_in[n] : 0.0) + (enable_bc ? -e : 0.0));
    }
}

/* Exact integer identity used by the tests: sum_t acc[t,n] = sum_k wq[n,k] colsum_xq[k]. */
void orc_colsum_acc_from_colsum_xq(const int8_t* wq, int64_t N, int64_t K,
                                   const int64_t* colsum_xq, int64_t* colsum_acc)
{
    for (int64_t n = 0; n < N; ++n) {
        int64_t a = 0;
        for (int64_t k = 0; k < K; ++k) a += (int64_t)wq[n * K + k] * colsum_xq[k];
        colsum_acc[n] = a;
    }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
