/*
 * CPU oracle for the ViDiT-Q quantized linear layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
 * correct statement of what the quantized linear layer computes, used only by
 * the test-suite, the smoke check and the CPU-baseline leg of the benchmark.
 * It shares no source, header, table or helper with the HIP library.
 *
 * What it follows (ViDiT-Q, arxiv 2406.02540):
 *   - Sec. 3.1, Eq. 2: uniform b-bit quantizer x_int = clamp(round(x / s) + z).
 *     Used here in its symmetric form (z = 0, s = absmax / (2^(b-1) - 1),
 *     integers in [-(2^(b-1)-1), 2^(b-1)-1]), so the min-max range is
 *     [-absmax, absmax] and nothing is clipped.
 *   - Sec. 4.1: one parameter set per token for activations, computed online
 *     from the token itself (dynamic), and one per output channel for weights.
 *   - Sec. 4.2, Eq. 3: scaling-based channel balancing
 *     Y = (X diag(s)^-1)(diag(s) W); the activation side receives
 *     chan_mul[k] = 1/s_k, the weight side is multiplied by s_k before it is
 *     quantized.
 *   - Appendix "Hardware implementation of quantized linear layers": integer
 *     products are summed along the input channels first, the two scales
 *     (s_x of the token, s_w of the output channel) multiply the integer sum
 *     afterwards.
 *   - Appendix "Performance under lower bitwidth": W4A8 stores 4-bit weights
 *     and widens them to 8 bits for the same integer contraction.
 *
 * Arithmetic fixed where the paper is silent (every fp32 operation is rounded
 * on its own, round-to-nearest-even, no fused multiply-add, no reassociation;
 * build with -ffp-contract=off -fno-fast-math):
 *   - token statistics in fp32: t = float(x_f16) * chan_mul[k];
 *     amax = max |t|; x_scale = amax / 127; inv = 127 / amax (one reciprocal
 *     per token); q = clamp(rint(t * inv), -127, 127); rint rounds halves to
 *     even; a token of zeros gives x_scale = 0 and q = 0.
 *   - weights the same way per output channel with qmax 127 (int8) or 7 (int4).
 *   - the integer sum is taken in int64 and must fit int32.
 *   - y = fp16_rne( ((float)acc * x_scale[m]) * w_scale[n] + float(bias[n]) ).
 *
 *   - producers fused with the quantizer (Sec. 5.1 "Hardware Implementation
 *     Settings": the quantization is integrated into the preceding LayerNorm,
 *     GELU and residual operations).  The paper gives no formulas for them, so
 *     the textbook ones are used: LayerNorm over the channels of a token with
 *     the biased variance, followed by the DiT feature modulation
 *     (1 + scale) * y + shift of the token's sample; GELU x Phi(x), exactly or
 *     in its tanh form; residual r = x + gate * y.  LayerNorm and GELU are
 *     evaluated in fp64 and rounded once to fp32, and that fp32 row is quantized
 *     with the steps above; the residual is fp32 (one multiply, one add, each
 *     rounded), narrowed to fp16 as the new residual stream, and that fp16 row is
 *     quantized.
 *
 *   - rotation-based balancing, the "dynamic" half of Sec. 4.2: Y = X W^T =
 *     (X Q)(W Q)^T for an orthogonal Q; the paper takes a Hadamard matrix and
 *     fuses the transform with the quantizer (Sec. 5.1).  It does not say how a
 *     channel count that is not a power of two (1152 = 9 * 128) is handled;
 *     here Q is block diagonal with blocks H_B / sqrt(B), H_B the Sylvester
 *     Hadamard matrix H[k][c] = (-1)^popcount(k & c) in natural order, B = 128
 *     (or any power of two that divides K).  Scaling comes first, then the
 *     rotation: t = ((x * chan_mul) Q) for activations, (w * s) Q for weights.
 *     fp64 throughout, one rounding to fp32 at the end.
 *
 * Matrices are dense row-major: X[M,K], W[N,K] (K contiguous), Y[M,N].
 * fp16 values travel as uint16_t bit patterns.
 *
 * Every function here is pinned by tests that do not go through this file
 * (hand examples, closed-form error bounds, symmetries, brute-force sums,
 * numpy's own float16 conversion); none is "parity unpinned".
 */
#define _USE_MATH_DEFINES
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifndef M_PI
#define M_PI 3.14159265358979323846
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG 1
#define ORACLE_ERR_OVERFLOW 2

/* ---- IEEE binary16 <-> binary32, written out bit by bit ------------------ */

/* Exact widening of a binary16 bit pattern. */
float oracle_half_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t exp = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t man = (uint32_t)h & 0x3FFu;
    double v;
    if (exp == 0) {
        v = ldexp((double)man, -24);            /* zero and subnormals: man * 2^-24 */
    } else if (exp == 31) {
        v = man ? (double)NAN : (double)INFINITY;
    } else {
        v = ldexp((double)(man + 1024u), (int)exp - 25); /* (1 + man/1024) * 2^(exp-15) */
    }
    return (float)(sign ? -v : v);
}

/* Narrowing with round-to-nearest-even; overflow goes to infinity (no saturation). */
uint16_t oracle_float_to_half(float f) {
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7E00u);
    if (a == 0.0) return sign;
    /* The spacing of binary16 values around a: 2^(e-10) for normal range,
       2^-24 below 2^-14.  Dividing by it and rounding to an integer with
       ties-to-even (rint in the default rounding mode) is the RNE narrowing. */
    int e;
    (void)frexp(a, &e);          /* a = m * 2^e, m in [0.5, 1)  ->  a in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1) - 10;  /* exponent of one unit in the last place */
    if (ulp_exp < -24) ulp_exp = -24;
    double n = rint(ldexp(a, -ulp_exp)); /* integer count of ulps, exact in double */
    double r = ldexp(n, ulp_exp);        /* the rounded value */
    if (r >= 65520.0) return (uint16_t)(sign | 0x7C00u); /* beyond the largest finite + half ulp */
    if (isinf(f)) return (uint16_t)(sign | 0x7C00u);
    /* encode r */
    if (r < ldexp(1.0, -14)) {
        return (uint16_t)(sign | (uint16_t)ldexp(r, 24)); /* subnormal: mantissa = r / 2^-24 */
    }
    int re;
    double rm = frexp(r, &re);                 /* r = rm * 2^re, rm in [0.5,1) */
    uint32_t mant = (uint32_t)ldexp(rm, 11) - 1024u; /* (2*rm - 1) * 1024 */
    uint32_t bexp = (uint32_t)(re - 1 + 15);
    return (uint16_t)(sign | (bexp << 10) | mant);
}

/* ---- Sec. 4.1 + Eq. 2 + Eq. 3: dynamic per-token activation quantizer ---- */

int oracle_quantize_per_token(const uint16_t* x_f16, const float* chan_mul,
                              int8_t* xq, float* x_scale, int64_t M, int64_t K) {
    if (!x_f16 || !xq || !x_scale || M < 0 || K <= 0) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t* row = x_f16 + m * K;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float t = oracle_half_to_float(row[k]);
            if (chan_mul) t = t * chan_mul[k];      /* X diag(s)^-1, Eq. 3 */
            float a = fabsf(t);
            if (a > amax) amax = a;
        }
        float scale = 0.0f, inv = 0.0f;
        if (amax != 0.0f) {
            scale = amax / 127.0f;                  /* s of Eq. 2, symmetric min-max */
            inv = 127.0f / amax;
        }
        x_scale[m] = scale;
        for (int64_t k = 0; k < K; ++k) {
            float t = oracle_half_to_float(row[k]);
            if (chan_mul) t = t * chan_mul[k];
            float q = rintf(t * inv);               /* round to nearest, halves to even */
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            xq[m * K + k] = (int8_t)q;
        }
    }
    return ORACLE_OK;
}

/* ---- producers fused with the quantizer (Sec. 5.1, hardware implementation) ----
 * A fused kernel never writes the producer's output: it quantizes it in
 * registers.  Here each producer is a function of its own that writes the row
 * it would hand to the quantizer, so that a test can look at it.              */

/* The quantizer steps of oracle_quantize_per_token on a row that already is fp32. */
int oracle_quantize_rows_f32(const float* t_f32, const float* chan_mul,
                             int8_t* xq, float* x_scale, int64_t M, int64_t K) {
    if (!t_f32 || !xq || !x_scale || M < 0 || K <= 0) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float* row = t_f32 + m * K;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float t = row[k];
            if (chan_mul) t = t * chan_mul[k];
            float a = fabsf(t);
            if (a > amax) amax = a;
        }
        float scale = 0.0f, inv = 0.0f;
        if (amax != 0.0f) {
            scale = amax / 127.0f;
            inv = 127.0f / amax;
        }
        x_scale[m] = scale;
        for (int64_t k = 0; k < K; ++k) {
            float t = row[k];
            if (chan_mul) t = t * chan_mul[k];
            float q = rintf(t * inv);
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            xq[m * K + k] = (int8_t)q;
        }
    }
    return ORACLE_OK;
}

/* GELU(x) = x * Phi(x) with Phi the standard normal distribution function.
 * approximate == 0: Phi(x) = (1 + erf(x / sqrt 2)) / 2.
 * approximate == 1: the tanh form, Phi(x) ~ (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) / 2.
 * fp64 throughout, one rounding to fp32 at the end.                            */
int oracle_gelu(const uint16_t* h_f16, int approximate, float* t_f32, int64_t M, int64_t K) {
    if (!h_f16 || !t_f32 || M < 0 || K <= 0 || (approximate != 0 && approximate != 1))
        return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M * K; ++i) {
        const double x = (double)oracle_half_to_float(h_f16[i]);
        double phi;
        if (approximate == 0)
            phi = 0.5 * (1.0 + erf(x / sqrt(2.0)));
        else
            phi = 0.5 * (1.0 + tanh(sqrt(2.0 / M_PI) * (x + 0.044715 * x * x * x)));
        t_f32[i] = (float)(x * phi);
    }
    return ORACLE_OK;
}

/* LayerNorm of every token over its K channels (mean and biased variance of the
 * token, eps inside the square root, no learned affine), then the modulation of
 * the token's sample b = m / tokens_per_sample: (1 + scale[b,k]) * y + shift[b,k].
 * scale and shift are fp32 [ceil(M / tokens_per_sample), K]; either may be NULL
 * (no scaling, no shift).  fp64 throughout, one rounding to fp32 at the end.    */
int oracle_layernorm_modulate(const uint16_t* x_f16, const float* scale, const float* shift,
                              int64_t tokens_per_sample, double eps, float* t_f32,
                              int64_t M, int64_t K) {
    if (!x_f16 || !t_f32 || M < 0 || K <= 0 || tokens_per_sample <= 0 || !(eps >= 0.0))
        return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const uint16_t* row = x_f16 + m * K;
        const int64_t b = m / tokens_per_sample;
        double mean = 0.0;
        for (int64_t k = 0; k < K; ++k) mean += (double)oracle_half_to_float(row[k]);
        mean /= (double)K;
        double var = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double d = (double)oracle_half_to_float(row[k]) - mean;
            var += d * d;
        }
        var /= (double)K;
        const double rstd = 1.0 / sqrt(var + eps);
        for (int64_t k = 0; k < K; ++k) {
            double y = ((double)oracle_half_to_float(row[k]) - mean) * rstd;
            if (scale) y = y * (1.0 + (double)scale[b * K + k]);
            if (shift) y = y + (double)shift[b * K + k];
            t_f32[m * K + k] = (float)y;
        }
    }
    return ORACLE_OK;
}

/* Residual connection r = x + gate * y with the gate of the token's sample
 * (fp32 [ceil(M / tokens_per_sample), K], NULL for 1): fp32, the product rounded,
 * then the sum rounded, then narrowed to fp16 -- the new residual stream.       */
int oracle_residual(const uint16_t* x_f16, const uint16_t* y_f16, const float* gate,
                    int64_t tokens_per_sample, uint16_t* r_f16, int64_t M, int64_t K) {
    if (!x_f16 || !y_f16 || !r_f16 || M < 0 || K <= 0 || tokens_per_sample <= 0)
        return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const int64_t b = m / tokens_per_sample;
        for (int64_t k = 0; k < K; ++k) {
            float p = oracle_half_to_float(y_f16[m * K + k]);
            if (gate) p = gate[b * K + k] * p;
            const float r = oracle_half_to_float(x_f16[m * K + k]) + p;
            r_f16[m * K + k] = oracle_float_to_half(r);
        }
    }
    return ORACLE_OK;
}

/* ---- Sec. 4.1 + Eq. 2 + Eq. 3: per-output-channel weight quantizer ------- */

int oracle_quantize_weight(const float* w, const float* chan_s, int bits,
                           int8_t* wq, float* w_scale, int64_t N, int64_t K) {
    if (!w || !wq || !w_scale || N < 0 || K <= 0) return ORACLE_ERR_ARG;
    if (bits != 8 && bits != 4) return ORACLE_ERR_ARG;
    const float qmax = (bits == 8) ? 127.0f : 7.0f;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float* row = w + n * K;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float t = row[k];
            if (chan_s) t = t * chan_s[k];          /* diag(s) W, Eq. 3 */
            float a = fabsf(t);
            if (a > amax) amax = a;
        }
        float scale = 0.0f, inv = 0.0f;
        if (amax != 0.0f) {
            scale = amax / qmax;
            inv = qmax / amax;
        }
        w_scale[n] = scale;
        for (int64_t k = 0; k < K; ++k) {
            float t = row[k];
            if (chan_s) t = t * chan_s[k];
            float q = rintf(t * inv);
            if (q > qmax) q = qmax;
            if (q < -qmax) q = -qmax;
            wq[n * K + k] = (int8_t)q;
        }
    }
    return ORACLE_OK;
}

/* ---- 4-bit storage: two's-complement nibbles, two per byte along K ------- */
/* byte j of a row holds k = 2j in bits 0..3 and k = 2j+1 in bits 4..7.       */

int oracle_pack_int4(const int8_t* wq, uint8_t* packed, int64_t N, int64_t K) {
    if (!wq || !packed || N < 0 || K <= 0 || (K & 1)) return ORACLE_ERR_ARG;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j) {
            int lo = wq[n * K + 2 * j], hi = wq[n * K + 2 * j + 1];
            if (lo < -8 || lo > 7 || hi < -8 || hi > 7) return ORACLE_ERR_ARG;
            packed[n * (K / 2) + j] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
        }
    return ORACLE_OK;
}

static int8_t nibble_value(unsigned nib) { /* 4-bit two's complement */
    return (int8_t)((nib & 8u) ? (int)nib - 16 : (int)nib);
}

int oracle_unpack_int4(const uint8_t* packed, int8_t* wq, int64_t N, int64_t K) {
    if (!wq || !packed || N < 0 || K <= 0 || (K & 1)) return ORACLE_ERR_ARG;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t b = packed[n * (K / 2) + j];
            wq[n * K + 2 * j] = nibble_value(b & 0xFu);
            wq[n * K + 2 * j + 1] = nibble_value((unsigned)b >> 4);
        }
    return ORACLE_OK;
}

/* ---- integer contraction along the input channels ------------------------ */

int oracle_gemm_i8(const int8_t* xq, const int8_t* wq, int32_t* acc,
                   int64_t M, int64_t N, int64_t K) {
    if (!xq || !wq || !acc || M < 0 || N < 0 || K <= 0) return ORACLE_ERR_ARG;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)xq[m * K + k] * (int64_t)wq[n * K + k];
            if (s > INT32_MAX || s < INT32_MIN) overflow |= 1;
            acc[m * N + n] = (int32_t)s;
        }
    return overflow ? ORACLE_ERR_OVERFLOW : ORACLE_OK;
}

/* ---- dequantization: the two scales, then the bias, then fp16 ------------ */

int oracle_dequant(const int32_t* acc, const float* x_scale, const float* w_scale,
                   const uint16_t* bias_f16, uint16_t* y_f16, int64_t M, int64_t N) {
    if (!acc || !x_scale || !w_scale || !y_f16 || M < 0 || N < 0) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float yf = (float)acc[m * N + n] * x_scale[m];
            yf = yf * w_scale[n];
            if (bias_f16) yf = yf + oracle_half_to_float(bias_f16[n]);
            y_f16[m * N + n] = oracle_float_to_half(yf);
        }
    return ORACLE_OK;
}

/* ---- Eq. 3 (Sec. 4.2): the balancing mask from absmax statistics ------------------
 * s_i = max|X_i|^alpha / max|W_i|^(1 - alpha) for every input channel i, the maxima
 * taken over the tokens of the calibration activations and over the output channels
 * of the weight.  Statistics below 1e-5 are raised to 1e-5 and s is kept within
 * [1e-5, 1e5] (a channel that is all zero must not produce 0 or infinity; the paper
 * does not treat the case).  chan_mul_i = 1 / s_i in fp32 is what the quantizers take. */

int oracle_channel_absmax_f16(const uint16_t* x_f16, float* amax, int64_t M, int64_t K) {
    if (!x_f16 || !amax || M < 0 || K <= 0) return ORACLE_ERR_ARG;
    for (int64_t k = 0; k < K; ++k) amax[k] = 0.0f;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            const float a = fabsf(oracle_half_to_float(x_f16[m * K + k]));
            if (a > amax[k]) amax[k] = a;
        }
    return ORACLE_OK;
}

int oracle_channel_absmax_f32(const float* w, float* amax, int64_t N, int64_t K) {
    if (!w || !amax || N < 0 || K <= 0) return ORACLE_ERR_ARG;
    for (int64_t k = 0; k < K; ++k) amax[k] = 0.0f;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const float a = fabsf(w[n * K + k]);
            if (a > amax[k]) amax[k] = a;
        }
    return ORACLE_OK;
}

int oracle_balance_mask(const float* amax_x, const float* amax_w, double alpha, float* s_out,
                        float* chan_mul_out, int64_t K) {
    if (!amax_x || !amax_w || !s_out || !chan_mul_out || K <= 0 || !(alpha >= 0.0 && alpha <= 1.0))
        return ORACLE_ERR_ARG;
    for (int64_t k = 0; k < K; ++k) {
        const double ax = amax_x[k] > 1e-5f ? (double)amax_x[k] : 1e-5;
        const double aw = amax_w[k] > 1e-5f ? (double)amax_w[k] : 1e-5;
        double s = pow(ax, alpha) / pow(aw, 1.0 - alpha);
        if (s < 1e-5) s = 1e-5;
        if (s > 1e5) s = 1e5;
        s_out[k] = (float)s;
        chan_mul_out[k] = 1.0f / s_out[k];
    }
    return ORACLE_OK;
}

/* ---- rotation-based balancing (Sec. 4.2), block-diagonal Hadamard matrix ---------- */

static int parity_of(uint64_t v) { /* popcount mod 2 */
    int p = 0;
    while (v) { p ^= 1; v &= v - 1; }
    return p;
}

/* rows [M,K] (fp64 values supplied by get(m,k)) times Q, written out as fp32. */
static void rotate_rows(const double* in, float* out, int64_t M, int64_t K, int64_t B) {
    const double norm = 1.0 / sqrt((double)B);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t b0 = 0; b0 < K; b0 += B) {
            for (int64_t c = 0; c < B; ++c) {
                double sum = 0.0;
                for (int64_t k = 0; k < B; ++k) {
                    const double v = in[m * K + b0 + k];
                    sum += parity_of((uint64_t)(k & c)) ? -v : v;
                }
                out[m * K + b0 + c] = (float)(sum * norm);
            }
        }
    }
}

static int bad_block(int64_t K, int64_t B) { return B <= 0 || (B & (B - 1)) != 0 || K % B != 0; }

/* Activations: t[m,:] = (float(x[m,:]) * chan_mul) Q, block size B. `scratch` is M*K doubles. */
int oracle_hadamard_rotate(const uint16_t* x_f16, const float* chan_mul, int64_t B, float* t_f32,
                           double* scratch, int64_t M, int64_t K) {
    if (!x_f16 || !t_f32 || !scratch || M < 0 || K <= 0 || bad_block(K, B)) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < M * K; ++i) {
        double v = (double)oracle_half_to_float(x_f16[i]);
        if (chan_mul) v = v * (double)chan_mul[i % K];
        scratch[i] = v;
    }
    rotate_rows(scratch, t_f32, M, K, B);
    return ORACLE_OK;
}

/* Weights: w'[n,:] = (w[n,:] * s) Q, the counterpart that keeps X W^T unchanged. */
int oracle_rotate_weight(const float* w, const float* chan_s, int64_t B, float* w_rot,
                         double* scratch, int64_t N, int64_t K) {
    if (!w || !w_rot || !scratch || N < 0 || K <= 0 || bad_block(K, B)) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N * K; ++i) {
        double v = (double)w[i];
        if (chan_s) v = v * (double)chan_s[i % K];
        scratch[i] = v;
    }
    rotate_rows(scratch, w_rot, N, K, B);
    return ORACLE_OK;
}

/* ---- comparison points of Sec. 5.3 "Hardware Resource Savings" -----------------
 * The paper measures its INT8 layers against FP16 layers (about 2x) and against a
 * "naive" W8A8 baseline without dynamic, fine-grained parameters.  Both are
 * stated here so that the GPU counterparts can be checked.                      */

/* FP16 linear layer: y[m,n] = fp16( sum_k x[m,k] w[n,k] + bias[n] ), the sum in fp64
 * (the products of two fp16 values are exact in fp64).                           */
int oracle_gemm_f16(const uint16_t* x_f16, const uint16_t* w_f16, const uint16_t* bias_f16,
                    uint16_t* y_f16, int64_t M, int64_t N, int64_t K) {
    if (!x_f16 || !w_f16 || !y_f16 || M < 0 || N < 0 || K <= 0) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double sum = 0.0;
            for (int64_t k = 0; k < K; ++k)
                sum += (double)oracle_half_to_float(x_f16[m * K + k]) *
                       (double)oracle_half_to_float(w_f16[n * K + k]);
            if (bias_f16) sum += (double)oracle_half_to_float(bias_f16[n]);
            y_f16[m * N + n] = oracle_float_to_half((float)sum);
        }
    }
    return ORACLE_OK;
}

/* Static activation quantizer: one scale for the whole tensor, fixed beforehand
 * (Sec. 4.1 describes it as what dynamic token-wise parameters replace).
 * inv = 1 / scale once in fp32; q = clamp(rint(t * inv), -127, 127) with
 * t = float(x) * chan_mul[k]: values beyond 127 * scale are clipped.              */
int oracle_quantize_static(const uint16_t* x_f16, const float* chan_mul, float scale,
                           int8_t* xq, int64_t M, int64_t K) {
    if (!x_f16 || !xq || M < 0 || K <= 0 || !(scale > 0.0f)) return ORACLE_ERR_ARG;
    const float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t k = 0; k < K; ++k) {
            float t = oracle_half_to_float(x_f16[m * K + k]);
            if (chan_mul) t = t * chan_mul[k];
            float q = rintf(t * inv);
            if (q > 127.0f) q = 127.0f;
            if (q < -127.0f) q = -127.0f;
            xq[m * K + k] = (int8_t)q;
        }
    }
    return ORACLE_OK;
}

/* ---- the whole layer, steps in the order above ---------------------------
 * w is int8 [N,K] when w_bits == 8, packed nibbles [N,K/2] when w_bits == 4.
 * xq_out [M,K], x_scale_out [M] and acc_out [M,N] are caller scratch and are
 * left filled so that a test can compare the intermediate integers too.
 * wq_unpacked [N,K] is scratch for the widened weights (used when w_bits == 4).
 */
int oracle_linear(const uint16_t* x_f16, const float* chan_mul, const void* w, int w_bits,
                  const float* w_scale, const uint16_t* bias_f16, uint16_t* y_f16,
                  int8_t* xq_out, float* x_scale_out, int32_t* acc_out, int8_t* wq_unpacked,
                  int64_t M, int64_t N, int64_t K) {
    int rc = oracle_quantize_per_token(x_f16, chan_mul, xq_out, x_scale_out, M, K);
    if (rc) return rc;
    const int8_t* wq8;
    if (w_bits == 8) {
        wq8 = (const int8_t*)w;
    } else if (w_bits == 4) {
        if (!wq_unpacked) return ORACLE_ERR_ARG;
        rc = oracle_unpack_int4((const uint8_t*)w, wq_unpacked, N, K);
        if (rc) return rc;
        wq8 = wq_unpacked;
    } else {
        return ORACLE_ERR_ARG;
    }
    rc = oracle_gemm_i8(xq_out, wq8, acc_out, M, N, K);
    if (rc) return rc;
    return oracle_dequant(acc_out, x_scale_out, w_scale, bias_f16, y_f16, M, N);
}
