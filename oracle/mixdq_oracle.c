/*
 * CPU oracle for the quantized-linear path of MixDQ (arxiv 2405.17873).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
 * correct statement of what the path computes.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code with the
 * HIP kernels and the HIP path never falls back to it.
 *
 * What the paper fixes (Sec. 4.1 "Quantization Scheme"): a uniform asymmetric
 * min-max quantiser whose scale and zero point are shared per tensor for
 * activations and per output channel for weights; layer-granular bit-widths
 * (Sec. 3.3, Sec. 4.1 "Mixed Precision Allocation"); the BOS token of the text
 * embedding is kept out of quantisation and its to_k/to_v output is taken in
 * floating point and concatenated with the dequantised outputs of the other
 * tokens (Sec. 3.1); weight-only layers keep FP16 compute (App. C item 2);
 * W8A8/W4A8 layers run an integer GEMM after an FP16->INT8 conversion
 * (Sec. 4.3, App. C item 4).
 *
 * The paper prints no formula, rounding mode or packing layout.  The readings
 * taken here (each one is listed with its reason in the design document):
 *   - the quantisation range always contains 0;
 *   - scale = (hi - lo) / qmax in fp32, one reciprocal, one fp32 multiply per
 *     element, round-half-to-even, zero point clamped into [0, qmax];
 *   - a constant-zero tensor gets scale 1, zero point 0;
 *   - symmetric variant: scale = absmax / (2^(b-1) - 1), codes in [-Q, Q];
 *   - packing: per row a little-endian bit stream, code k at bits [k*b, k*b+b);
 *   - floating point accumulation in fp64, one rounding to the 16-bit output.
 *
 * Every operation of the weight and activation quantisers that decides an
 * integer code is a single IEEE fp32 operation; build with -ffp-contract=off
 * and without -ffast-math.  The gated feed-forward extension is stated in
 * fp64 with the C library's erf (see there for how its codes are compared).
 *
 * All functions return 0 on success, a negative value on a bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_BAD_ARG (-1)
#define ORC_OVERFLOW (-2)

#define ORC_F16 0
#define ORC_BF16 1

/* ------------------------------------------------------------------------- */
/* 16-bit float formats (IEEE binary16 and bfloat16), written out by hand.   */
/* ------------------------------------------------------------------------- */

/* binary16 -> double, exact. */
static double half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)m, -24); /* subnormal: m * 2^-24 */
    } else if (e == 31) {
        v = m ? NAN : INFINITY;
    } else {
        v = ldexp((double)(m + 1024), e - 25); /* (1 + m/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

/* double -> binary16, one round-half-to-even rounding. */
static uint16_t double_to_half(double v) {
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isnan(v)) return (uint16_t)(sign | 0x7e00);
    if (a == 0.0) return sign;
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00); /* rounds to infinity */
    if (a < 6.103515625e-05) {                          /* below 2^-14: subnormal grid 2^-24 */
        double q = rint(ldexp(a, 24));                  /* 0 .. 1024; 1024 is the least normal */
        return (uint16_t)(sign | (uint16_t)q);
    }
    int e2;
    (void)frexp(a, &e2); /* a = f * 2^e2, f in [0.5,1) -> exponent e = e2-1 */
    int e = e2 - 1;
    double frac = ldexp(a, -e) - 1.0;      /* in [0,1) */
    double q = rint(ldexp(frac, 10));      /* 0 .. 1024 */
    int m = (int)q;
    if (m == 1024) { m = 0; e += 1; }
    if (e > 15) return (uint16_t)(sign | 0x7c00);
    return (uint16_t)(sign | ((e + 15) << 10) | m);
}

/* bfloat16 -> double, exact (bfloat16 is the top half of a binary32). */
static double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* double -> bfloat16, one round-half-to-even rounding (8 significant bits). */
static uint16_t double_to_bf16(double v) {
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isnan(v)) return (uint16_t)(sign | 0x7fc0);
    if (a == 0.0) return sign;
    if (isinf(v)) return (uint16_t)(sign | 0x7f80);
    int e2;
    (void)frexp(a, &e2);
    int e = e2 - 1;
    if (e < -126) { /* subnormal grid 2^-133 */
        double q = rint(ldexp(a, 133));
        return (uint16_t)(sign | (uint16_t)q);
    }
    double frac = ldexp(a, -e) - 1.0;
    double q = rint(ldexp(frac, 7));
    int m = (int)q;
    if (m == 128) { m = 0; e += 1; }
    if (e > 127) return (uint16_t)(sign | 0x7f80);
    return (uint16_t)(sign | ((e + 127) << 7) | m);
}

static double in16(uint16_t v, int dtype) { return dtype == ORC_BF16 ? bf16_to_double(v) : half_to_double(v); }
static uint16_t out16(double v, int dtype) { return dtype == ORC_BF16 ? double_to_bf16(v) : double_to_half(v); }

/* Exposed so that the tests can pin the conversions against an independent library. */
int orc_f16_to_f64(const uint16_t* in, double* out, long n, int dtype) {
    if (!in || !out || n < 0) return ORC_BAD_ARG;
    for (long i = 0; i < n; ++i) out[i] = in16(in[i], dtype);
    return ORC_OK;
}
int orc_f64_to_f16(const double* in, uint16_t* out, long n, int dtype) {
    if (!in || !out || n < 0) return ORC_BAD_ARG;
    for (long i = 0; i < n; ++i) out[i] = out16(in[i], dtype);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Uniform min-max quantiser (Sec. 4.1 "Quantization Scheme").                */
/* ------------------------------------------------------------------------- */

static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* Asymmetric parameters from the observed minimum and maximum.
 * The range is widened to contain 0 so that 0 is a code.                     */
int orc_asym_params(float xmin, float xmax, int bits, float* scale, int32_t* zp) {
    if (bits < 1 || bits > 8 || !scale || !zp) return ORC_BAD_ARG;
    int qmax = (1 << bits) - 1;
    float lo = xmin < 0.0f ? xmin : 0.0f;
    float hi = xmax > 0.0f ? xmax : 0.0f;
    float s;
    if (hi == lo) {
        s = 1.0f;
    } else {
        float range = hi - lo;
        s = range / (float)qmax;
    }
    float inv = 1.0f / s;
    float zf = rintf((-lo) * inv);
    *scale = s;
    *zp = clampi((int)zf, 0, qmax);
    return ORC_OK;
}

/* One element: code = clamp(rne(x / s) + z, 0, qmax), with x / s taken as one
 * fp32 multiply by the reciprocal of s.  The guard keeps the float->int
 * conversion defined for values far outside the range; it cannot change a code. */
static int asym_code(float x, float inv, int z, int qmax) {
    float r = rintf(x * inv);
    if (r > 1.0e6f) r = 1.0e6f;
    if (r < -1.0e6f) r = -1.0e6f;
    return clampi((int)r + z, 0, qmax);
}

static int sym_code(float x, float inv, int Q) {
    float r = rintf(x * inv);
    if (r > 1.0e6f) r = 1.0e6f;
    if (r < -1.0e6f) r = -1.0e6f;
    return clampi((int)r, -Q, Q);
}

/* Weights W[N,K] (row = output channel), per-row parameters.
 * symmetric == 0: codes are unsigned in [0, 2^bits - 1], zp in the same range.
 * symmetric == 1: codes are two's complement int8 in [-Q, Q], Q = 2^(bits-1)-1, zp = 0. */
int orc_quantize_weights(const uint16_t* w, int N, int K, int bits, int symmetric, int dtype,
                         uint8_t* codes, float* scale, int32_t* zp) {
    if (!w || !codes || !scale || !zp || N <= 0 || K <= 0) return ORC_BAD_ARG;
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return ORC_BAD_ARG;
    for (int n = 0; n < N; ++n) {
        const uint16_t* row = w + (size_t)n * K;
        float mn = (float)in16(row[0], dtype), mx = mn, amax = fabsf(mn);
        for (int k = 1; k < K; ++k) {
            float v = (float)in16(row[k], dtype);
            if (v < mn) mn = v;
            if (v > mx) mx = v;
            if (fabsf(v) > amax) amax = fabsf(v);
        }
        if (symmetric) {
            int Q = (1 << (bits - 1)) - 1;
            float s = (amax == 0.0f) ? 1.0f : amax / (float)Q;
            float inv = 1.0f / s;
            scale[n] = s;
            zp[n] = 0;
            for (int k = 0; k < K; ++k)
                codes[(size_t)n * K + k] = (uint8_t)(int8_t)sym_code((float)in16(row[k], dtype), inv, Q);
        } else {
            int qmax = (1 << bits) - 1;
            float s;
            int32_t z;
            orc_asym_params(mn, mx, bits, &s, &z);
            float inv = 1.0f / s;
            scale[n] = s;
            zp[n] = z;
            for (int k = 0; k < K; ++k)
                codes[(size_t)n * K + k] = (uint8_t)asym_code((float)in16(row[k], dtype), inv, z, qmax);
        }
    }
    return ORC_OK;
}

/* Per-tensor 8-bit activation parameters over the M x K view with row stride ldx. */
int orc_act_params(const uint16_t* x, long M, int K, long ldx, int dtype, float* scale, int32_t* zp) {
    if (!x || M <= 0 || K <= 0 || ldx < K || !scale || !zp) return ORC_BAD_ARG;
    float mn = (float)in16(x[0], dtype), mx = mn;
    for (long m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k) {
            float v = (float)in16(x[m * ldx + k], dtype);
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
    return orc_asym_params(mn, mx, 8, scale, zp);
}

/* Unsigned 8-bit activation codes with the given parameters. */
int orc_act_quantize(const uint16_t* x, long M, int K, long ldx, int dtype, float scale, int32_t zp, uint8_t* qx) {
    if (!x || !qx || M <= 0 || K <= 0 || ldx < K || !(scale > 0.0f) || zp < 0 || zp > 255) return ORC_BAD_ARG;
    float inv = 1.0f / scale;
    for (long m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k)
            qx[m * (long)K + k] = (uint8_t)asym_code((float)in16(x[m * ldx + k], dtype), inv, zp, 255);
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Canonical packing: each row is a little-endian bit stream.                 */
/* ------------------------------------------------------------------------- */

long orc_packed_row_bytes(int K, int bits) {
    if (K <= 0 || (bits != 2 && bits != 3 && bits != 4 && bits != 8)) return ORC_BAD_ARG;
    if (((long)K * bits) % 8 != 0) return ORC_BAD_ARG;
    return (long)K * bits / 8;
}

int orc_pack_weights(const uint8_t* codes, int N, int K, int bits, uint8_t* packed) {
    long rb = orc_packed_row_bytes(K, bits);
    if (!codes || !packed || N <= 0 || rb < 0) return ORC_BAD_ARG;
    unsigned mask = (1u << bits) - 1u;
    memset(packed, 0, (size_t)N * rb);
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            unsigned c = codes[(size_t)n * K + k] & mask;
            for (int b = 0; b < bits; ++b) {
                long bit = (long)k * bits + b; /* position in the row's bit string */
                if ((c >> b) & 1u) packed[(size_t)n * rb + bit / 8] |= (uint8_t)(1u << (bit % 8));
            }
        }
    return ORC_OK;
}

int orc_unpack_weights(const uint8_t* packed, int N, int K, int bits, uint8_t* codes) {
    long rb = orc_packed_row_bytes(K, bits);
    if (!codes || !packed || N <= 0 || rb < 0) return ORC_BAD_ARG;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            unsigned c = 0;
            for (int b = 0; b < bits; ++b) {
                long bit = (long)k * bits + b;
                if ((packed[(size_t)n * rb + bit / 8] >> (bit % 8)) & 1u) c |= 1u << b;
            }
            codes[(size_t)n * K + k] = (uint8_t)c;
        }
    return ORC_OK;
}

/* Per-channel sum of codes over k (the quantity an integer epilogue needs). */
int orc_code_rowsum(const uint8_t* codes, int N, int K, int is_signed, int32_t* rowsum) {
    if (!codes || !rowsum || N <= 0 || K <= 0) return ORC_BAD_ARG;
    for (int n = 0; n < N; ++n) {
        int64_t s = 0;
        for (int k = 0; k < K; ++k)
            s += is_signed ? (int)(int8_t)codes[(size_t)n * K + k] : (int)codes[(size_t)n * K + k];
        rowsum[n] = (int32_t)s;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Linear layers.  rows == NULL: all M rows, y is [M, ldy].                   */
/* rows != NULL: only the listed rows of x, y (and acc) are compact [nrows,.] */
/* residual != NULL: a 16-bit [M, ldr] operand (indexed by the row of x, not */
/* by the position in `rows`) added to the sum before its single rounding.   */
/* It carries the skip connection of a block, and the first half of a layer  */
/* whose channel-concatenated input [trunk | shortcut] is split into two     */
/* layers with their own quantisation parameters (Sec. 4.1, "Quantization    */
/* Scheme": the two parts have different ranges); the second call then adds  */
/* the first call's output.                                                  */
/* ------------------------------------------------------------------------- */

/* Weight-only (App. C item 2: floating-point compute on dequantised weights):
 * w_hat[n,k] = s[n] * (q[n,k] - z[n]);  y[m,n] = round16( sum_k x[m,k] w_hat[n,k] + bias[n] ). */
int orc_linear_w_only(const uint16_t* x, long M, int K, long ldx, const uint8_t* codes, int N,
                      const float* w_scale, const int32_t* w_zp, const uint16_t* bias, int dtype,
                      uint16_t* y, long ldy, const int64_t* rows, long nrows, const uint16_t* residual, long ldr) {
    if (!x || !codes || !w_scale || !w_zp || !y || M <= 0 || K <= 0 || N <= 0 || ldx < K || ldy < N)
        return ORC_BAD_ARG;
    long R = rows ? nrows : M;
    if (R <= 0) return ORC_BAD_ARG;
    double* what = (double*)malloc((size_t)N * K * sizeof(double));
    if (!what) return ORC_BAD_ARG;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            what[(size_t)n * K + k] = (double)w_scale[n] * (double)((int)codes[(size_t)n * K + k] - w_zp[n]);
#pragma omp parallel for schedule(static)
    for (long r = 0; r < R; ++r) {
        long m = rows ? rows[r] : r;
        double* xr = (double*)malloc((size_t)K * sizeof(double));
        for (int k = 0; k < K; ++k) xr[k] = in16(x[m * ldx + k], dtype);
        for (int n = 0; n < N; ++n) {
            const double* wr = what + (size_t)n * K;
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += xr[k] * wr[k];
            if (bias) acc += in16(bias[n], dtype);
            if (residual) acc += in16(residual[m * ldr + n], dtype); /* y = linear(x) + residual, one rounding */
            y[r * ldy + n] = out16(acc, dtype);
        }
        free(xr);
    }
    free(what);
    return ORC_OK;
}

/* Plain 16-bit floating-point linear with unquantised weights W[N,K] (used for the BOS row). */
int orc_linear_fp(const uint16_t* x, long M, int K, long ldx, const uint16_t* w, int N,
                  const uint16_t* bias, int dtype, uint16_t* y, long ldy, const uint16_t* residual, long ldr) {
    if (!x || !w || !y || M <= 0 || K <= 0 || N <= 0 || ldx < K || ldy < N) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += in16(x[m * ldx + k], dtype) * in16(w[(size_t)n * K + k], dtype);
            if (bias) acc += in16(bias[n], dtype);
            if (residual) acc += in16(residual[m * ldr + n], dtype);
            y[m * ldy + n] = out16(acc, dtype);
        }
    return ORC_OK;
}

/* 8-bit-activation linear (Sec. 4.3: integer GEMM after the FP16->INT8 conversion).
 *   qx     = quantise(x; s_x, z_x)  per tensor, unsigned 8 bit
 *   ACC    = sum_k (qx[m,k] - z_x) * (qw[n,k] - z_w[n])          int32, compared bit-exact
 *   y      = round16( ACC * s_x * s_w[n] + bias[n] )
 * dynamic != 0: (s_x, z_x) come from the min/max of ALL M rows of x and are written
 * to *act_scale / *act_zp; otherwise they are read from there.
 * w_signed != 0: weight codes are two's complement int8 (symmetric scheme).           */
int orc_linear_a8(const uint16_t* x, long M, int K, long ldx, const uint8_t* wcodes, int N, int w_signed,
                  const float* w_scale, const int32_t* w_zp, int dynamic, float* act_scale, int32_t* act_zp,
                  const uint16_t* bias, uint16_t* y, long ldy, int32_t* acc_out, const int64_t* rows,
                  long nrows, const uint16_t* residual, long ldr) {
    if (!x || !wcodes || !w_scale || !w_zp || !act_scale || !act_zp || !y || M <= 0 || K <= 0 || N <= 0 ||
        ldx < K || ldy < N)
        return ORC_BAD_ARG;
    long R = rows ? nrows : M;
    if (R <= 0) return ORC_BAD_ARG;
    if (dynamic) {
        int rc = orc_act_params(x, M, K, ldx, ORC_F16, act_scale, act_zp);
        if (rc) return rc;
    }
    float sx = *act_scale;
    int32_t zx = *act_zp;
    if (!(sx > 0.0f) || zx < 0 || zx > 255) return ORC_BAD_ARG;
    float inv = 1.0f / sx;
    int overflow = 0;
    /* weights with the zero point removed, as int16 */
    int16_t* wd = (int16_t*)malloc((size_t)N * K * sizeof(int16_t));
    if (!wd) return ORC_BAD_ARG;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            int q = w_signed ? (int)(int8_t)wcodes[(size_t)n * K + k] : (int)wcodes[(size_t)n * K + k];
            wd[(size_t)n * K + k] = (int16_t)(q - w_zp[n]);
        }
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (long r = 0; r < R; ++r) {
        long m = rows ? rows[r] : r;
        int16_t* xd = (int16_t*)malloc((size_t)K * sizeof(int16_t));
        for (int k = 0; k < K; ++k)
            xd[k] = (int16_t)(asym_code((float)half_to_double(x[m * ldx + k]), inv, zx, 255) - zx);
        for (int n = 0; n < N; ++n) {
            const int16_t* wr = wd + (size_t)n * K;
            int64_t acc = 0;
            for (int k = 0; k < K; ++k) acc += (int32_t)xd[k] * (int32_t)wr[k];
            if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
            if (acc_out) acc_out[r * (long)N + n] = (int32_t)acc;
            double v = (double)acc * ((double)sx * (double)w_scale[n]);
            if (bias) v += half_to_double(bias[n]);
            if (residual) v += half_to_double(residual[m * ldr + n]);
            y[r * ldy + n] = double_to_half(v);
        }
        free(xd);
    }
    free(wd);
    return overflow ? ORC_OVERFLOW : ORC_OK;
}

/* BOS-aware K/V projection (Sec. 3.1).  ctx is [B,T,K]; token 0 of each prompt is the BOS row.
 *  - tokens 1..T-1 of all prompts form the activation tensor of the 8-bit path above
 *    (their min/max only when dynamic);
 *  - token 0 takes the floating-point result with the unquantised weights w_f16[N,K]
 *    (bos_out == NULL), or a copy of the pre-computed vector bos_out[N];
 *  - naive_all_rows != 0: comparator that sends all B*T rows through the 8-bit path.
 * y is [B,T,N]. */
int orc_bos_aware_kv_proj(const uint16_t* ctx, int B, int T, int K, const uint8_t* wcodes, int N, int w_signed,
                          const float* w_scale, const int32_t* w_zp, const uint16_t* w_f16,
                          const uint16_t* bos_out, int dynamic, float* act_scale, int32_t* act_zp,
                          const uint16_t* bias, uint16_t* y, int naive_all_rows) {
    if (!ctx || !y || B <= 0 || T <= 0 || K <= 0 || N <= 0) return ORC_BAD_ARG;
    if (naive_all_rows)
        return orc_linear_a8(ctx, (long)B * T, K, K, wcodes, N, w_signed, w_scale, w_zp, dynamic, act_scale,
                             act_zp, bias, y, N, NULL, NULL, 0, NULL, 0);
    if ((w_f16 == NULL) == (bos_out == NULL)) return ORC_BAD_ARG; /* exactly one of the two */
    int rc = ORC_OK;
    if (T > 1) {
        long R = (long)B * (T - 1);
        uint16_t* body = (uint16_t*)malloc((size_t)R * K * 2);
        uint16_t* ybody = (uint16_t*)malloc((size_t)R * N * 2);
        if (!body || !ybody) return ORC_BAD_ARG;
        for (int b = 0; b < B; ++b)
            memcpy(body + (size_t)b * (T - 1) * K, ctx + ((size_t)b * T + 1) * K, (size_t)(T - 1) * K * 2);
        rc = orc_linear_a8(body, R, K, K, wcodes, N, w_signed, w_scale, w_zp, dynamic, act_scale, act_zp, bias,
                           ybody, N, NULL, NULL, 0, NULL, 0);
        for (int b = 0; b < B; ++b)
            memcpy(y + ((size_t)b * T + 1) * N, ybody + (size_t)b * (T - 1) * N, (size_t)(T - 1) * N * 2);
        free(body);
        free(ybody);
        if (rc) return rc;
    }
    for (int b = 0; b < B; ++b) {
        uint16_t* y0 = y + (size_t)b * T * N;
        if (bos_out) {
            memcpy(y0, bos_out, (size_t)N * 2);
        } else {
            rc = orc_linear_fp(ctx + (size_t)b * T * K, 1, K, K, w_f16, N, bias, ORC_F16, y0, N, NULL, 0);
            if (rc) return rc;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Feed-forward pair with the activation kept in 8 bits between the two      */
/* linears (an extension; the paper's Sec. 4.3 names the separate FP16->INT8 */
/* conversion layers as the overhead of the W8A8 path, this removes the one  */
/* between the GEGLU projection and the output linear of a transformer       */
/* block's feed-forward).  Stated by the mathematics, in fp64:               */
/*                                                                           */
/*   lin[m,n] = ACC[m,n] * (s_x * s_w[n]) + bias[n]            n in [0, 2H)   */
/*   h[m,j]   = lin[m,j] * gelu(lin[m,H+j])                    j in [0, H)    */
/*   gelu(g)  = 0.5 g (1 + erf(g / sqrt 2))                    C library erf  */
/*   u[m,j]   = h / s_o                                                       */
/*   code     = clamp(rne(u) + z_o, 0, 255)                    Sec. 4.1       */
/*                                                                           */
/* (first half of the projection = value, second half = gate).  ACC is the   */
/* exact integer accumulator of the A8 linear above.  A code is an integer   */
/* decided by floating point: an implementation that evaluates h in a lower  */
/* precision reaches the same code except where u lies within its own error  */
/* of a rounding boundary, so the un-rounded u and lin are handed back for a */
/* checker to apply that rule element by element.                            */
/* ------------------------------------------------------------------------- */

static double gelu64(double g) { return 0.5 * g * (1.0 + erf(g / sqrt(2.0))); }

/* GEGLU projection with 8-bit activations in and out.  wcodes [2H,K]; codes_out [R,H] unsigned codes of the
 * gated product under the given static output parameters; h16_out nullable [R,H]: the same product rounded to fp16;
 * u_out nullable [R,H]: h / s_o before the rounding; lin_out nullable [R,2H]: the projection before the gate. */
int orc_linear_a8_geglu(const uint16_t* x, long M, int K, long ldx, const uint8_t* wcodes, int H, int w_signed,
                        const float* w_scale, const int32_t* w_zp, int dynamic, float* act_scale, int32_t* act_zp,
                        const uint16_t* bias, float out_scale, int32_t out_zp, uint8_t* codes_out, uint16_t* h16_out,
                        double* u_out, double* lin_out, const int64_t* rows, long nrows) {
    if (!x || !wcodes || !w_scale || !w_zp || !act_scale || !act_zp || !codes_out || M <= 0 || K <= 0 || H <= 0 ||
        ldx < K || !(out_scale > 0.0f) || out_zp < 0 || out_zp > 255)
        return ORC_BAD_ARG;
    long R = rows ? nrows : M;
    if (R <= 0) return ORC_BAD_ARG;
    if (dynamic) {
        int rc = orc_act_params(x, M, K, ldx, ORC_F16, act_scale, act_zp);
        if (rc) return rc;
    }
    float sx = *act_scale;
    int32_t zx = *act_zp;
    if (!(sx > 0.0f) || zx < 0 || zx > 255) return ORC_BAD_ARG;
    float inv = 1.0f / sx;
    int N = 2 * H;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (long r = 0; r < R; ++r) {
        long m = rows ? rows[r] : r;
        int* xd = (int*)malloc((size_t)K * sizeof(int));
        double* lin = (double*)malloc((size_t)N * sizeof(double));
        for (int k = 0; k < K; ++k) xd[k] = asym_code((float)half_to_double(x[m * ldx + k]), inv, zx, 255) - zx;
        for (int n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k) {
                int q = w_signed ? (int)(int8_t)wcodes[(size_t)n * K + k] : (int)wcodes[(size_t)n * K + k];
                acc += (int64_t)xd[k] * (q - w_zp[n]);
            }
            if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
            lin[n] = (double)acc * ((double)sx * (double)w_scale[n]) + (bias ? half_to_double(bias[n]) : 0.0);
            if (lin_out) lin_out[r * (long)N + n] = lin[n];
        }
        for (int j = 0; j < H; ++j) {
            double h = lin[j] * gelu64(lin[H + j]);
            double u = h / (double)out_scale;
            double t = rint(u) + (double)out_zp; /* round-half-to-even (the default rounding mode) */
            t = t < 0.0 ? 0.0 : (t > 255.0 ? 255.0 : t);
            codes_out[r * (long)H + j] = (uint8_t)(int)t;
            if (h16_out) h16_out[r * (long)H + j] = double_to_half(h);
            if (u_out) u_out[r * (long)H + j] = u;
        }
        free(xd);
        free(lin);
    }
    return overflow ? ORC_OVERFLOW : ORC_OK;
}

/* A8 linear whose activations arrive as unsigned 8-bit codes with their parameters (the consumer of the above). */
int orc_linear_a8_codes(const uint8_t* qx, long M, int K, float act_scale, int32_t act_zp, const uint8_t* wcodes, int N,
                        int w_signed, const float* w_scale, const int32_t* w_zp, const uint16_t* bias, uint16_t* y,
                        long ldy, int32_t* acc_out, const uint16_t* residual, long ldr) {
    if (!qx || !wcodes || !w_scale || !w_zp || !y || M <= 0 || K <= 0 || N <= 0 || ldy < N || !(act_scale > 0.0f) ||
        act_zp < 0 || act_zp > 255)
        return ORC_BAD_ARG;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (long m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k) {
                int q = w_signed ? (int)(int8_t)wcodes[(size_t)n * K + k] : (int)wcodes[(size_t)n * K + k];
                acc += (int64_t)((int)qx[m * (long)K + k] - act_zp) * (q - w_zp[n]);
            }
            if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
            if (acc_out) acc_out[m * (long)N + n] = (int32_t)acc;
            double v = (double)acc * ((double)act_scale * (double)w_scale[n]);
            if (bias) v += half_to_double(bias[n]);
            if (residual) v += half_to_double(residual[m * ldr + n]);
            y[m * ldy + n] = double_to_half(v);
        }
    }
    return overflow ? ORC_OVERFLOW : ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* 3x3 convolution, stride 1, zero padding 1 (the paper quantises "all the   */
/* linear and convolution layers", Sec. 4.1 "Quantization Scheme": weights   */
/* per output channel -- here over the whole 3x3xCin filter --, activations  */
/* per tensor).  Layouts: x [B,H,W,Cin] and y [B,H,W,N] channels-last; the   */
/* weight codes [N, 9*Cin] with k = (r*3 + s)*Cin + c for filter row r,      */
/* filter column s, input channel c.                                         */
/*     y[b,i,j,n] = sum_{r,s,c} x[b,i+r-1,j+s-1,c] * w[n,r,s,c] + bias[n]    */
/* with x = 0 outside the image.  `pix` selects output pixels (flat index    */
/* (b*H + i)*W + j), NULL = all.  residual: [B,H,W,N] or NULL, as for the    */
/* linear layers.                                                            */
/* stride 2 (the UNet's downsampling convolutions; same filter, padding 1):  */
/* the output is [B,Ho,Wo,N] with Ho = (H-1)/2 + 1, Wo = (W-1)/2 + 1, and    */
/*     y[b,i,j,n] = sum_{r,s,c} x[b,2i+r-1,2j+s-1,c] * w[n,r,s,c] + bias[n]; */
/* pix and residual then index output pixels (b*Ho + i)*Wo + j.              */
/* ------------------------------------------------------------------------- */
int orc_conv3x3_w_only(const uint16_t* x, int B, int H, int W, int Cin, const uint8_t* codes, int N,
                       const float* w_scale, const int32_t* w_zp, const uint16_t* bias, int dtype, uint16_t* y,
                       const int64_t* pix, long npix, const uint16_t* residual, int stride) {
    if (!x || !codes || !w_scale || !w_zp || !y || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || N <= 0) return ORC_BAD_ARG;
    if (stride != 1 && stride != 2) return ORC_BAD_ARG;
    const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
    long R = pix ? npix : (long)B * Ho * Wo;
    if (R <= 0) return ORC_BAD_ARG;
    int K = 9 * Cin;
    double* what = (double*)malloc((size_t)N * K * sizeof(double));
    if (!what) return ORC_BAD_ARG;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            what[(size_t)n * K + k] = (double)w_scale[n] * (double)((int)codes[(size_t)n * K + k] - w_zp[n]);
#pragma omp parallel for schedule(static)
    for (long rr = 0; rr < R; ++rr) {
        long m = pix ? pix[rr] : rr;
        int j = (int)(m % Wo), i = (int)((m / Wo) % Ho), b = (int)(m / ((long)Wo * Ho));
        double* col = (double*)calloc((size_t)K, sizeof(double));
        for (int r = 0; r < 3; ++r)
            for (int s = 0; s < 3; ++s) {
                int ii = stride * i + r - 1, jj = stride * j + s - 1;
                if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                const uint16_t* px = x + (((long)b * H + ii) * W + jj) * Cin;
                for (int c = 0; c < Cin; ++c) col[(r * 3 + s) * Cin + c] = in16(px[c], dtype);
            }
        for (int n = 0; n < N; ++n) {
            const double* wr = what + (size_t)n * K;
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += col[k] * wr[k];
            if (bias) acc += in16(bias[n], dtype);
            if (residual) acc += in16(residual[m * (long)N + n], dtype); /* [B,H,W,N], added before the rounding */
            y[rr * (long)N + n] = out16(acc, dtype);
        }
        free(col);
    }
    free(what);
    return ORC_OK;
}

/* The same convolution on 8-bit activations: one (scale, zero point) for the whole input tensor, dynamic (min-max
 * over all of x) or given; a padded position holds the value 0, whose code is the zero point, so it adds nothing:
 *     ACC[m,n] = sum over in-image (r,s), c of (qx - z_x)(qw - z_w[n]);  y = fp16(ACC * s_x * s_w[n] + bias[n]). */
int orc_conv3x3_a8(const uint16_t* x, int B, int H, int W, int Cin, const uint8_t* wcodes, int N, int w_signed,
                   const float* w_scale, const int32_t* w_zp, int dynamic, float* act_scale, int32_t* act_zp,
                   const uint16_t* bias, uint16_t* y, int32_t* acc_out, const int64_t* pix, long npix,
                   const uint16_t* residual, int stride) {
    if (!x || !wcodes || !w_scale || !w_zp || !act_scale || !act_zp || !y || B <= 0 || H <= 0 || W <= 0 || Cin <= 0 ||
        N <= 0 || (stride != 1 && stride != 2))
        return ORC_BAD_ARG;
    const int Ho = (H - 1) / stride + 1, Wo = (W - 1) / stride + 1;
    long M = (long)B * H * W; /* input pixels: the activation parameters are those of the whole input tensor */
    long R = pix ? npix : (long)B * Ho * Wo;
    if (R <= 0) return ORC_BAD_ARG;
    if (dynamic) {
        int rc = orc_act_params(x, M, Cin, Cin, ORC_F16, act_scale, act_zp);
        if (rc) return rc;
    }
    float sx = *act_scale;
    int32_t zx = *act_zp;
    if (!(sx > 0.0f) || zx < 0 || zx > 255) return ORC_BAD_ARG;
    float inv = 1.0f / sx;
    int K = 9 * Cin;
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (long rr = 0; rr < R; ++rr) {
        long m = pix ? pix[rr] : rr;
        int j = (int)(m % Wo), i = (int)((m / Wo) % Ho), b = (int)(m / ((long)Wo * Ho));
        int* col = (int*)calloc((size_t)K, sizeof(int));
        for (int r = 0; r < 3; ++r)
            for (int s = 0; s < 3; ++s) {
                int ii = stride * i + r - 1, jj = stride * j + s - 1;
                if (ii < 0 || ii >= H || jj < 0 || jj >= W) continue;
                const uint16_t* px = x + (((long)b * H + ii) * W + jj) * Cin;
                for (int c = 0; c < Cin; ++c)
                    col[(r * 3 + s) * Cin + c] = asym_code((float)half_to_double(px[c]), inv, zx, 255) - zx;
            }
        for (int n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k) {
                int q = w_signed ? (int)(int8_t)wcodes[(size_t)n * K + k] : (int)wcodes[(size_t)n * K + k];
                acc += (int64_t)col[k] * (q - w_zp[n]);
            }
            if (acc > INT32_MAX || acc < INT32_MIN) overflow |= 1;
            if (acc_out) acc_out[rr * (long)N + n] = (int32_t)acc;
            double v = (double)acc * ((double)sx * (double)w_scale[n]);
            if (bias) v += half_to_double(bias[n]);
            if (residual) v += half_to_double(residual[m * (long)N + n]);
            y[rr * (long)N + n] = double_to_half(v);
        }
        free(col);
    }
    return overflow ? ORC_OVERFLOW : ORC_OK;
}

/* Weight-only gated projection: h[m,j] = lin[m,j] * gelu(lin[m,H+j]) with lin the weight-only linear over the 2H rows
 * of the weight matrix (first half value, second half gate), everything in fp64 with the library erf, one rounding to
 * the 16-bit output.  With codes_out the gated product also leaves as 8-bit codes of the affine quantiser with the
 * given static parameters, taken from the un-rounded product exactly as orc_linear_a8_geglu does:
 * code = clamp(rne(h / s_o) + z_o, 0, 255); u_out (h / s_o before the rounding) and lin_out (the projection before the
 * gate) are what a checker needs to tell a borderline rounding from a wrong code.  h16 may be NULL then. */
int orc_linear_w_only_geglu(const uint16_t* x, long M, int K, long ldx, const uint8_t* codes, int H,
                            const float* w_scale, const int32_t* w_zp, const uint16_t* bias, int dtype, uint16_t* h16,
                            float out_scale, int32_t out_zp, uint8_t* codes_out, double* u_out, double* lin_out,
                            const int64_t* rows, long nrows) {
    if (!x || !codes || !w_scale || !w_zp || (!h16 && !codes_out) || M <= 0 || K <= 0 || H <= 0 || ldx < K)
        return ORC_BAD_ARG;
    if (codes_out && !(out_scale > 0.0f)) return ORC_BAD_ARG;
    long R = rows ? nrows : M;
    if (R <= 0) return ORC_BAD_ARG;
    int N = 2 * H;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < R; ++r) {
        long m = rows ? rows[r] : r;
        double* lin = (double*)malloc((size_t)N * sizeof(double));
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += in16(x[m * ldx + k], dtype) * ((double)w_scale[n] * (double)((int)codes[(size_t)n * K + k] - w_zp[n]));
            if (bias) acc += in16(bias[n], dtype);
            lin[n] = acc;
            if (lin_out) lin_out[r * (long)N + n] = acc;
        }
        for (int j = 0; j < H; ++j) {
            double g = lin[H + j];
            double h = lin[j] * gelu64(g);
            if (h16) h16[r * (long)H + j] = out16(h, dtype);
            if (codes_out) {
                double u = h / (double)out_scale;
                double t = rint(u) + (double)out_zp;
                if (t < 0.0) t = 0.0;
                if (t > 255.0) t = 255.0;
                codes_out[r * (long)H + j] = (uint8_t)t;
                if (u_out) u_out[r * (long)H + j] = u;
            }
        }
        free(lin);
    }
    return ORC_OK;
}
