/*
 * CPU oracle for the fused-MLP path (MatMul + bias + activation chains in fp32, bf16, int8 and 8-bit float).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the plain definition of what the GPU library must
 * compute, written to be checked against the paper by eye: a triple-loop GEMM, one layer at a
 * time, explicit dequantize / requantize, no blocking, no fusion, no reordering.  It shares no
 * code with the HIP path and must never be called from it; only the tests, the smoke check and
 * the cpu_baseline leg of the benchmark may use it.
 *
 * What the paper fixes (arxiv 2301.01333):
 *   - matmul A[M,K] x B[K,N] -> C[M,N]                                    (Section III)
 *   - an MLP is a chain of such matmuls with activations such as ReLU       (Section VII)
 *   - int8 scheme: u8 asymmetric activations, s8 symmetric per-output-channel weights,
 *     plain row-major inputs and outputs                                    (Section VII)
 *   - the int8 graph is a mathematically equivalent rewrite of
 *     dequantize -> fp32 matmul -> quantize, with everything that depends only on constant
 *     weights / scales / zero points ("compensated weight") computed ahead of time
 *                                                                           (Section V)
 * What the paper leaves open (rounding mode, saturation, op order in the requantize, bias
 * placement, GELU/sigmoid formulas, bf16) follows the readings listed in the design notes of
 * this repository; each is marked "reading:" below.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (no fast-math: every fp32 operation
 * below is individually rounded to nearest-even, and fmaf() is the only fused operation).
 * OpenMP parallelises over batch rows only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_RELU = 1, ORACLE_ACT_GELU_TANH = 2, ORACLE_ACT_SIGMOID = 3 };

/* ---- bf16 <-> fp32 (bf16 = upper 16 bits of an IEEE fp32; conversion rounds to nearest even) ---- */
static float bf16_bits_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint16_t f32_to_bf16_bits_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* quiet NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

uint16_t oracle_f32_to_bf16(float f) { return f32_to_bf16_bits_rne(f); }
float oracle_bf16_to_f32(uint16_t h) { return bf16_bits_to_f32(h); }

/* ---- activations.  ReLU is the one the paper names (Section IV example, Section VII); GELU is
 * listed there only as a complex op that decomposes into basic ops, so the tanh form is a
 * reading: 0.5*y*(1+tanh(sqrt(2/pi)*(y+0.044715*y^3))).  Sigmoid = 1/(1+exp(-y)). ---- */
static float act_f32(float y, int act) {
    switch (act) {
    case ORACLE_ACT_RELU: return (y > 0.0f) ? y : 0.0f;
    case ORACLE_ACT_GELU_TANH: {
        float y3 = y * y * y;
        float u = 0.7978845608028654f * (y + 0.044715f * y3);
        return 0.5f * y * (1.0f + tanhf(u));
    }
    case ORACLE_ACT_SIGMOID: return 1.0f / (1.0f + expf(-y));
    default: return y;
    }
}

static double act_f64(double y, int act) {
    switch (act) {
    case ORACLE_ACT_RELU: return (y > 0.0) ? y : 0.0;
    case ORACLE_ACT_GELU_TANH: {
        double u = 0.7978845608028654 * (y + 0.044715 * y * y * y);
        return 0.5 * y * (1.0 + tanh(u));
    }
    case ORACLE_ACT_SIGMOID: return 1.0 / (1.0 + exp(-y));
    default: return y;
    }
}

double oracle_act_f64(double y, int act) { return act_f64(y, act); }
float oracle_act_f32(float y, int act) { return act_f32(y, act); }

/*
 * One fp32 layer:  Y[m,n] = act( sum_k X[m,k]*W[k,n] + bias[n] ) (+ R[m,n] if R != NULL).
 * W is plain row-major [K,N] (Section III orientation).  bias may be NULL.
 * accum_double == 0: products and the running sum are fp32, k ascending (the "fp32 accumulate"
 *                    definition); bias add, activation and residual add in fp32.
 * accum_double != 0: the same formula evaluated in fp64 and rounded to fp32 once at the end
 *                    (the reference any summation order is measured against).
 * Returns 0, or -1 on a bad argument.
 */
int oracle_layer_f32(int M, int K, int N, const float* X, int ldx, const float* W, const float* bias, int act,
                     const float* R, int ldr, float* Y, int ldy, int accum_double) {
    if (M < 0 || K < 0 || N < 0 || !Y || (M && K && N && (!X || !W))) return -1;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            if (accum_double) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) acc += (double)X[(size_t)m * ldx + k] * (double)W[(size_t)k * N + n];
                double y = acc + (bias ? (double)bias[n] : 0.0);
                y = act_f64(y, act);
                if (R) y += (double)R[(size_t)m * ldr + n];
                Y[(size_t)m * ldy + n] = (float)y;
            } else {
                float acc = 0.0f;
                for (int k = 0; k < K; ++k) {
                    float prod = X[(size_t)m * ldx + k] * W[(size_t)k * N + n];
                    acc = acc + prod;
                }
                float y = bias ? acc + bias[n] : acc;
                y = act_f32(y, act);
                if (R) y = y + R[(size_t)m * ldr + n];
                Y[(size_t)m * ldy + n] = y;
            }
        }
    }
    return 0;
}

/*
 * One bf16 layer.  X, W, R and Y hold bf16 bit patterns; bias is fp32 (reading: fp32 bias for
 * every dtype).  Products of two bf16 values are exact in fp32.  The accumulator, bias add,
 * activation and residual add are fp32 (or fp64 if accum_double), and the result is rounded to
 * bf16 once, to nearest even; that rounded value is what the next layer consumes.
 * reading (residual): Y = bf16( act(acc+bias) + (float)R ), the add in fp32, one final rounding.
 */
int oracle_layer_bf16(int M, int K, int N, const uint16_t* X, int ldx, const uint16_t* W, const float* bias, int act,
                      const uint16_t* R, int ldr, uint16_t* Y, int ldy, int accum_double) {
    if (M < 0 || K < 0 || N < 0 || !Y || (M && K && N && (!X || !W))) return -1;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            if (accum_double) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k)
                    acc += (double)bf16_bits_to_f32(X[(size_t)m * ldx + k]) * (double)bf16_bits_to_f32(W[(size_t)k * N + n]);
                double y = acc + (bias ? (double)bias[n] : 0.0);
                y = act_f64(y, act);
                if (R) y += (double)bf16_bits_to_f32(R[(size_t)m * ldr + n]);
                Y[(size_t)m * ldy + n] = f32_to_bf16_bits_rne((float)y);
            } else {
                float acc = 0.0f;
                for (int k = 0; k < K; ++k) {
                    float prod = bf16_bits_to_f32(X[(size_t)m * ldx + k]) * bf16_bits_to_f32(W[(size_t)k * N + n]);
                    acc = acc + prod;
                }
                float y = bias ? acc + bias[n] : acc;
                y = act_f32(y, act);
                if (R) y = y + bf16_bits_to_f32(R[(size_t)m * ldr + n]);
                Y[(size_t)m * ldy + n] = f32_to_bf16_bits_rne(y);
            }
        }
    }
    return 0;
}

/*
 * One int8 layer (Section V: low-precision conversion + constant-weight preprocessing).
 * Real-value model (reading: the standard affine form, the only one under which subtracting
 * a_z * sum_k w_q is the equivalent rewrite):  x = a_s*(x_q - a_z),  w[k,n] = b_s[n]*w_q[k,n].
 *
 *   acc  (i32) = sum_k x_q[m,k] * w_q[k,n]                 exact, any order
 *   acc2 (i32) = acc - a_z * sum_k w_q[k,n]                exact ("compensation")
 *   f    (f32) = (float)acc2                               int -> float, nearest even
 *   s    (f32) = a_s * b_s[n]                              one fp32 multiply
 *   y    (f32) = fmaf(f, s, bias[n])   (no bias: y = f*s)  single rounding
 *   y          = act(y)                                    ReLU in fp32 before the requantize
 *   out_f32 != 0:  Y[m,n] = y as fp32, stop                (last layer of a chain)
 *   inv  (f32) = 1.0f / c_s                                one fp32 divide
 *   t    (f32) = y * inv
 *   r    (f32) = nearbyintf(t)                             ties to even
 *   r          = r + (float)c_z ; clamp to [0,255] ; q = (uint8_t)r
 *
 * readings: RNE + saturate; multiply by the reciprocal rather than divide; fused multiply-add
 * for dequant+bias; fp32 bias added after the dequantize scale.
 * Limits: K <= 65536 so that acc cannot overflow int32 (255*128*65536 < 2^31).
 */
int oracle_layer_i8(int M, int K, int N, const uint8_t* Xq, int ldx, const int8_t* Wq, const float* w_scale,
                    const float* bias, float a_s, int a_z, int act, int out_f32, float c_s, int c_z, void* Yv, int ldy) {
    if (M < 0 || K < 0 || N < 0 || K > 65536 || !Yv || !w_scale || (M && K && N && (!Xq || !Wq))) return -1;
    int32_t* wsum = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    if (!wsum) return -2;
    for (int n = 0; n < N; ++n) {
        int32_t s = 0;
        for (int k = 0; k < K; ++k) s += (int32_t)Wq[(size_t)k * N + n];
        wsum[n] = s;
    }
    const float inv = out_f32 ? 0.0f : 1.0f / c_s;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int k = 0; k < K; ++k) acc += (int32_t)Xq[(size_t)m * ldx + k] * (int32_t)Wq[(size_t)k * N + n];
            int32_t acc2 = acc - (int32_t)a_z * wsum[n];
            float f = (float)acc2;
            float s = a_s * w_scale[n];
            float y = bias ? fmaf(f, s, bias[n]) : f * s;
            y = act_f32(y, act);
            if (out_f32) {
                ((float*)Yv)[(size_t)m * ldy + n] = y;
            } else {
                float t = y * inv;
                float r = nearbyintf(t);
                r = r + (float)c_z;
                r = fminf(fmaxf(r, 0.0f), 255.0f);
                ((uint8_t*)Yv)[(size_t)m * ldy + n] = (uint8_t)r;
            }
        }
    }
    free(wsum);
    return 0;
}

/*
 * The un-rewritten int8 graph of Section V (Fig. 5.1 as described in the text): dequantize both
 * operands to real values, multiply in floating point (fp64 here, so the matmul itself adds no
 * error), add bias, activate, quantize with a true division.  Kept only so a test can check
 * that the rewritten form above is "mathematically equivalent" up to rounding at ties.
 */
int oracle_layer_i8_unfused(int M, int K, int N, const uint8_t* Xq, int ldx, const int8_t* Wq, const float* w_scale,
                            const float* bias, float a_s, int a_z, int act, float c_s, int c_z, uint8_t* Y, int ldy) {
    if (M < 0 || K < 0 || N < 0 || !Y || !w_scale || (M && K && N && (!Xq || !Wq))) return -1;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                double x = (double)a_s * ((double)Xq[(size_t)m * ldx + k] - (double)a_z);
                double w = (double)w_scale[n] * (double)Wq[(size_t)k * N + n];
                acc += x * w;
            }
            double y = acc + (bias ? (double)bias[n] : 0.0);
            y = act_f64(y, act);
            double r = nearbyint(y / (double)c_s) + (double)c_z;
            if (r < 0.0) r = 0.0;
            if (r > 255.0) r = 255.0;
            Y[(size_t)m * ldy + n] = (uint8_t)r;
        }
    }
    return 0;
}

/* ---- 8-bit floating point, the OCP "E4M3" encoding: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits;
 * exponent field 0 holds the subnormals m/8 * 2^-6; there are no infinities; S.1111.111 is the only NaN, so the
 * largest finite magnitude is S.1111.110 = 1.75 * 2^8 = 448.  (The paper has no 8-bit float path; this is the
 * fp8 variant of its int8 scheme, with the encoding fixed by the matrix instructions of the target.) ---- */
static double e4m3_to_f64(uint8_t b) {
    int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);             /* m/8 * 2^-6 */
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* fp32 -> E4M3, round to nearest with ties to the even mantissa, saturating: every finite value (and +-inf) whose
 * rounded magnitude would exceed 448 gives +-448; NaN gives the NaN code with the sign kept.  -0 keeps its sign. */
static uint8_t f32_to_e4m3_rne_sat(float f) {
    uint8_t sign = signbit(f) ? 0x80 : 0x00;
    if (isnan(f)) return (uint8_t)(sign | 0x7f);
    double a = fabs((double)f);
    if (a >= 464.0) return (uint8_t)(sign | 0x7e);    /* 464 is the midpoint of 448 and the absent 480; the tie goes to 448 */
    int ex;
    (void)frexp(a, &ex);                              /* a = frac * 2^ex, frac in [0.5, 1) : floor(log2 a) = ex - 1 */
    int e = (a == 0.0) ? -6 : ex - 1;
    if (e < -6) e = -6;                               /* subnormal range: fixed step 2^-9 */
    double step = ldexp(1.0, e - 3);                  /* spacing of representable values in [2^e, 2^(e+1)) */
    double q = nearbyint(a / step);                   /* exact division by a power of two; ties to even */
    double v = q * step;                              /* may be 2^(e+1): the next binade's first value */
    /* encode v, which is representable */
    if (v == 0.0) return sign;
    if (v < ldexp(1.0, -6)) return (uint8_t)(sign | (uint8_t)(v / ldexp(1.0, -9)));
    (void)frexp(v, &ex);
    int ee = ex - 1;
    int mant = (int)((v / ldexp(1.0, ee) - 1.0) * 8.0);
    return (uint8_t)(sign | ((ee + 7) << 3) | mant);
}

float oracle_e4m3_to_f32(uint8_t b) { return (float)e4m3_to_f64(b); }
uint8_t oracle_f32_to_e4m3(float f) { return f32_to_e4m3_rne_sat(f); }

/*
 * One fp8 layer: the int8 scheme of Section V carried over to E4M3 operands.  There is no zero point (the format
 * is signed and symmetric), so the constant-weight preprocessing reduces to the scale product:
 *   real x = a_s * x8,  real w[k,n] = b_s[n] * w8[k,n]
 *   acc        = sum_k x8[m,k] * w8[k,n]      each product is exact (two 4-bit significands);
 *                accum_double != 0: summed in fp64 (exact for any K the tests use) and rounded to fp32 once;
 *                accum_double == 0: fp32 running sum, k ascending
 *   s    (f32) = a_s * b_s[n]
 *   y    (f32) = fmaf(acc, s, bias[n])   (no bias: y = acc*s)
 *   y          = act(y)
 *   out_f32 != 0:  Y[m,n] = y as fp32, stop
 *   inv  (f32) = 1.0f / c_s ;  t = y * inv ;  Y[m,n] = E4M3(t), nearest-even, saturating at +-448
 * readings: as for int8 (reciprocal multiply, fused dequantize+bias, fp32 bias, fp32 activation), plus saturation
 * instead of NaN on overflow.  A NaN operand code propagates as the arithmetic propagates it.
 */
int oracle_layer_f8(int M, int K, int N, const uint8_t* X8, int ldx, const uint8_t* W8, const float* w_scale,
                    const float* bias, float a_s, int act, int out_f32, float c_s, void* Yv, int ldy, int accum_double) {
    if (M < 0 || K < 0 || N < 0 || !Yv || !w_scale || (M && K && N && (!X8 || !W8))) return -1;
    const float inv = out_f32 ? 0.0f : 1.0f / c_s;
    double val[256]; /* the value of every code, decoded once (every E4M3 value is exact in fp32 and fp64) */
    for (int c = 0; c < 256; ++c) val[c] = e4m3_to_f64((uint8_t)c);
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            float f;
            if (accum_double) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) acc += val[X8[(size_t)m * ldx + k]] * val[W8[(size_t)k * N + n]];
                f = (float)acc;
            } else {
                float acc = 0.0f;
                for (int k = 0; k < K; ++k) {
                    float prod = (float)val[X8[(size_t)m * ldx + k]] * (float)val[W8[(size_t)k * N + n]];
                    acc = acc + prod;
                }
                f = acc;
            }
            float s = a_s * w_scale[n];
            float y = bias ? fmaf(f, s, bias[n]) : f * s;
            y = act_f32(y, act);
            if (out_f32) {
                ((float*)Yv)[(size_t)m * ldy + n] = y;
            } else {
                float t = y * inv;
                ((uint8_t*)Yv)[(size_t)m * ldy + n] = f32_to_e4m3_rne_sat(t);
            }
        }
    }
    return 0;
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
