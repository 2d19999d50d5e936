/*
 * CPU oracle for the fused-MLP path (MatMul + bias + activation chains in fp32, bf16 and int8).
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
