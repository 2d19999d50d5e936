// Int8 scaled dot-product attention for gfx950 (the Int8 rows of Table I, Section VII): both batch matmuls on the
// int8 matrix instruction, the scalar, the mask and the softmax in between, one kernel, scores never leaving the
// compute unit.
//
// Definition (per batch entry, head and query i; q, k, v int8 with zero point 0):
//   S[j]  = sum_c q[i][c] k[j][c]                         int32
//   s[j]  = S[j] * (q_scale*k_scale*scale) + mask[j]      fp32, here in the base-2 logarithm domain
//   e[j]  = 2^(s[j] - max_j s[j])
//   P[j]  = rne(127 e[j])                                 7 bits unsigned: the signed int8 operand of the second product
//   A[c]  = sum_j P[j] v[j][c],  L = sum_j P[j]           int32
//   o[c]  = clamp(rne((float(A[c]) / float(L)) * (v_scale/o_scale)), -128, 127)
// The normalisation uses the integer sum of the QUANTIZED numerators and comes after the integer product, so nothing
// has to be rescaled while the keys stream by; the price is that the row maximum must be known before the first
// numerator is quantized: the kernel makes two passes over the keys, the first computing scores and their maximum
// only (the first product on the int8 matrix pipe is cheap next to the softmax arithmetic of the second pass).
//
// One workgroup = 4 wavefronts = 128 queries of one (batch, head), a lane owns one query; both products are computed
// transposed (S^T = K Q^T, O^T = V^T P^T) so that, in the 32x32 accumulator layout, a lane's 16 scores of a 32-key
// group become, after quantization, exactly its 16 bytes of the second product's operand: V^T goes to LDS with the
// key index permuted to the order in which the accumulator registers hold the keys.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>

#include "ogc_mha.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

#define MHA8_DEV static __device__ __forceinline__

struct MhaI8Args {
    const uint8_t* q;
    const uint8_t* k;
    const uint8_t* v;
    const float* mask;
    uint8_t* o;
    long long sq[3], sk[3], sv[3], so[3];  // element (= byte) strides: batch, head, token
    int batch, heads, seq;
    int q_tiles;    // ceil(seq / 128)
    int xcd_order;  // 1: the query tiles of one (batch, head) are placed on one XCD
    float c1;       // q_scale * k_scale * scale * log2(e)
    float r;        // v_scale / o_scale
};

MHA8_DEV void swap32_i8(uint32_t& a, uint32_t& b) {
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r[0];
    b = r[1];
}
MHA8_DEV float other_half_f(float x) {
    uint32_t a = __builtin_bit_cast(uint32_t, x), b = a;
    swap32_i8(a, b);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? a : b);
}
MHA8_DEV int other_half_i(int x) {
    uint32_t a = (uint32_t)x, b = a;
    swap32_i8(a, b);
    return (int)((threadIdx.x & 32) ? a : b);
}

// D32 = head_dim / 32.  Key blocks of 64 (two 32-key groups).
template <int D32> __global__ __launch_bounds__(256, 2) void ogc_mha_i8_kernel(MhaI8Args a) {
    constexpr int D = D32 * 32, KB = 64, SB = 2;
    constexpr int KSTR = D + 16;    // bytes per key row of K in LDS (padded: consecutive rows start 4 banks apart)
    constexpr int VSTR = KB + 16;   // bytes per channel row of V^T in LDS
    constexpr int CH = D / 16;      // 16-byte chunks per token row
    constexpr int UNITS = KB * CH;  // 16-byte chunks per block of keys (or values)
    constexpr int KU = (UNITS + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint8_t k_lds[KB * KSTR];
    __shared__ __attribute__((aligned(16))) uint8_t vt_lds[D * VSTR];
    __shared__ __attribute__((aligned(16))) float m_lds[KB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, col = lane & 31;
    int bh, qt;
    if (a.xcd_order) {
        const int L = blockIdx.x, x = L & 7, r = L >> 3;
        bh = x + 8 * (r / a.q_tiles);
        qt = r % a.q_tiles;
    } else {
        bh = blockIdx.x / a.q_tiles;
        qt = blockIdx.x % a.q_tiles;
    }
    const int b = bh / a.heads, hd = bh % a.heads, S = a.seq;
    const uint8_t* kbase = a.k + b * a.sk[0] + hd * a.sk[1];
    const uint8_t* vbase = a.v + b * a.sv[0] + hd * a.sv[1];
    const long long kss = a.sk[2], vss = a.sv[2];

    // this lane's query row as the second operand of the first product: bytes 32 i + 16 h .. + 15 of the row
    const int query = (qt * 4 + wave) * 32 + col;
    v4i qreg[D32];
    {
        const int qrow = query < S ? query : S - 1;
        const uint8_t* qp = a.q + b * a.sq[0] + hd * a.sq[1] + qrow * a.sq[2];
#pragma unroll
        for (int i = 0; i < D32; ++i) qreg[i] = *(const v4i*)(qp + i * 32 + h * 16);
    }

    v4i kreg[KU], vreg[KU];
    float mreg = 0.0f;   // the mask value as loaded; scaled when it is written to LDS (scaling here would wait for the load,
                         // and with it for every key / value load issued just before)
    bool mpad = false;   // the key lies beyond the sequence
    auto prefetch = [&](int key0, bool with_v) {
#pragma unroll
        for (int i = 0; i < KU; ++i) {
            const int u = tid + 256 * i, key = key0 + u / CH, part = u % CH;
            const bool on = (UNITS % 256 == 0 || u < UNITS) && key < S;
            kreg[i] = on ? *(const v4i*)(kbase + key * kss + part * 16) : (v4i){0, 0, 0, 0};
            if (with_v) vreg[i] = on ? *(const v4i*)(vbase + key * vss + part * 16) : (v4i){0, 0, 0, 0};
        }
        if (tid < KB) {
            const int key = key0 + tid;
            mpad = key >= S;
            mreg = 0.0f;
            if (!mpad && a.mask) mreg = a.mask[(long long)b * S + key];
        }
    };
    auto fill_lds = [&](bool with_v) {
#pragma unroll
        for (int i = 0; i < KU; ++i) {
            const int u = tid + 256 * i;
            if (UNITS % 256 == 0 || u < UNITS) {
                const int kk = u / CH, part = u % CH;
                *(v4i*)(k_lds + kk * KSTR + part * 16) = kreg[i];
                if (with_v) {
                    // key kk of the block sits, inside its group of 32, at offset 8g + 4hh + e; the accumulator
                    // registers of a lane in half hh hold it as byte 4g + e: position 16hh + 4g + e
                    const int ko = kk & 31, pos = (kk & 32) + 16 * ((ko >> 2) & 1) + 4 * (ko >> 3) + (ko & 3);
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        vt_lds[(16 * part + j) * VSTR + pos] = (uint8_t)((uint32_t)vreg[i][j >> 2] >> (8 * (j & 3)));
                }
            }
        }
        if (tid < KB) m_lds[tid] = mpad ? -INFINITY : mreg * 1.44269504088896340736f;
    };
    // scores of the current block in the base-2 domain, scalar and mask applied: t[sb][4g+e] <-> key 32 sb + 8g + 4h + e
    auto scores = [&](float (&t)[SB][16]) {
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            const uint8_t* krow = k_lds + (sb * 32 + col) * KSTR + h * 16;
            v16i acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0;
#pragma unroll
            for (int i = 0; i < D32; ++i) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(*(const v4i*)(krow + i * 32), qreg[i], acc, 0, 0, 0);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const v4f mk = *(const v4f*)(m_lds + sb * 32 + 8 * g + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) t[sb][4 * g + e] = __builtin_fmaf((float)acc[4 * g + e], a.c1, mk[e]);
            }
        }
    };

    const int nkb = (S + KB - 1) / KB;
    // ---- pass 1: the row maximum
    float row_max = -INFINITY;
    prefetch(0, false);
    for (int kb = 0; kb < nkb; ++kb) {
        __syncthreads();
        fill_lds(false);
        __syncthreads();
        if (kb + 1 < nkb) prefetch((kb + 1) * KB, false);
        float t[SB][16];
        scores(t);
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int r = 0; r < 16; ++r) row_max = fmaxf(row_max, t[sb][r]);
    }
    row_max = fmaxf(row_max, other_half_f(row_max));  // key 0 always exists: finite

    // ---- pass 2: numerators, quantized, and the second product
    v16i oacc[D32];
#pragma unroll
    for (int d = 0; d < D32; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[d][r] = 0;
    uint32_t row_sum = 0;  // this lane's keys only; the halves are added at the end
    prefetch(0, true);
    for (int kb = 0; kb < nkb; ++kb) {
        __syncthreads();
        fill_lds(true);
        __syncthreads();
        if (kb + 1 < nkb) prefetch((kb + 1) * KB, true);
        float t[SB][16];
        scores(t);
#pragma unroll
        for (int sb = 0; sb < SB; ++sb) {
            uint32_t dw[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t w = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float ex = __builtin_amdgcn_exp2f(t[sb][4 * g + e] - row_max);   // in [0, 1]; a key past the end: 0
                    w = __builtin_amdgcn_cvt_pk_u8_f32(ex * 127.0f, e, w);                 // round to nearest even
                }
                dw[g] = w;
                row_sum = __builtin_amdgcn_sad_u8(w, 0u, row_sum);                         // + the four bytes
            }
            const v4i pw = {(int)dw[0], (int)dw[1], (int)dw[2], (int)dw[3]};
#pragma unroll
            for (int d = 0; d < D32; ++d) {
                const v4i vv = *(const v4i*)(vt_lds + (d * 32 + col) * VSTR + sb * 32 + 16 * h);
                oacc[d] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vv, pw, oacc[d], 0, 0, 0);
            }
        }
    }

    // ---- normalise, requantize, store: after the half exchange a lane holds 16 consecutive channels of its query
    const int total = (int)row_sum + other_half_i((int)row_sum);
    const float lf = (float)total;
    uint8_t* op = a.o + b * a.so[0] + hd * a.so[1] + (long long)query * a.so[2];
#pragma unroll
    for (int d = 0; d < D32; ++d) {
        uint32_t dw[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float tt = ((float)oacc[d][4 * g + e] / lf) * a.r;
                const int qi = (int)__builtin_rintf(fminf(fmaxf(tt, -128.0f), 127.0f));
                w |= ((uint32_t)qi & 0xffu) << (8 * e);
            }
            dw[g] = w;
        }
        swap32_i8(dw[0], dw[2]);
        swap32_i8(dw[1], dw[3]);
        if (query < S) *(v4i*)(op + d * 32 + 16 * h) = (v4i){(int)dw[0], (int)dw[2], (int)dw[1], (int)dw[3]};
    }
}

namespace {

bool stride_ok_i8(const int64_t s[3]) {
    for (int i = 0; i < 3; ++i)
        if (s[i] < 0 || s[i] % 16 != 0) return false;
    return true;
}

}  // namespace

extern "C" {

ogc_status ogc_mha_i8_validate(const ogc_mha_desc* d, const ogc_mha_quant* qp) {
    if (!d || !qp) return OGC_ERR_INVALID_ARG;
    if (d->dtype != OGC_I8) return OGC_ERR_INVALID_ARG;
    if (d->softmax != OGC_SOFTMAX_STABLE && d->softmax != OGC_SOFTMAX_FAST) return OGC_ERR_INVALID_ARG;
    if (!isfinite(d->scale)) return OGC_ERR_INVALID_ARG;
    const float sc[4] = {qp->q_scale, qp->k_scale, qp->v_scale, qp->o_scale};
    for (int i = 0; i < 4; ++i)
        if (!(sc[i] > 0.0f) || !isfinite(sc[i])) return OGC_ERR_INVALID_ARG;
    if (d->batch <= 0 || d->heads <= 0 || d->seq <= 0 || d->head_dim <= 0) return OGC_ERR_SHAPE;
    if (d->seq > 65536 || (int64_t)d->batch * d->heads > 65535) return OGC_ERR_SHAPE;
    // the numerators are quantized against the row maximum: without the max reduction they have no fixed range
    if (d->softmax == OGC_SOFTMAX_FAST) return OGC_ERR_UNSUPPORTED;
    if (d->head_dim != 32 && d->head_dim != 64 && d->head_dim != 96 && d->head_dim != 128) return OGC_ERR_UNSUPPORTED;
    if (!stride_ok_i8(d->q_stride) || !stride_ok_i8(d->k_stride) || !stride_ok_i8(d->v_stride) || !stride_ok_i8(d->o_stride))
        return OGC_ERR_ALIGNMENT;
    return OGC_OK;
}

ogc_status ogc_mha_run_i8(const ogc_mha_desc* d, const ogc_mha_quant* qp, const void* q, const void* k, const void* v,
                          const float* mask, void* o, void* stream) {
    const ogc_status st = ogc_mha_i8_validate(d, qp);
    if (st != OGC_OK) return st;
    if (!q || !k || !v || !o) return OGC_ERR_INVALID_ARG;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return OGC_ERR_ALIGNMENT;
    if ((uintptr_t)mask & 3) return OGC_ERR_ALIGNMENT;
    MhaI8Args a;
    a.q = (const uint8_t*)q;
    a.k = (const uint8_t*)k;
    a.v = (const uint8_t*)v;
    a.mask = mask;
    a.o = (uint8_t*)o;
    for (int i = 0; i < 3; ++i) {
        a.sq[i] = d->q_stride[i];
        a.sk[i] = d->k_stride[i];
        a.sv[i] = d->v_stride[i];
        a.so[i] = d->o_stride[i];
    }
    a.batch = d->batch;
    a.heads = d->heads;
    a.seq = d->seq;
    a.q_tiles = (d->seq + 127) / 128;
    const int bh = d->batch * d->heads;
    a.xcd_order = (bh % 8 == 0) ? 1 : 0;
    a.c1 = ((qp->q_scale * qp->k_scale) * d->scale) * 1.44269504088896340736f;  // fp32 products, left to right
    a.r = qp->v_scale / qp->o_scale;                                             // one fp32 division
    const dim3 grid((unsigned)(bh * a.q_tiles));
    hipStream_t s = (hipStream_t)stream;
    switch (d->head_dim / 32) {
    case 1: hipLaunchKernelGGL((ogc_mha_i8_kernel<1>), grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL((ogc_mha_i8_kernel<2>), grid, dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL((ogc_mha_i8_kernel<3>), grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((ogc_mha_i8_kernel<4>), grid, dim3(256), 0, s, a); break;
    }
    return hipGetLastError() == hipSuccess ? OGC_OK : OGC_ERR_DEVICE;
}

const char* ogc_mha_i8_kernel_name(const ogc_mha_desc* d) {
    if (!d || d->dtype != OGC_I8) return nullptr;
    switch (d->head_dim) {
    case 32: return "ogc_mha_i8_kernel<1>";
    case 64: return "ogc_mha_i8_kernel<2>";
    case 96: return "ogc_mha_i8_kernel<3>";
    case 128: return "ogc_mha_i8_kernel<4>";
    }
    return nullptr;
}

}  // extern "C"
