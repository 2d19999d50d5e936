// Fused scaled dot-product attention for gfx950 (the MHA subgraph of Section VII / Table I): both batch
// matmuls, the scalar, the mask and the softmax in one kernel, scores never leaving the compute unit.
//
// One workgroup = 4 wavefronts = 128 queries of one (batch, head); a wavefront owns 32 queries (64, as two
// groups of 32, in the bf16 variant for head dimensions up to 64).  Keys and
// values stream through LDS in blocks of KB keys (bf16: 64, fp32: 32), prefetched one block ahead in
// registers.  Both products are computed TRANSPOSED so that a lane owns one query:
//
//   S^T[key][query] = K * Q^T     first MFMA operand = 32 keys x k from LDS, second = Q^T, held in registers
//   O^T[c][query]   = V^T * P^T   first operand = 32 channels x keys from LDS (V is transposed on its way into
//                                 LDS), second = the softmax weights exactly where the first product left them
//
// In the 32x32 accumulator layout lane l holds column (query) l%32 and rows 8g + 4(l/32) + e, g,e = 0..3.  The
// softmax reductions of a query are therefore 16 values inside a lane plus one exchange with lane l^32, the
// running maximum / sum / rescale factors are per-lane scalars, and the weights feed the second product without
// any data movement: the reduction axis of that product (keys) may be summed in any order, so V^T is simply
// written to LDS with its key index permuted to the order in which the accumulator registers hold the keys.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ogc_mha.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

#define MHA_DEV static __device__ __forceinline__

struct MhaArgs {
    const uint8_t* q;
    const uint8_t* k;
    const uint8_t* v;
    const float* mask;
    uint8_t* o;
    long long sq[3], sk[3], sv[3], so[3];  // element strides: batch, head, token
    int batch, heads, seq;
    int q_tiles;       // ceil(seq / queries per workgroup)
    int xcd_order;     // 1: workgroups of one (batch, head) are placed on one XCD
    float scale_log2;  // scale * log2(e)
};

constexpr float LOG2E = 1.44269504088896340736f;

MHA_DEV void swap32(uint32_t& a, uint32_t& b) {
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r[0];
    b = r[1];
}
// value of x in the other half of the wavefront (lane ^ 32)
MHA_DEV float other_half(float x) {
    uint32_t a = __builtin_bit_cast(uint32_t, x), b = a;
    swap32(a, b);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? a : b);
}
MHA_DEV uint32_t pack_bf16(float lo, float hi) {  // round to nearest even, two values per register
    v2bf r = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, r);
}

template <int DT> struct MhaCfg;
template <> struct MhaCfg<OGC_BF16> {
    static constexpr int E = 2, KB = 64;
};
template <> struct MhaCfg<OGC_F32> {
    static constexpr int E = 4, KB = 32;
};

// DT: OGC_F32 / OGC_BF16.  D32 = head_dim / 32.  FAST: softmax without the running maximum.  PLAIN: no mask, the
// sequence is a whole number of key blocks and the scalar is positive, so no key needs an addend.
// QS: 32-query groups per wavefront (1 or 2).  With 2, every key / value operand read from LDS feeds two matrix
// instructions (one per group): the bf16 kernel is bound by LDS reads, one KiB per instruction, otherwise.
template <int DT, int D32, int FAST, int PLAIN, int QS> __global__ __launch_bounds__(256, 2) void ogc_mha_kernel(MhaArgs a) {
    constexpr int E = MhaCfg<DT>::E, KB = MhaCfg<DT>::KB, D = D32 * 32;
    constexpr int SB = KB / 32;                 // 32-key sub-blocks per block
    constexpr int KSTR = D * E + 16;            // bytes per key row of K in LDS (padded)
    constexpr int VSTR = KB * E + 16;           // bytes per channel row of V^T in LDS (padded)
    constexpr int CH = D * E / 16;              // 16-byte chunks per token row
    constexpr int KU = KB * CH / 256;                          // 16-byte chunks of K per thread
    constexpr int KP = KB / 2;                                 // bf16: key pairs per block
    constexpr int VU = DT == OGC_BF16 ? (KP * CH + 255) / 256 : D32;  // V units per thread (bf16: a unit is two keys)
    __shared__ __attribute__((aligned(16))) uint8_t k_lds[KB * KSTR];
    __shared__ __attribute__((aligned(16))) uint8_t vt_lds[D * VSTR];
    __shared__ __attribute__((aligned(16))) float m_lds[KB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, col = lane & 31;
    int bh, qt;
    if (a.xcd_order) {  // consecutive workgroup ids go round the 8 XCDs: keep one (batch, head) on one of them
        const int L = blockIdx.x, x = L & 7, r = L >> 3;
        bh = x + 8 * (r / a.q_tiles);
        qt = r % a.q_tiles;
    } else {
        bh = blockIdx.x / a.q_tiles;
        qt = blockIdx.x % a.q_tiles;
    }
    const int b = bh / a.heads, hd = bh % a.heads, S = a.seq;
    const uint8_t* kbase = a.k + (b * a.sk[0] + hd * a.sk[1]) * E;
    const uint8_t* vbase = a.v + (b * a.sv[0] + hd * a.sv[1]) * E;
    const long long kss = a.sk[2] * E, vss = a.sv[2] * E;

    // ---- this lane's query row as the second MFMA operand, resident for the whole kernel
    constexpr int QN = DT == OGC_BF16 ? D / 16 : D / 8;
    int query[QS];
    v4i qreg[QS][QN];
    v16f oacc[QS][D32];
    float run_max[QS], run_sum[QS];  // run_sum: this lane's keys only, halves are added at the end
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
        query[qs] = (qt * 4 + wave) * (32 * QS) + qs * 32 + col;
        const int qrow = query[qs] < S ? query[qs] : S - 1;
        const uint8_t* qp = a.q + (b * a.sq[0] + hd * a.sq[1] + qrow * a.sq[2]) * E;
#pragma unroll
        for (int i = 0; i < QN; ++i) qreg[qs][i] = *(const v4i*)(qp + i * 32 + h * 16);
#pragma unroll
        for (int d = 0; d < D32; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qs][d][r] = 0.0f;
        run_max[qs] = -INFINITY;
        run_sum[qs] = 0.0f;
    }

    // ---- prefetch registers for one block of keys / values / mask
    v4i kreg[KU], vreg[VU][DT == OGC_BF16 ? 2 : 1];
    float mreg = 0.0f;   // the mask value as loaded; scaled when it is written to LDS (scaling here would wait for the load,
                         // and with it for every key / value load issued just before)
    bool mpad = false;   // the key lies beyond the sequence
    auto prefetch = [&](int key0) {
        const bool full = key0 + KB <= S;  // uniform: every key of the block exists, no row needs a zero fill
#pragma unroll
        for (int i = 0; i < KU; ++i) {
            const int u = tid + 256 * i, key = key0 + u / CH, part = u % CH;
            kreg[i] = (full || key < S) ? *(const v4i*)(kbase + key * kss + part * 16) : (v4i){0, 0, 0, 0};
        }
        if constexpr (DT == OGC_BF16) {
#pragma unroll
            for (int i = 0; i < VU; ++i) {
                const int u = tid + 256 * i, kp = u % KP, c = u / KP, key = key0 + 2 * kp;
                const bool on = (KP * CH) % 256 == 0 || 256 * (i + 1) <= KP * CH || c < CH;
                vreg[i][0] = (on && (full || key < S)) ? *(const v4i*)(vbase + key * vss + c * 16) : (v4i){0, 0, 0, 0};
                vreg[i][1] = (on && (full || key + 1 < S)) ? *(const v4i*)(vbase + (key + 1) * vss + c * 16) : (v4i){0, 0, 0, 0};
            }
        } else {
#pragma unroll
            for (int i = 0; i < VU; ++i) {
                const int u = tid + 256 * i, key = key0 + (u & 31), c = u >> 5;
                vreg[i][0] = (full || key < S) ? *(const v4i*)(vbase + key * vss + c * 16) : (v4i){0, 0, 0, 0};
            }
        }
        if (tid < KB) {
            const int key = key0 + tid;
            mpad = key >= S;
            mreg = 0.0f;
            if (!mpad && a.mask) mreg = a.mask[(long long)b * S + key];
        }
    };
    auto fill_lds = [&]() {
#pragma unroll
        for (int i = 0; i < KU; ++i) {
            const int u = tid + 256 * i;
            *(v4i*)(k_lds + (u / CH) * KSTR + (u % CH) * 16) = kreg[i];
        }
        if constexpr (DT == OGC_BF16) {
            // two keys x eight channels per unit -> eight dwords (key, key+1) at the permuted key position:
            // within a group of 16 keys, key offset 8*gg + 4*hh + e sits at 8*hh + 4*gg + e
#pragma unroll
            for (int i = 0; i < VU; ++i) {
                const int u = tid + 256 * i, kp = u % KP, c = u / KP, o = (2 * kp) & 15;
                const int pos = ((2 * kp) & ~15) + ((o & 3) | ((o & 8) >> 1) | ((o & 4) << 1));
                if (c < CH) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t lo = (uint32_t)vreg[i][0][j >> 1], hi = (uint32_t)vreg[i][1][j >> 1];
                        const uint32_t w = __builtin_amdgcn_perm(hi, lo, (j & 1) ? 0x07060302u : 0x05040100u);
                        *(uint32_t*)(vt_lds + (8 * c + j) * VSTR + pos * 2) = w;
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < VU; ++i) {
                const int u = tid + 256 * i, kl = u & 31, c = u >> 5;
#pragma unroll
                for (int j = 0; j < 4; ++j) *(int*)(vt_lds + (4 * c + j) * VSTR + kl * 4) = vreg[i][0][j];
            }
        }
        if (tid < KB) m_lds[tid] = mpad ? -INFINITY : mreg * LOG2E;
    };

    const int nkb = (S + KB - 1) / KB;
    prefetch(0);
    for (int kb = 0; kb < nkb; ++kb) {
        __syncthreads();  // every wavefront is done with the previous block
        fill_lds();
        __syncthreads();
        if (kb + 1 < nkb) prefetch((kb + 1) * KB);

        // ---- scores, transposed: rows = keys, columns = queries
        v16f sacc[QS][SB];
        {
            // bf16: the operand reads of a 32-key group go out before its first matrix instruction (the compiler
            // would otherwise issue each read just ahead of its use and wait for it)
            const v16f zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const uint8_t* krow = k_lds + (sb * 32 + col) * KSTR + h * 16;
                v4i kfrag[QN];
                if constexpr (DT == OGC_BF16) {
#pragma unroll
                    for (int i = 0; i < QN; ++i) kfrag[i] = *(const v4i*)(krow + i * 32);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int i = 0; i < QN; ++i)
#pragma unroll
                    for (int qs = 0; qs < QS; ++qs) {
                        const v4i kv = DT == OGC_BF16 ? kfrag[i] : *(const v4i*)(krow + i * 32);
                        if constexpr (DT == OGC_BF16) {
                            sacc[qs][sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(v8bf, kv), __builtin_bit_cast(v8bf, qreg[qs][i]), i ? sacc[qs][sb] : zero, 0, 0, 0);
                        } else {
                            const v4f kf = __builtin_bit_cast(v4f, kv), qf = __builtin_bit_cast(v4f, qreg[qs][i]);
                            sacc[qs][sb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.x, qf.x, i ? sacc[qs][sb] : zero, 0, 0, 0);
                            sacc[qs][sb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.y, qf.y, sacc[qs][sb], 0, 0, 0);
                            sacc[qs][sb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.z, qf.z, sacc[qs][sb], 0, 0, 0);
                            sacc[qs][sb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf.w, qf.w, sacc[qs][sb], 0, 0, 0);
                        }
                    }
            }
        }
        // ---- scalar, mask, running maximum (base-2 logarithm domain; a key beyond the sequence carries
        // -infinity).  A block of valid keys without a mask needs no per-key addend: the maximum is taken on
        // the raw products and the scalar rides in the exponent's multiply-add.
        const float c = a.scale_log2;
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            float cand = -INFINITY;
            if constexpr (PLAIN) {
                if constexpr (!FAST) {
#pragma unroll
                    for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) cand = fmaxf(cand, sacc[qs][sb][r]);
                    cand *= c;
                }
            } else {
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const v4f mk = *(const v4f*)(m_lds + sb * 32 + 8 * g + 4 * h);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float t = __builtin_fmaf(sacc[qs][sb][4 * g + e], c, mk[e]);
                            sacc[qs][sb][4 * g + e] = t;
                            if constexpr (!FAST) cand = fmaxf(cand, t);
                        }
                    }
            }
            float off = 0.0f;
            if constexpr (!FAST) {
                // The reference point of the exponentials only has to be NEAR the maximum: it moves when a block
                // exceeds it by more than 2^8, so most blocks skip the rescaling of the output accumulators.  The
                // result is the same function (numerator and denominator carry the same factor); weights reach
                // 256 at most, far from any overflow.  Key 0 of block 0 is always valid: the first block sets it.
                cand = fmaxf(cand, other_half(cand));
                const bool need = cand > run_max[qs] + 8.0f;
                if (__builtin_amdgcn_ballot_w64(need) != 0) {
                    const float new_max = need ? cand : run_max[qs];
                    const float alpha = __builtin_amdgcn_exp2f(run_max[qs] - new_max);
                    run_max[qs] = new_max;
                    run_sum[qs] *= alpha;
#pragma unroll
                    for (int d = 0; d < D32; ++d)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[qs][d][r] *= alpha;
                }
                off = -run_max[qs];
            }
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float x;
                    if constexpr (PLAIN) x = __builtin_fmaf(sacc[qs][sb][r], c, off);
                    else x = FAST ? sacc[qs][sb][r] : sacc[qs][sb][r] + off;
                    sacc[qs][sb][r] = __builtin_amdgcn_exp2f(x);
                }
        }
        // ---- O^T += V^T P^T
        if constexpr (DT == OGC_BF16) {
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    // the row sum takes the weights as rounded, the values the second product multiplies
                    v4i pw[QS];
#pragma unroll
                    for (int qs = 0; qs < QS; ++qs) {
                        const v16f& p = sacc[qs][sb];
                        uint32_t w[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const v2bf pr = {(__bf16)p[8 * j + 2 * t], (__bf16)p[8 * j + 2 * t + 1]};
                            run_sum[qs] = __builtin_amdgcn_fdot2_f32_bf16(pr, (v2bf){(__bf16)1.0f, (__bf16)1.0f}, run_sum[qs], false);
                            w[t] = __builtin_bit_cast(uint32_t, pr);
                        }
                        pw[qs] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
                    }
#pragma unroll
                    for (int d = 0; d < D32; ++d) {
                        const v4i vv = *(const v4i*)(vt_lds + (d * 32 + col) * VSTR + (sb * 32 + 16 * j + 8 * h) * 2);
#pragma unroll
                        for (int qs = 0; qs < QS; ++qs)
                            oacc[qs][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, vv),
                                                                                  __builtin_bit_cast(v8bf, pw[qs]), oacc[qs][d], 0, 0, 0);
                    }
                }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int qs = 0; qs < QS; ++qs) run_sum[qs] += sacc[qs][0][r];
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int d = 0; d < D32; ++d) {
                    const v4f vv = *(const v4f*)(vt_lds + (d * 32 + col) * VSTR + (8 * g + 4 * h) * 4);
#pragma unroll
                    for (int qs = 0; qs < QS; ++qs) {
                        oacc[qs][d] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv.x, sacc[qs][0][4 * g], oacc[qs][d], 0, 0, 0);
                        oacc[qs][d] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv.y, sacc[qs][0][4 * g + 1], oacc[qs][d], 0, 0, 0);
                        oacc[qs][d] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv.z, sacc[qs][0][4 * g + 2], oacc[qs][d], 0, 0, 0);
                        oacc[qs][d] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv.w, sacc[qs][0][4 * g + 3], oacc[qs][d], 0, 0, 0);
                    }
                }
        }
    }

    // ---- normalise and store: after the half exchange a lane holds 16 consecutive channels of its query
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
        const float total = run_sum[qs] + other_half(run_sum[qs]);
        const float inv = 1.0f / total;
        uint8_t* op = a.o + (b * a.so[0] + hd * a.so[1] + (long long)query[qs] * a.so[2]) * E;
#pragma unroll
        for (int d = 0; d < D32; ++d) {
            if constexpr (DT == OGC_BF16) {
                uint32_t dw[4][2];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    dw[g][0] = pack_bf16(oacc[qs][d][4 * g] * inv, oacc[qs][d][4 * g + 1] * inv);
                    dw[g][1] = pack_bf16(oacc[qs][d][4 * g + 2] * inv, oacc[qs][d][4 * g + 3] * inv);
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    swap32(dw[0][j], dw[2][j]);
                    swap32(dw[1][j], dw[3][j]);
                }
                if (query[qs] < S) {
                    uint8_t* dst = op + (d * 32 + 16 * h) * 2;
                    *(v4i*)dst = (v4i){(int)dw[0][0], (int)dw[0][1], (int)dw[2][0], (int)dw[2][1]};
                    *(v4i*)(dst + 16) = (v4i){(int)dw[1][0], (int)dw[1][1], (int)dw[3][0], (int)dw[3][1]};
                }
            } else {
                uint32_t dw[4][4];
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int e = 0; e < 4; ++e) dw[g][e] = __builtin_bit_cast(uint32_t, oacc[qs][d][4 * g + e] * inv);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    swap32(dw[0][e], dw[2][e]);
                    swap32(dw[1][e], dw[3][e]);
                }
                if (query[qs] < S) {
                    uint8_t* dst = op + (d * 32 + 16 * h) * 4;
                    const int order[4] = {0, 2, 1, 3};
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        *(v4i*)(dst + 16 * g) = (v4i){(int)dw[order[g]][0], (int)dw[order[g]][1], (int)dw[order[g]][2], (int)dw[order[g]][3]};
                }
            }
        }
    }
}

namespace {

template <int DT, int D32, int QS> hipError_t launch_fast(int fast, int plain, const MhaArgs& a, dim3 grid, hipStream_t st) {
    if (fast && plain) hipLaunchKernelGGL((ogc_mha_kernel<DT, D32, 1, 1, QS>), grid, dim3(256), 0, st, a);
    else if (fast) hipLaunchKernelGGL((ogc_mha_kernel<DT, D32, 1, 0, QS>), grid, dim3(256), 0, st, a);
    else if (plain) hipLaunchKernelGGL((ogc_mha_kernel<DT, D32, 0, 1, QS>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((ogc_mha_kernel<DT, D32, 0, 0, QS>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}
template <int DT> hipError_t launch_dim(int d32, int qs, int fast, int plain, const MhaArgs& a, dim3 grid, hipStream_t st) {
    if (qs == 2) {  // bf16 with head_dim <= 64 only (query_groups)
        if constexpr (DT == OGC_BF16) return d32 == 1 ? launch_fast<DT, 1, 2>(fast, plain, a, grid, st) : launch_fast<DT, 2, 2>(fast, plain, a, grid, st);
    }
    switch (d32) {
    case 1: return launch_fast<DT, 1, 1>(fast, plain, a, grid, st);
    case 2: return launch_fast<DT, 2, 1>(fast, plain, a, grid, st);
    case 3: return launch_fast<DT, 3, 1>(fast, plain, a, grid, st);
    default: return launch_fast<DT, 4, 1>(fast, plain, a, grid, st);
    }
}

// 32-query groups per wavefront.  Two where the registers allow it (bf16, head_dim <= 64) and the sequence is long
// enough to keep the four wavefronts of a workgroup busy: the bf16 kernel is then no longer bound by LDS reads.
int query_groups(const ogc_mha_desc* d) {
    const bool can = d->dtype == OGC_BF16 && d->head_dim <= 64;
    if (d->query_groups != 0) return (d->query_groups == 2 && can) ? 2 : 1;
    return (can && d->seq >= 256) ? 2 : 1;
}

// no mask, whole key blocks only, positive scalar
bool plain_case(const ogc_mha_desc* d, const float* mask) {
    const int kb = d->dtype == OGC_BF16 ? MhaCfg<OGC_BF16>::KB : MhaCfg<OGC_F32>::KB;
    return mask == nullptr && d->seq % kb == 0 && d->scale > 0.0f;
}

bool stride_ok(const int64_t s[3], int elt) {
    for (int i = 0; i < 3; ++i)
        if (s[i] < 0 || (s[i] * elt) % 16 != 0) return false;
    return true;
}

}  // namespace

extern "C" {

ogc_status ogc_mha_validate(const ogc_mha_desc* d) {
    if (!d) return OGC_ERR_INVALID_ARG;
    if (d->dtype != OGC_F32 && d->dtype != OGC_BF16 && d->dtype != OGC_I8) return OGC_ERR_INVALID_ARG;
    if (d->softmax != OGC_SOFTMAX_STABLE && d->softmax != OGC_SOFTMAX_FAST) return OGC_ERR_INVALID_ARG;
    if (d->query_groups < 0 || d->query_groups > 2) return OGC_ERR_INVALID_ARG;
    if (!isfinite(d->scale)) return OGC_ERR_INVALID_ARG;
    if (d->batch <= 0 || d->heads <= 0 || d->seq <= 0 || d->head_dim <= 0) return OGC_ERR_SHAPE;
    if (d->seq > 65536 || (int64_t)d->batch * d->heads > 65535) return OGC_ERR_SHAPE;
    if (d->dtype == OGC_I8) return OGC_ERR_UNSUPPORTED;
    if (d->head_dim != 32 && d->head_dim != 64 && d->head_dim != 96 && d->head_dim != 128) return OGC_ERR_UNSUPPORTED;
    const int e = d->dtype == OGC_F32 ? 4 : 2;
    if (!stride_ok(d->q_stride, e) || !stride_ok(d->k_stride, e) || !stride_ok(d->v_stride, e) || !stride_ok(d->o_stride, e))
        return OGC_ERR_ALIGNMENT;
    return OGC_OK;
}

ogc_status ogc_mha_run(const ogc_mha_desc* d, const void* q, const void* k, const void* v, const float* mask, void* o,
                       void* stream) {
    const ogc_status st = ogc_mha_validate(d);
    if (st != OGC_OK) return st;
    if (!q || !k || !v || !o) return OGC_ERR_INVALID_ARG;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return OGC_ERR_ALIGNMENT;
    if ((uintptr_t)mask & 3) return OGC_ERR_ALIGNMENT;
    MhaArgs a;
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
    const int qs = query_groups(d);
    a.q_tiles = (d->seq + 128 * qs - 1) / (128 * qs);
    const int bh = d->batch * d->heads;
    a.xcd_order = (bh % 8 == 0) ? 1 : 0;
    a.scale_log2 = d->scale * 1.44269504088896340736f;
    const dim3 grid((unsigned)(bh * a.q_tiles));
    const int plain = plain_case(d, mask);
    const hipError_t e = d->dtype == OGC_F32 ? launch_dim<OGC_F32>(d->head_dim / 32, qs, d->softmax, plain, a, grid, (hipStream_t)stream)
                                             : launch_dim<OGC_BF16>(d->head_dim / 32, qs, d->softmax, plain, a, grid, (hipStream_t)stream);
    return e == hipSuccess ? OGC_OK : OGC_ERR_DEVICE;
}

const char* ogc_mha_kernel_name(const ogc_mha_desc* d, int32_t has_mask) {
    if (ogc_mha_validate(d) != OGC_OK) return nullptr;
    static char names[2][4][2][2][2][48];
    const int plain = plain_case(d, has_mask ? (const float*)d : nullptr), qs = query_groups(d);
    char* s = names[d->dtype == OGC_BF16][d->head_dim / 32 - 1][d->softmax][plain][qs - 1];
    if (!s[0]) snprintf(s, 48, "ogc_mha_kernel<%d, %d, %d, %d, %d>", d->dtype, d->head_dim / 32, d->softmax, plain, qs);
    return s;
}

}  // extern "C"
