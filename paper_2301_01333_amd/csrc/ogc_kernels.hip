// gfx950 (MI355X, CDNA4) kernels of the fused-MLP library: weight prepack, per-layer GEMM + register
// epilogue, and the fused multi-layer chain kernel.  Wave64, 32x32 MFMA tiles, LDS staging.
//
// Orientation.  Every kernel computes the TRANSPOSED product tile D[n][m] = sum_k W[n][k] X[m][k]: the
// packed weights are the first MFMA operand (rows = output channel n) and the activations the second
// (columns = batch row m).  In the 32x32 MFMA result layout a lane then owns one batch row (m = lane%32)
// and 16 output channels in four runs of four (n = 8*g + 4*(lane/32) + e for register 4*g+e), so the
// per-channel post-ops read their parameters as float4 and the outputs of one row are packed along n,
// which is contiguous both in the plain row-major result and in the next layer's operand layout.
#include <hip/hip_runtime.h>

#include <stdio.h>
#include <string.h>
#include <atomic>
#include <mutex>
#include <type_traits>

#include "ogc_internal.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef long v2l __attribute__((ext_vector_type(2)));

#define OGC_DEV static __device__ __forceinline__

template <int DT> struct AccT { typedef v16f type; };
template <> struct AccT<OGC_I8> { typedef v16i type; };

template <int DT> struct Elt { enum { size = DT == OGC_F32 ? 4 : (DT == OGC_BF16 ? 2 : 1) }; };
// dtypes that follow the quantized scheme of Section V: one-byte operands, a combined per-channel scale, a
// requantized or fp32 result
template <int DT> struct Quant { enum { yes = DT == OGC_I8 || DT == OGC_F8 }; };

// Four fp32 -> four packed E4M3 bytes (v_cvt_pk_fp8_f32: nearest even), saturating at +-448; a NaN stays a NaN.
OGC_DEV float e4m3_clamp(float t) { return t != t ? t : __builtin_amdgcn_fmed3f(t, -448.0f, 448.0f); }
OGC_DEV uint32_t f32x4_to_e4m3x4(float a, float b, float c, float d) {
    int r = __builtin_amdgcn_cvt_pk_fp8_f32(e4m3_clamp(a), e4m3_clamp(b), 0, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(e4m3_clamp(c), e4m3_clamp(d), r, true);
    return (uint32_t)r;
}

// One 32(n) x 32(m) x 32-byte-of-K MFMA step (GEMM main loop; the role of the batch-reduce GEMM
// microkernel of Section III).  w and x are the lane's 16 bytes of the two operands.
template <int DT> OGC_DEV void mma32(typename AccT<DT>::type& c, const v4i& w, const v4i& x) {
    if constexpr (DT == OGC_I8) {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(w, x, c, 0, 0, 0);
    } else if constexpr (DT == OGC_BF16) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, w), __builtin_bit_cast(v8bf, x), c, 0, 0, 0);
    } else if constexpr (DT == OGC_F8) {
        // two 8-byte halves of the lane's 16 bytes: which k a byte stands for is the same in both operands, and that
        // is all a dot product needs
        const v2l wl = __builtin_bit_cast(v2l, w), xl = __builtin_bit_cast(v2l, x);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(wl.x, xl.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(wl.y, xl.y, c, 0, 0, 0);
    } else {
        const v4f wf = __builtin_bit_cast(v4f, w), xf = __builtin_bit_cast(v4f, x);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.x, xf.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.y, xf.y, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.z, xf.z, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf.w, xf.w, c, 0, 0, 0);
    }
}

typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
// Two fp32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32); lo goes to bits 15:0.
OGC_DEV uint32_t f32x2_to_bf16x2(float lo, float hi) {
    const v2bf p = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, p);
}
OGC_DEV float bf16_to_f32(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// Exchange between the two half-waves: afterwards a = {a.lo, b.lo}, b = {a.hi, b.hi} (lo = lanes 0..31).
OGC_DEV void swap32(uint32_t& a, uint32_t& b) {
    auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    a = r[0];
    b = r[1];
}

// ------------------------------------------------------------------------------------------------
// Epilogue (post-op anchor #1 of the fused-op template, Section IV: the post-ops run on the accumulator
// tile while it is still in registers).  Turns one 32x32 accumulator block into 16 fp32 values per lane.
//   float dtypes: y = act(acc + bias[n])
//   I8: y = act(fma((float)(acc + ncomp[n]), scale[n], bias[n])); unless out_f32:
//       out = min(max(rne(y * inv_cs) + zp_out, 0), 255)      (an integer-valued float)
// ------------------------------------------------------------------------------------------------
// Accurate logistic function (correctly rounded division, libm-grade exp); kept out of line: it is the
// rare last-layer activation and its code would otherwise be replicated for every accumulator block.
static __device__ __attribute__((noinline)) float sigmoid_accurate(float y) { return 1.0f / (1.0f + expf(-y)); }

// Applies the activation to the 16 values of a lane.  `act` is uniform over the launch.
// CALLS = false leaves out the sigmoid (an out-of-line call), for kernels that keep state in fixed registers.
template <bool CALLS> OGC_DEV void act_apply16(float (&out)[16], int act) {
    if (act == OGC_ACT_RELU) {
#pragma unroll
        for (int i = 0; i < 16; ++i) out[i] = __builtin_fmaxf(out[i], 0.0f);
    } else if (act == OGC_ACT_GELU_TANH) {
        // 0.5*y*(1+tanh(u)) == y / (1 + exp(-2u)), u = sqrt(2/pi)*(y + 0.044715*y^3);
        // exp(-2u) = exp2(y*(k1 + k2*y^2)) with k1 = -2*sqrt(2/pi)*log2(e), k2 = k1*0.044715
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float y = out[i];
            const float arg = y * __builtin_fmaf(-0.10294324f, y * y, -2.3022082f);
            out[i] = y * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(arg));
        }
    } else if (CALLS && act == OGC_ACT_SIGMOID) {
        for (int i = 0; i < 16; ++i) out[i] = sigmoid_accurate(out[i]);
    }
}

// Per-channel post-op parameters of one 32-channel block as a lane needs them: entry g covers the channels
// n0 + 8g + 4*(lane/32) .. +3 (the lane's registers 4g .. 4g+3).  s: combined scale (I8), b: bias, c: negated
// zero-point compensation (I8).
struct BlockParams {
    v4f s[4];
    v4f b[4];
    v4i c[4];
};

// From the packed blob in global memory (arrays indexed by absolute channel).
template <int DT>
OGC_DEV void load_block_params(BlockParams& p, const OgcLayerArgs& a, int n0, int h) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int n = n0 + 8 * g + 4 * h;
        p.s[g] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        p.b[g] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        p.c[g] = (v4i){0, 0, 0, 0};
        if (a.has_bias) p.b[g] = *(const v4f*)(a.bias + n);
        if constexpr (Quant<DT>::yes) p.s[g] = *(const v4f*)(a.scale + n);
        if constexpr (DT == OGC_I8) {
            if (a.has_comp) p.c[g] = *(const v4i*)(a.ncomp + n);
        }
    }
}

template <int DT, bool CALLS>
OGC_DEV void epilogue_values(const typename AccT<DT>::type& acc, const OgcLayerArgs& a, const BlockParams& p, float (&out)[16]) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        if constexpr (DT == OGC_I8) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float f = (float)(acc[4 * g + e] + p.c[g][e]);
                out[4 * g + e] = __builtin_fmaf(f, p.s[g][e], p.b[g][e]);
            }
        } else if constexpr (DT == OGC_F8) {
#pragma unroll
            for (int e = 0; e < 4; ++e) out[4 * g + e] = __builtin_fmaf(acc[4 * g + e], p.s[g][e], p.b[g][e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) out[4 * g + e] = acc[4 * g + e] + p.b[g][e];
        }
    }
    act_apply16<CALLS>(out, a.act);
    if constexpr (DT == OGC_F8) {
        if (!a.out_f32) {  // the value the E4M3 conversion in pack_block rounds
            const float inv = a.inv_cs;
#pragma unroll
            for (int i = 0; i < 16; ++i) out[i] = out[i] * inv;
        }
    }
    if constexpr (DT == OGC_I8) {
        if (!a.out_f32) {
            const float inv = a.inv_cs, zp = a.zp_out;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float r = __builtin_rintf(out[i] * inv);
                r = r + zp;
                out[i] = __builtin_fminf(__builtin_fmaxf(r, 0.0f), 255.0f);
            }
        }
    }
}

// 16-byte result stores.  Results that go to global memory are written through (system-scope bits on the store):
// a layer's whole output otherwise sits dirty in the L2s until the kernel ends and is written back in one burst
// that the kernel has to wait for; written through, it drains while the kernel computes.  GlobalY marks a
// pointer that is known to be global memory; a plain uint8_t* may also point into LDS (fused chain kernel).
struct GlobalY {
    uint8_t* p;
    __device__ __forceinline__ GlobalY operator+(size_t o) const { return GlobalY{p + o}; }
};
OGC_DEV void store16_through(uint8_t* p, const v4i& v) {
    // the s_nop keeps the next instruction (which may overwrite the data registers) two wait states away from a
    // store of more than 64 bits, as this target requires; the compiler inserts that for its own stores but
    // does not look inside this one
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
OGC_DEV void store16(uint8_t* p, const v4i& v) { *(v4i*)p = v; }
OGC_DEV void store16(GlobalY g, const v4i& v) { store16_through(g.p, v); }

// Converts the 16 values of a lane to the stored type, exchanges quads between the half-waves so that
// each lane holds 16 CONSECUTIVE channels (n0 + 16*(lane/32) ...), and returns them as NDW 16-byte chunks.
//   EO = bytes per stored element (1: u8/s8, 2: bf16, 4: fp32); NDW == EO.
//   bias_s8: store u8 values with 128 subtracted (internal activation form).
//   F8: EO == 1 and the bytes are E4M3 codes of the values (rounded here) instead of integers already rounded.
template <int EO, bool F8 = false>
OGC_DEV void pack_block(const float (&out)[16], bool bias_s8, v4i (&chunk)[EO]) {
    uint32_t dw[4][EO];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        if constexpr (EO == 1 && F8) {
            dw[g][0] = f32x4_to_e4m3x4(out[4 * g], out[4 * g + 1], out[4 * g + 2], out[4 * g + 3]);
        } else if constexpr (EO == 1) {
            uint32_t p = (uint32_t)out[4 * g] | ((uint32_t)out[4 * g + 1] << 8) | ((uint32_t)out[4 * g + 2] << 16) |
                         ((uint32_t)out[4 * g + 3] << 24);
            dw[g][0] = bias_s8 ? (p ^ 0x80808080u) : p;
        } else if constexpr (EO == 2) {
            dw[g][0] = f32x2_to_bf16x2(out[4 * g], out[4 * g + 1]);
            dw[g][1] = f32x2_to_bf16x2(out[4 * g + 2], out[4 * g + 3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) dw[g][e] = __builtin_bit_cast(uint32_t, out[4 * g + e]);
        }
    }
#pragma unroll
    for (int j = 0; j < EO; ++j) {
        swap32(dw[0][j], dw[2][j]);
        swap32(dw[1][j], dw[3][j]);
    }
    // lane order after the exchange: quads [0],[2],[1],[3]
    uint32_t seq[4 * EO];
    const int order[4] = {0, 2, 1, 3};
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < EO; ++j) seq[q * EO + j] = dw[order[q]][j];
#pragma unroll
    for (int c = 0; c < EO; ++c) chunk[c] = (v4i){(int)seq[4 * c], (int)seq[4 * c + 1], (int)seq[4 * c + 2], (int)seq[4 * c + 3]};
}

// Adds the residual x0[m, n0+16h .. +15] (plain row-major, same dtype) to the lane's 16 values.  The
// exchange has not happened yet, so the values are still in register order: out[4g+e] <-> n0+8g+4h+e.
template <int DT>
OGC_DEV void add_residual(float (&out)[16], const OgcLayerArgs& a, int m, int n0, int h) {
    if (m >= a.M) return;
    const uint8_t* row = a.res + (long long)m * a.ldres_bytes;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int n = n0 + 8 * g + 4 * h;
        if (a.res_vec_ok && n + 4 <= a.N) {  // four consecutive channels in one load (n is a multiple of 4)
            if constexpr (DT == OGC_F32) {
                const v4f r = *(const v4f*)(row + (size_t)n * 4);
                out[4 * g] += r.x, out[4 * g + 1] += r.y, out[4 * g + 2] += r.z, out[4 * g + 3] += r.w;
            }
            if constexpr (DT == OGC_BF16) {
                const uint2 r = *(const uint2*)(row + (size_t)n * 2);
                out[4 * g] += __builtin_bit_cast(float, r.x << 16);
                out[4 * g + 1] += __builtin_bit_cast(float, r.x & 0xffff0000u);
                out[4 * g + 2] += __builtin_bit_cast(float, r.y << 16);
                out[4 * g + 3] += __builtin_bit_cast(float, r.y & 0xffff0000u);
            }
            continue;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (n + e < a.N) {
                if constexpr (DT == OGC_F32) out[4 * g + e] = out[4 * g + e] + *(const float*)(row + (size_t)(n + e) * 4);
                if constexpr (DT == OGC_BF16) out[4 * g + e] = out[4 * g + e] + bf16_to_f32(*(const uint16_t*)(row + (size_t)(n + e) * 2));
            }
        }
    }
}

// Final store of a block to the caller's plain row-major y (post-op reorder to the plain layout at the
// graph boundary, Sections IV-V).  The lane holds channels nl .. nl+15 of row m as EO chunks.
template <int EO>
OGC_DEV void store_plain(const v4i (&chunk)[EO], const OgcLayerArgs& a, int m, int nl) {
    if (m >= a.M || nl >= a.N) return;
    uint8_t* p = a.y + (long long)m * a.ldy_bytes + (size_t)nl * EO;
    if (a.y_vec_ok && nl + 16 <= a.N) {
#pragma unroll
        for (int c = 0; c < EO; ++c) store16_through(p + 16 * c, chunk[c]);
    } else {
        const int cnt = (a.N - nl < 16) ? (a.N - nl) : 16;
#pragma unroll
        for (int c = 0; c < EO; ++c) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const uint32_t v = (uint32_t)chunk[c][d];
                if constexpr (EO == 1) {
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (c * 16 + d * 4 + b < cnt) p[c * 16 + d * 4 + b] = (uint8_t)(v >> (8 * b));
                } else if constexpr (EO == 2) {
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        if (c * 8 + d * 2 + b < cnt) ((uint16_t*)p)[c * 8 + d * 2 + b] = (uint16_t)(v >> (16 * b));
                } else {
                    if (c * 4 + d < cnt) ((uint32_t*)p)[c * 4 + d] = v;
                }
            }
        }
    }
}

// Complete epilogue of one 32x32 block.  OUT_PLAIN = 0: write the block into a KB16 activation buffer at
// `yblk` (base of the 32-row block row: global workspace or LDS), directly in the next layer's operand
// layout (layout propagation, Section V).  OUT_PLAIN = 1: write to the caller's y.
// Int8 layer with ReLU and a requantized u8 result: the common case, five VALU operations per element.
// Equivalent, value for value, to the reference sequence relu -> *inv -> rne -> +zp -> clamp[0,255]:
//   t = y*inv; t = med3(t, 0, 255-zp)  (a negative y lands on 0 exactly as relu(y)=0 does; 255-zp is an
//   integer, so clamping before the rounding cannot change which integer is reached);
//   v_cvt_pk_u8_f32 rounds to nearest even and packs the byte; zp is added to four packed bytes at once
//   (no byte can carry: each is <= 255-zp).  q_add / q_xor are precomputed on the host: zp*0x01010101 and,
//   for the internal s8 form, 0x80808080 (both 0 when zp = 128 and the result stays internal).
// The arithmetic of that epilogue alone: the lane's 16 consecutive result bytes (channels n0 + 16*(lane/32) ..) of
// row lane%32, as one 16-byte chunk.
OGC_DEV v4i requant_block_i8_relu(const v16i& acc, const OgcLayerArgs& a, const BlockParams& p) {
    const float inv = a.inv_cs, hi = a.q_hi;
    uint32_t dw[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint32_t q = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float f = (float)(acc[4 * g + e] + p.c[g][e]);
            const float y = __builtin_fmaf(f, p.s[g][e], p.b[g][e]);
            const float t = __builtin_amdgcn_fmed3f(y * inv, 0.0f, hi);
            q = __builtin_amdgcn_cvt_pk_u8_f32(t, e, q);
        }
        dw[g] = (q + a.q_add) ^ a.q_xor;
    }
    swap32(dw[0], dw[2]);
    swap32(dw[1], dw[3]);
    return (v4i){(int)dw[0], (int)dw[2], (int)dw[1], (int)dw[3]};  // 16 consecutive channels from n0+16h
}

template <int OUT_PLAIN, typename YP>
OGC_DEV void epilogue_block_i8_relu(const v16i& acc, const OgcLayerArgs& a, const BlockParams& p, int n0, int m0, int lane,
                                    YP yblk) {
    const int h = lane >> 5, mm = lane & 31;
    const v4i ch = requant_block_i8_relu(acc, a, p);
    if constexpr (OUT_PLAIN) {
        const v4i arr[1] = {ch};
        store_plain<1>(arr, a, m0 + mm, n0 + 16 * h);
    } else {
        store16(yblk + ((size_t)((n0 >> 5) * 2 + h) * 32 + mm) * 16, ch);
    }
}

// The E4M3 counterpart: ReLU and a requantized E4M3 result in three and a half operations per element.  Equivalent,
// code for code, to the general sequence relu -> *inv -> clamp[-448, 448] (NaN kept) -> convert: a negative y lands on
// zero either way, a NaN does not survive the ReLU in either (the maximum of a NaN and 0 is 0, and so is the median of a
// NaN, 0 and 448), and the conversion instruction rounds to nearest even.
OGC_DEV v4i requant_block_f8_relu(const v16f& acc, const OgcLayerArgs& a, const BlockParams& p) {
    const float inv = a.inv_cs;
    uint32_t dw[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        float t[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float y = __builtin_fmaf(acc[4 * g + e], p.s[g][e], p.b[g][e]);
            t[e] = __builtin_amdgcn_fmed3f(y * inv, 0.0f, 448.0f);
        }
        int r = __builtin_amdgcn_cvt_pk_fp8_f32(t[0], t[1], 0, false);
        dw[g] = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(t[2], t[3], r, true);
    }
    swap32(dw[0], dw[2]);
    swap32(dw[1], dw[3]);
    return (v4i){(int)dw[0], (int)dw[2], (int)dw[1], (int)dw[3]};  // 16 consecutive channels from n0+16h
}

// The ReLU-requantize arithmetic of a block for the dtype at hand (int8: u8 results, E4M3: E4M3 codes).
template <int DT> OGC_DEV v4i requant_block_relu(const typename AccT<DT>::type& acc, const OgcLayerArgs& a, const BlockParams& p) {
    if constexpr (DT == OGC_F8) return requant_block_f8_relu(acc, a, p);
    else return requant_block_i8_relu(acc, a, p);
}

template <int OUT_PLAIN, typename YP>
OGC_DEV void epilogue_block_f8_relu(const v16f& acc, const OgcLayerArgs& a, const BlockParams& p, int n0, int m0, int lane, YP yblk) {
    const int h = lane >> 5, mm = lane & 31;
    const v4i ch = requant_block_f8_relu(acc, a, p);
    if constexpr (OUT_PLAIN) {
        const v4i arr[1] = {ch};
        store_plain<1>(arr, a, m0 + mm, n0 + 16 * h);
    } else {
        store16(yblk + ((size_t)((n0 >> 5) * 2 + h) * 32 + mm) * 16, ch);
    }
}

// Final store of two neighbouring 32-channel blocks of the same 32 rows (u8 results, 64 consecutive bytes per row) to
// the caller's plain y as whole 64-byte row segments: the chunks cross the wave through 2 KiB of LDS (row r keeps
// piece c in slot (c + r/4) mod 4: conflict-free both ways), after which four neighbouring lanes hold one row's
// segment and a store instruction writes 16 rows x 64 bytes instead of 32 rows x two separate 16-byte pieces.
// c0 / c1: the lane's chunk of the block at channels n0 / n0 + 32.  Needs 16-byte aligned rows and N % 64 == 0.
typedef __attribute__((address_space(3))) uint8_t ogc_lds_u8;
OGC_DEV void store_plain_rows64(const v4i& c0, const v4i& c1, const OgcLayerArgs& a, int n0, int m0, int lane, ogc_lds_u8* scratch) {
    typedef __attribute__((address_space(3))) v4i lds_v4i;
    const int r = lane & 31, h = lane >> 5, rot = r >> 2;
    *(lds_v4i*)(scratch + r * 64 + (((h + rot) & 3) << 4)) = c0;
    *(lds_v4i*)(scratch + r * 64 + (((2 + h + rot) & 3) << 4)) = c1;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int rr = pass * 16 + (lane >> 2), c = lane & 3;
        const v4i v = *(const lds_v4i*)(scratch + rr * 64 + (((c + (rr >> 2)) & 3) << 4));
        const int m = m0 + rr;
        if (m < a.M) store16_through(a.y + (long long)m * a.ldy_bytes + n0 + c * 16, v);
    }
}

// One value through activation ACT (a compile-time constant here: the caller branches once per block, not per value).
template <int ACT> OGC_DEV float act_apply1(float y) {
    if constexpr (ACT == OGC_ACT_RELU) return __builtin_fmaxf(y, 0.0f);
    if constexpr (ACT == OGC_ACT_GELU_TANH) {  // as in act_apply16
        const float arg = y * __builtin_fmaf(-0.10294324f, y * y, -2.3022082f);
        return y * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(arg));
    }
    return y;
}

// A quantized block with activation ACT (none, ReLU or GELU) and a requantized result (u8 or E4M3 codes), four values at
// a time: each quad is scaled, activated, rounded and packed into its dword on its own.  Same results as
// epilogue_values + pack_block:
//   int8: clamp(rne(t) + zp, 0, 255) = rne(med3(t, -zp, 255 - zp)) + zp, both bounds being integers; the sum of two
//         integers is exact and `v_cvt_pk_u8_f32` then packs it unchanged; `internal` results are stored as s8 (x ^ 0x80);
//   E4M3: the clamp to +-448 that keeps NaN, then the packed conversion (nearest, ties to even).
template <int DT, int ACT>
OGC_DEV v4i requant_block_act(const typename AccT<DT>::type& acc, const OgcLayerArgs& a, const BlockParams& p, bool internal) {
    static_assert(Quant<DT>::yes, "requantized results are those of the int8 and E4M3 schemes");
    const float inv = a.inv_cs, zp = a.zp_out, lo = -zp, hi = a.q_hi;
    uint32_t dw[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        float t[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float f;
            if constexpr (DT == OGC_I8) f = (float)(acc[4 * g + e] + p.c[g][e]);
            else f = acc[4 * g + e];
            t[e] = act_apply1<ACT>(__builtin_fmaf(f, p.s[g][e], p.b[g][e])) * inv;
        }
        if constexpr (DT == OGC_I8) {
            uint32_t q = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                q = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_rintf(__builtin_amdgcn_fmed3f(t[e], lo, hi)) + zp, e, q);
            dw[g] = internal ? (q ^ 0x80808080u) : q;
        } else {
            dw[g] = f32x4_to_e4m3x4(t[0], t[1], t[2], t[3]);
        }
    }
    swap32(dw[0], dw[2]);
    swap32(dw[1], dw[3]);
    return (v4i){(int)dw[0], (int)dw[2], (int)dw[1], (int)dw[3]};  // 16 consecutive channels from n0+16h
}
// The requantizing arithmetic of a block whose epilogue the caller has fixed at compile time (the stream kernel's EPI:
// 1 ReLU, 3 no activation, 4 GELU), for a result in the caller's plain rows.
template <int DT, int EPI> OGC_DEV v4i requant_block_epi(const typename AccT<DT>::type& acc, const OgcLayerArgs& a, const BlockParams& p) {
    if constexpr (EPI == 1) return requant_block_relu<DT>(acc, a, p);
    else return requant_block_act<DT, EPI == 3 ? OGC_ACT_NONE : OGC_ACT_GELU_TANH>(acc, a, p, false);
}

// PATH: -1 = pick the int8 ReLU-requantize fast path at run time, 1 = the caller knows it applies (only that
// code is generated), 0 = the caller knows it does not; 3 / 4 = the caller knows: a quantized layer without activation /
// with GELU and a requantized result (only that code is generated).
template <int DT, int OUT_PLAIN, bool CALLS = true, int PATH = -1, typename YP>
OGC_DEV void epilogue_block(const typename AccT<DT>::type& acc, const OgcLayerArgs& a, const BlockParams& p, int n0, int m0,
                            int lane, YP yblk) {
    if constexpr (DT == OGC_I8 && (PATH == -1 || PATH == 1)) {
        if (PATH == 1 || (a.act == OGC_ACT_RELU && !a.out_f32)) {
            epilogue_block_i8_relu<OUT_PLAIN>(acc, a, p, n0, m0, lane, yblk);
            return;
        }
    }
    if constexpr (DT == OGC_F8 && PATH == 1) {  // the caller knows: ReLU, E4M3 result
        epilogue_block_f8_relu<OUT_PLAIN>(acc, a, p, n0, m0, lane, yblk);
        return;
    }
    const int h = lane >> 5, mm = lane & 31;
    if constexpr (Quant<DT>::yes && (PATH == 3 || PATH == 4)) {  // the caller knows: no activation / GELU, requantized result
        const v4i ch = requant_block_act<DT, PATH == 3 ? OGC_ACT_NONE : OGC_ACT_GELU_TANH>(acc, a, p, DT == OGC_I8 && !OUT_PLAIN);
        if constexpr (OUT_PLAIN) {
            const v4i arr[1] = {ch};
            store_plain<1>(arr, a, m0 + mm, n0 + 16 * h);
        } else {
            store16(yblk + ((size_t)((n0 >> 5) * 2 + h) * 32 + mm) * 16, ch);
        }
        return;
    }
    float out[16];
    epilogue_values<DT, CALLS>(acc, a, p, out);
    constexpr int E = Elt<DT>::size;
    if constexpr (OUT_PLAIN) {
        if constexpr (!Quant<DT>::yes) {
            if (a.res) add_residual<DT>(out, a, m0 + mm, n0, h);
        }
        if (Quant<DT>::yes && a.out_f32) {
            v4i ch[4];
            pack_block<4>(out, false, ch);
            store_plain<4>(ch, a, m0 + mm, n0 + 16 * h);
        } else {
            v4i ch[E];
            pack_block<E, DT == OGC_F8>(out, false, ch);
            store_plain<E>(ch, a, m0 + mm, n0 + 16 * h);
        }
    } else {
        v4i ch[E];
        pack_block<E, DT == OGC_F8>(out, DT == OGC_I8, ch);
        const int c0 = ((n0 >> 5) * 2 + h) * E;
#pragma unroll
        for (int c = 0; c < E; ++c) store16(yblk + ((size_t)(c0 + c) * 32 + mm) * 16, ch[c]);
    }
}

// Same, reading the block's parameters from the packed blob.
template <int DT, int OUT_PLAIN, bool CALLS = true, typename YP>
OGC_DEV void epilogue_block(const typename AccT<DT>::type& acc, const OgcLayerArgs& a, int n0, int m0, int lane, YP yblk) {
    BlockParams p;
    load_block_params<DT>(p, a, n0, lane >> 5);
    epilogue_block<DT, OUT_PLAIN, CALLS>(acc, a, p, n0, m0, lane, yblk);
}

// Loads one 16-byte chunk (row m, bytes kb..kb+15 of the row) of the caller's plain x, zero-filling
// everything outside [0,M) x [0,K*elt) (pre-op reorder from the plain layout, Section IV, anchor #4).
// u8 inputs are converted to the internal s8 form on the way.
template <int DT> OGC_DEV v4i load_plain_chunk(const OgcLayerArgs& a, int m, int kb) {
    const int kbytes = a.K * Elt<DT>::size;
    v4i v = {0, 0, 0, 0};
    if (m < a.M && kb < kbytes) {
        const uint8_t* p = a.x + (long long)m * a.ldx_bytes + kb;
        if (a.x_vec_ok) {
            v = *(const v4i*)p;
        } else {
            // Rows that are not 16-byte aligned (K = 479 bytes, say): up to five aligned dwords that each hold at
            // least one valid byte (so none lies outside the caller's allocation, whose end is dword aligned),
            // shifted into place; bytes past the row's end are cleared.
            const int n = kbytes - kb < 16 ? kbytes - kb : 16;
            const uintptr_t addr = (uintptr_t)p;
            const uint32_t sh = (uint32_t)(addr & 3);
            const uint32_t* q = (const uint32_t*)(addr - sh);
            const int count = (int)(sh + n + 3) >> 2;
            uint32_t w[5];
#pragma unroll
            for (int j = 0; j < 5; ++j) w[j] = j < count ? q[j] : 0u;
            uint32_t d[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                d[j] = __builtin_amdgcn_alignbyte(w[j + 1], w[j], sh);
                const int rem = n - 4 * j;
                d[j] &= rem >= 4 ? 0xffffffffu : (rem <= 0 ? 0u : (0xffffffffu >> (8 * (4 - rem))));
            }
            v = (v4i){(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
        }
        if constexpr (DT == OGC_I8) {
            // bytes past K hold 0x80 after the flip only if they were flipped: flip valid bytes only
            uint32_t msk[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int rem = kbytes - (kb + 4 * q);
                msk[q] = rem >= 4 ? 0x80808080u : (rem <= 0 ? 0u : (0x80808080u >> (8 * (4 - rem))));
            }
            v = (v4i){(int)((uint32_t)v[0] ^ msk[0]), (int)((uint32_t)v[1] ^ msk[1]), (int)((uint32_t)v[2] ^ msk[2]),
                      (int)((uint32_t)v[3] ^ msk[3])};
        }
    }
    return v;
}

// ------------------------------------------------------------------------------------------------
// Per-layer kernel: one workgroup computes a BN x BM tile of D = W X^T over the whole K, LDS double
// buffered, then runs the epilogue in registers.  Grid: one workgroup per tile, XCD-aware order.
// ------------------------------------------------------------------------------------------------
template <int TILE> struct TileCfg;
template <> struct TileCfg<OGC_TILE_BIG> { enum { WN = 2, WM = 2, TN = 4, TM = 4 }; };
template <> struct TileCfg<OGC_TILE_MID> { enum { WN = 2, WM = 2, TN = 2, TM = 2 }; };
template <> struct TileCfg<OGC_TILE_SMALL> { enum { WN = 2, WM = 1, TN = 1, TM = 1 }; };

template <int DT, int TILE, int X_PLAIN, int OUT_PLAIN>
__global__ void __launch_bounds__(TileCfg<TILE>::WN* TileCfg<TILE>::WM * 64)
ogc_layer_kernel(const OgcLayerArgs a, int tiles_n, int tiles_total, int tiles_per_xcd) {
    typedef TileCfg<TILE> C;
    constexpr int NT = C::WN * C::WM * 64;
    constexpr int BN = C::WN * C::TN * 32, BM = C::WM * C::TM * 32;
    constexpr int W_BYTES = BN * 64, X_BYTES = BM * 64, STAGE = W_BYTES + X_BYTES;
    constexpr int PW = W_BYTES / 16 / NT, PX = X_BYTES / 16 / NT;
    static_assert(PW >= 1 && PX >= 1 && PW * NT * 16 == W_BYTES && PX * NT * 16 == X_BYTES, "tile/thread mismatch");
    extern __shared__ __align__(16) uint8_t smem[];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles so that the
    // workgroups sharing an activation tile share one L2.
    const int wg = blockIdx.x;
    const int t = (wg & 7) * tiles_per_xcd + (wg >> 3);
    if (t >= tiles_total) return;
    const int n_base = (t % tiles_n) * BN, m_base = (t / tiles_n) * BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave % C::WN, wm = wave / C::WN;
    const int KT = a.KC >> 2;  // 64-byte k-steps

    v4i wreg[PW], xreg[PX];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < PW; ++i) {
            const int p = tid + i * NT;
            const uint8_t* g = a.w + ((size_t)((n_base >> 5) + (p >> 7)) * a.KC + (size_t)kt * 4) * 512 + (p & 127) * 16;
            wreg[i] = *(const v4i*)g;
        }
#pragma unroll
        for (int i = 0; i < PX; ++i) {
            const int p = tid + i * NT;
            if constexpr (X_PLAIN) {
                const int mr = p % BM, kc = p / BM;
                xreg[i] = load_plain_chunk<DT>(a, m_base + mr, kt * 64 + kc * 16);
            } else {
                const uint8_t* g = a.x + ((size_t)((m_base >> 5) + (p >> 7)) * a.KC + (size_t)kt * 4) * 512 + (p & 127) * 16;
                xreg[i] = *(const v4i*)g;
            }
        }
    };
    auto store_lds = [&](int buf) {
        uint8_t* ws = smem + buf * STAGE;
        uint8_t* xs = ws + W_BYTES;
#pragma unroll
        for (int i = 0; i < PW; ++i) *(v4i*)(ws + (tid + i * NT) * 16) = wreg[i];
#pragma unroll
        for (int i = 0; i < PX; ++i) {
            const int p = tid + i * NT;
            if constexpr (X_PLAIN) {
                const int mr = p % BM, kc = p / BM;
                *(v4i*)(xs + (((mr >> 5) * 4 + kc) * 32 + (mr & 31)) * 16) = xreg[i];
            } else {
                *(v4i*)(xs + p * 16) = xreg[i];
            }
        }
    };

    typename AccT<DT>::type acc[C::TN][C::TM];
#pragma unroll
    for (int i = 0; i < C::TN; ++i)
#pragma unroll
        for (int j = 0; j < C::TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) load_global(kt + 1);
        const uint8_t* ws = smem + (kt & 1) * STAGE + (wn * C::TN) * 2048 + lane * 16;
        const uint8_t* xs = smem + (kt & 1) * STAGE + W_BYTES + (wm * C::TM) * 2048 + lane * 16;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v4i wf[C::TN], xf[C::TM];
#pragma unroll
            for (int i = 0; i < C::TN; ++i) wf[i] = *(const v4i*)(ws + i * 2048 + s * 1024);
#pragma unroll
            for (int j = 0; j < C::TM; ++j) xf[j] = *(const v4i*)(xs + j * 2048 + s * 1024);
#pragma unroll
            for (int i = 0; i < C::TN; ++i)
#pragma unroll
                for (int j = 0; j < C::TM; ++j) mma32<DT>(acc[i][j], wf[i], xf[j]);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < C::TN; ++i) {
        const int n0 = n_base + (wn * C::TN + i) * 32;
#pragma unroll
        for (int j = 0; j < C::TM; ++j) {
            const int m0 = m_base + (wm * C::TM + j) * 32;
            if constexpr (OUT_PLAIN) {
                if (n0 < a.N && m0 < a.M) epilogue_block<DT, 1>(acc[i][j], a, n0, m0, lane, (uint8_t*)nullptr);
            } else {
                if ((n0 >> 5) < a.NB_out)
                    epilogue_block<DT, 0>(acc[i][j], a, n0, m0, lane, GlobalY{a.y + (size_t)(m0 >> 5) * a.KC_out * 512});
            }
        }
    }
}

#include "ogc_layer_stream.h"

// ------------------------------------------------------------------------------------------------
// Fused multi-layer chain kernel (coarse-grain fusion, Section V: the batch loops of consecutive layers
// are merged, so a batch tile's activations stay in the fastest memory for the next matmul).  One
// workgroup owns 32 batch rows for the whole chain.  The tile's activations ping-pong between two LDS
// buffers in KB16 layout; weights are used once per workgroup and stream from global memory straight
// into the MFMA operand registers (the packed layout is already in lane order, 1 KiB per wave load).
// ------------------------------------------------------------------------------------------------
#define OGC_FUSED_WAVES 8
#define OGC_FUSED_THREADS (OGC_FUSED_WAVES * 64)

// CNT output-channel blocks of one wave at a time: the activation operand read from LDS feeds CNT MFMAs, and
// the CNT accumulator chains overlap (a single chain would wait out the full MFMA latency at every k-step).
// stride: distance in channel blocks between a wave's consecutive blocks (the number of waves that share the layer).
template <int DT, int OUT_PLAIN, int CNT, class YT>
OGC_DEV void fused_blocks(const OgcLayerArgs& a, const uint8_t* xin, YT xout, int m0, int nb0, int lane, int stride) {
    const int KP2 = a.KC >> 1;  // 32-byte k-steps
    typename AccT<DT>::type acc[CNT];
#pragma unroll
    for (int i = 0; i < CNT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    const uint8_t* wp = a.w + (size_t)nb0 * a.KC * 512 + lane * 16;
    const size_t wstep = (size_t)stride * a.KC * 512;  // this wave's next block is `stride` further
    const uint8_t* xp = xin + lane * 16;
    int kp = 0;
    for (; kp + 4 <= KP2; kp += 4) {
        v4i wf[CNT][4], xf[4];
#pragma unroll
        for (int i = 0; i < CNT; ++i)
#pragma unroll
            for (int u = 0; u < 4; ++u) wf[i][u] = *(const v4i*)(wp + i * wstep + (size_t)(kp + u) * 1024);
#pragma unroll
        for (int u = 0; u < 4; ++u) xf[u] = *(const v4i*)(xp + (size_t)(kp + u) * 1024);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < CNT; ++i) mma32<DT>(acc[i], wf[i][u], xf[u]);
    }
    for (; kp < KP2; ++kp) {
        const v4i xf = *(const v4i*)(xp + (size_t)kp * 1024);
#pragma unroll
        for (int i = 0; i < CNT; ++i) mma32<DT>(acc[i], *(const v4i*)(wp + i * wstep + (size_t)kp * 1024), xf);
    }
#pragma unroll
    for (int i = 0; i < CNT; ++i) epilogue_block<DT, OUT_PLAIN>(acc[i], a, (nb0 + i * stride) * 32, m0, lane, xout);
}

// One layer of the fused chain for a 32-row tile: wave w of `waves` (the eight of one workgroup, or those of all
// the workgroups that share the tile) owns the channel blocks w, w + waves, w + 2 waves, ...
template <int DT, int OUT_PLAIN, class YT>
OGC_DEV void fused_layer(const OgcLayerArgs& a, const uint8_t* xin, YT xout, int m0, int wave, int waves, int lane) {
    const int nblocks = OUT_PLAIN ? ((a.N + 31) >> 5) : a.NB_out;
    for (int nb0 = wave; nb0 < nblocks; nb0 += 4 * waves) {
        const int cnt = (nblocks - nb0 + waves - 1) / waves;  // blocks of this wave from nb0 on
        if (cnt >= 4) fused_blocks<DT, OUT_PLAIN, 4>(a, xin, xout, m0, nb0, lane, waves);
        else if (cnt == 3) fused_blocks<DT, OUT_PLAIN, 3>(a, xin, xout, m0, nb0, lane, waves);
        else if (cnt == 2) fused_blocks<DT, OUT_PLAIN, 2>(a, xin, xout, m0, nb0, lane, waves);
        else fused_blocks<DT, OUT_PLAIN, 1>(a, xin, xout, m0, nb0, lane, waves);
    }
}

template <int DT>
__global__ void __launch_bounds__(OGC_FUSED_THREADS) ogc_fused_chain_kernel(const OgcChainArgs c) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroup b runs on XCD b%8.  A small batch is kept on few XCDs so that their L2s fetch the weights once
    // for all of their workgroups; the workgroups dealt to the other XCDs leave at once.
    const int xcd = blockIdx.x & 7;
    const int tile = (blockIdx.x >> 3) * c.fused_xcds + xcd;
    if (xcd >= c.fused_xcds || tile >= c.fused_tiles) return;
    const int m0 = tile * 32;
    uint8_t* buf0 = smem;
    uint8_t* buf1 = smem + c.lds_buf_bytes;

    // Stage the plain input tile into LDS in operand layout (pre-op reorder fused at the chain entry).
    {
        const OgcLayerArgs& a = c.layer[0];
        const int pieces = a.KC * 32;
        for (int p = tid; p < pieces; p += OGC_FUSED_THREADS) {
            const int mr = p & 31, kc = p >> 5;
            *(v4i*)(buf0 + (size_t)p * 16) = load_plain_chunk<DT>(a, m0 + mr, kc * 16);
        }
    }
    __syncthreads();
    for (int l = 0; l < c.n_layers; ++l) {
        const uint8_t* xin = (l & 1) ? buf1 : buf0;
        uint8_t* xout = (l & 1) ? buf0 : buf1;
        if (l + 1 < c.n_layers) {
            fused_layer<DT, 0>(c.layer[l], xin, xout, m0, wave, OGC_FUSED_WAVES, lane);
            __syncthreads();
        } else {
            fused_layer<DT, 1>(c.layer[l], xin, (uint8_t*)nullptr, m0, wave, OGC_FUSED_WAVES, lane);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Constant-weight preprocessing (Section V): plain [K,N] -> KB16 blocked, zero padded; per-channel
// parameters.  One thread per 16-byte chunk / per channel.
// ------------------------------------------------------------------------------------------------
__global__ void ogc_prepack_weights_kernel(const uint8_t* __restrict__ w, uint8_t* __restrict__ out, int K, int N, int KC,
                                           int NPw, int esz) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = (long long)(NPw >> 5) * KC * 32;
    if (idx >= total) return;
    const int r = (int)(idx & 31);
    const long long q = idx >> 5;
    const int c = (int)(q % KC);
    const int nb = (int)(q / KC);
    const int n = nb * 32 + r;
    const int epc = 16 / esz;  // elements per chunk
    uint32_t d[4] = {0, 0, 0, 0};
    if (n < N) {
        for (int j = 0; j < epc; ++j) {
            const int k = c * epc + j;
            if (k < K) {
                const uint8_t* src = w + ((size_t)k * N + n) * esz;
                for (int b = 0; b < esz; ++b) {
                    const int byte = j * esz + b;
                    d[byte >> 2] |= (uint32_t)src[b] << (8 * (byte & 3));
                }
            }
        }
    }
    *(v4i*)(out + (size_t)idx * 16) = (v4i){(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
}

// Per-channel parameters.  A workgroup covers 64 channels; its eight waves take every eighth row of the plain [K,N]
// weights each (a wave's 64 lanes read 64 consecutive bytes of a row) and their partial column sums are added through
// LDS.  The sums are integers: the order does not matter.
#define OGC_PARAMS_SLICES 8
__global__ void __launch_bounds__(64 * OGC_PARAMS_SLICES)
ogc_prepack_params_kernel(int dtype, const int8_t* __restrict__ wq, const float* __restrict__ w_scale,
                          const float* __restrict__ bias, float in_scale, int in_zp, int K, int N, int NPw,
                          float* __restrict__ scale_out, float* __restrict__ bias_out, int32_t* __restrict__ ncomp_out) {
    __shared__ int32_t part[OGC_PARAMS_SLICES][64];
    const int col = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + col;
    const bool valid = n < N;
    int32_t wsum = 0;
    if (dtype == OGC_I8 && valid) {
        const int8_t* p = wq + n;
        int k = slice;
        for (; k + 3 * OGC_PARAMS_SLICES < K; k += 4 * OGC_PARAMS_SLICES) {  // four rows in flight
            const int32_t a = p[(size_t)k * N], b = p[(size_t)(k + OGC_PARAMS_SLICES) * N];
            const int32_t c = p[(size_t)(k + 2 * OGC_PARAMS_SLICES) * N], d = p[(size_t)(k + 3 * OGC_PARAMS_SLICES) * N];
            wsum += (a + b) + (c + d);
        }
        for (; k < K; k += OGC_PARAMS_SLICES) wsum += (int32_t)p[(size_t)k * N];
    }
    part[slice][col] = wsum;
    __syncthreads();
    if (slice != 0 || n >= NPw) return;
    bias_out[n] = (valid && bias) ? bias[n] : 0.0f;
    if (dtype == OGC_I8) {
        int32_t total = 0;
#pragma unroll
        for (int s2 = 0; s2 < OGC_PARAMS_SLICES; ++s2) total += part[s2][col];
        ncomp_out[n] = -(in_zp - 128) * total;
    }
    if (dtype == OGC_I8 || dtype == OGC_F8) scale_out[n] = valid ? in_scale * w_scale[n] : 0.0f;
}

// Quantize / dequantize nodes of the low-precision graph (Section V) for E4M3 tensors at the boundary: elementwise,
// four elements per thread, the same reciprocal multiply, rounding and saturation as a layer's requantized output.
__global__ void ogc_quantize_e4m3_kernel(const float* __restrict__ x, uint8_t* __restrict__ out, size_t n, float inv_scale) {
    const size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= n) return;
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = i + j < n ? x[i + j] * inv_scale : 0.0f;
    const uint32_t q = f32x4_to_e4m3x4(v[0], v[1], v[2], v[3]);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (i + j < n) out[i + j] = (uint8_t)(q >> (8 * j));
}
__global__ void ogc_dequantize_e4m3_kernel(const uint8_t* __restrict__ x, float* __restrict__ out, size_t n, float scale) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    out[i] = __builtin_amdgcn_cvt_f32_fp8((int)x[i], 0) * scale;
}
extern "C" int ogc_launch_quantize_e4m3(const float* x, uint8_t* out, size_t n, float inv_scale, void* stream) {
    const size_t threads = (n + 3) / 4, blocks = (threads + 255) / 256;
    if (blocks == 0) return 0;
    if (blocks > 0x7fffffffu) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(ogc_quantize_e4m3_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, x, out, n, inv_scale);
    return (int)hipGetLastError();
}
extern "C" int ogc_launch_dequantize_e4m3(const uint8_t* x, float* out, size_t n, float scale, void* stream) {
    const size_t blocks = (n + 255) / 256;
    if (blocks == 0) return 0;
    if (blocks > 0x7fffffffu) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(ogc_dequantize_e4m3_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, x, out, n, scale);
    return (int)hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Launchers
// ------------------------------------------------------------------------------------------------
template <int TILE> static OgcTileInfo tile_info_t() {
    typedef TileCfg<TILE> C;
    OgcTileInfo i;
    i.bn = C::WN * C::TN * 32;
    i.bm = C::WM * C::TM * 32;
    i.threads = C::WN * C::WM * 64;
    i.lds_bytes = (size_t)2 * (i.bn + i.bm) * 64;
    return i;
}

extern "C" OgcTileInfo ogc_tile_info(int tile) {
    if (tile == OGC_TILE_DMA || tile == OGC_TILE_DMA8 || tile == OGC_TILE_DMAK2) {
        OgcTileInfo i;
        if (tile == OGC_TILE_DMA) {
            typedef StreamCfg<0> C;
            i.bn = C::BN, i.bm = C::BM, i.threads = C::NT, i.lds_bytes = C::LDS;
        } else if (tile == OGC_TILE_DMAK2) {
            typedef StreamCfg<2> C;
            i.bn = C::BN, i.bm = C::BM, i.threads = C::NT, i.lds_bytes = C::LDS;
        } else {
            typedef StreamCfg<1> C;
            i.bn = C::BN, i.bm = C::BM, i.threads = C::NT, i.lds_bytes = C::LDS;
        }
        return i;
    }
    switch (tile) {
    case OGC_TILE_BIG: return tile_info_t<OGC_TILE_BIG>();
    case OGC_TILE_MID: return tile_info_t<OGC_TILE_MID>();
    default: return tile_info_t<OGC_TILE_SMALL>();
    }
}

// ------------------------------------------------------------------------------------------------
// Cooperative chain kernel for small batches (the multi-core loop and k-slicing of Section III applied to
// shapes where one workgroup per row tile leaves most CUs idle).  One launch for the whole chain; every
// resident workgroup takes 32x32 output blocks of the current layer (block b -> workgroup b mod G), its eight
// waves split the reduction axis between them (wave w takes the 32-byte k-steps w, w+8, ...) and add their
// partial sums through LDS in a fixed order; between layers all workgroups meet at a barrier on a counter in
// global memory.  Activations travel through the workspace buffers in the blocked layout.
//
// Cross-XCD visibility without cache maintenance: results are stored with write-through system-scope stores and
// every wave waits for its stores before its workgroup arrives at the barrier (an agent-scope atomic add); a
// workgroup leaves the barrier when an agent-scope atomic load shows all arrivals, and reads the other
// workgroups' results with system-scope loads, which no stale cache line can serve.  (Agent-scope release /
// acquire fences instead cost 4-5 us per barrier: they write back and invalidate whole L2s.)
// All workgroups must be resident at once: the grid is at most one workgroup per CU.  A cooperative launch
// would guarantee that but costs 18 us per call on this stack, more than the kernel saves, so the launch is
// an ordinary one and the barrier wait is bounded instead (about 2^22 polls, seconds): a device kept busy by
// another kernel for longer than that makes this chain finish with wrong data rather than hang.
// sync[0]: barrier arrivals, sync[1]: workgroups finished.  Both are zero between runs: prepack zeroes them and
// the last workgroup to finish a run zeroes them again (by then nobody waits on them).
// ------------------------------------------------------------------------------------------------
// Partial accumulators of the k-slices of a workgroup's waves travel through LDS as four 16-byte pieces per lane
// ([wave][piece][lane]: consecutive lanes, consecutive 16 bytes, so the 128-bit LDS accesses are conflict-free).
template <int DT> OGC_DEV void partial_store(v4i (*red)[4][64], int slot, int lane, const typename AccT<DT>::type& acc) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if constexpr (DT == OGC_I8) {
            red[slot][q][lane] = (v4i){acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        } else {
            const v4f t = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
            red[slot][q][lane] = __builtin_bit_cast(v4i, t);
        }
    }
}
template <int DT> OGC_DEV void partial_add(v4i (*red)[4][64], int slot, int lane, typename AccT<DT>::type& acc) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const v4i v = red[slot][q][lane];
        if constexpr (DT == OGC_I8) {
            acc[4 * q] += v[0], acc[4 * q + 1] += v[1], acc[4 * q + 2] += v[2], acc[4 * q + 3] += v[3];
        } else {
            const v4f t = __builtin_bit_cast(v4f, v);
            acc[4 * q] += t[0], acc[4 * q + 1] += t[1], acc[4 * q + 2] += t[2], acc[4 * q + 3] += t[3];
        }
    }
}

#define OGC_COOP_WAVES 8  // measured against 4 and 16: 10-25 % faster than 4 on 1024- and 2048-wide layers
#define OGC_COOP_U 4      // k-steps a wave keeps in flight (8 measured: no better)
#define OGC_COOP_THREADS (OGC_COOP_WAVES * 64)

// The wait of a barrier on a counter in global memory, after the caller's waves have synchronised: thread 0 arrives and
// polls until `target` arrivals or until `budget` polls have passed.  A wait that gives up sets the error word of the
// sync area (system scope: the host reads it, ogc_mlp_check) and the function returns false in every thread of the
// workgroup, which then abandons the rest of the chain; the workgroups still waiting for it give up the same way, so
// every workgroup exits.  flag: four bytes of LDS that are free at this point (the verdict crosses the workgroup there).
OGC_DEV bool barrier_wait(unsigned long long* ctr, unsigned long long target, int budget, unsigned long long* err, int* flag,
                          int tid) {
    if (tid == 0) {
        __hip_atomic_fetch_add(ctr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool reached = false;
        for (int polls = 0; polls < budget; ++polls) {
            if (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) {
                reached = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!reached) __hip_atomic_store(err, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        *(volatile int*)flag = reached ? 1 : 0;
    }
    __syncthreads();
    const bool ok = *(volatile int*)flag != 0;
    __syncthreads();  // the caller reuses the flag's storage
    return ok;
}

OGC_DEV bool coop_grid_barrier(unsigned long long* ctr, unsigned long long target, int budget, unsigned long long* err, int* flag,
                               int tid) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's result stores (inline assembly) have completed
    __syncthreads();
    return barrier_wait(ctr, target, budget, err, flag, tid);
}

// 16 bytes of another workgroup's result, read coherently at system scope (two relaxed 64-bit atomic loads)
OGC_DEV v4i load16_coherent(const uint8_t* p) {
    const unsigned long long lo = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    const unsigned long long hi = __hip_atomic_load((const unsigned long long*)(p + 8), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return (v4i){(int)(uint32_t)lo, (int)(uint32_t)(lo >> 32), (int)(uint32_t)hi, (int)(uint32_t)(hi >> 32)};
}

// four 16-byte pieces of other workgroups' results, read at system scope, in flight together
OGC_DEV void load16x4_coherent(const uint8_t* p0, const uint8_t* p1, const uint8_t* p2, const uint8_t* p3, v4i (&v)[4]) {
    asm volatile("global_load_dwordx4 %0, %4, off sc0 sc1\n\t"
                 "global_load_dwordx4 %1, %5, off sc0 sc1\n\t"
                 "global_load_dwordx4 %2, %6, off sc0 sc1\n\t"
                 "global_load_dwordx4 %3, %7, off sc0 sc1\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
                 : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
                 : "memory");
}

// eight pieces in flight: the copy of a wide tile back into LDS is a few such batches, each one round trip
OGC_DEV void load16x8_coherent(const uint8_t* p, size_t stride, v4i (&v)[8]) {
    const uint8_t *p1 = p + stride, *p2 = p + 2 * stride, *p3 = p + 3 * stride, *p4 = p + 4 * stride, *p5 = p + 5 * stride,
                  *p6 = p + 6 * stride, *p7 = p + 7 * stride;
    asm volatile("global_load_dwordx4 %0, %8, off sc0 sc1\n\t"
                 "global_load_dwordx4 %1, %9, off sc0 sc1\n\t"
                 "global_load_dwordx4 %2, %10, off sc0 sc1\n\t"
                 "global_load_dwordx4 %3, %11, off sc0 sc1\n\t"
                 "global_load_dwordx4 %4, %12, off sc0 sc1\n\t"
                 "global_load_dwordx4 %5, %13, off sc0 sc1\n\t"
                 "global_load_dwordx4 %6, %14, off sc0 sc1\n\t"
                 "global_load_dwordx4 %7, %15, off sc0 sc1\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
                 : "v"(p), "v"(p1), "v"(p2), "v"(p3), "v"(p4), "v"(p5), "v"(p6), "v"(p7)
                 : "memory");
}

// Copies a tile's image (pieces x 16 bytes, written by other workgroups) from global memory into LDS.
OGC_DEV void copy_tile_coherent(uint8_t* lds, const uint8_t* g, int pieces, int tid) {
    constexpr size_t T = OGC_FUSED_THREADS;
    int p = tid;
    for (; p + 7 * (int)T < pieces; p += 8 * (int)T) {
        v4i v[8];
        load16x8_coherent(g + (size_t)p * 16, T * 16, v);
#pragma unroll
        for (int u = 0; u < 8; ++u) *(v4i*)(lds + ((size_t)p + u * T) * 16) = v[u];
    }
    for (; p + 3 * (int)T < pieces; p += 4 * (int)T) {
        v4i v[4];
        const uint8_t* q = g + (size_t)p * 16;
        load16x4_coherent(q, q + T * 16, q + 2 * T * 16, q + 3 * T * 16, v);
#pragma unroll
        for (int u = 0; u < 4; ++u) *(v4i*)(lds + ((size_t)p + u * T) * 16) = v[u];
    }
    for (; p < pieces; p += (int)T) *(v4i*)(lds + (size_t)p * 16) = load16_coherent(g + (size_t)p * 16);
}

template <int DT>
__global__ void __launch_bounds__(OGC_COOP_THREADS) ogc_coop_chain_kernel(const OgcChainArgs c, unsigned long long* sync, int m_blocks) {
    __shared__ v4i red[OGC_COOP_WAVES - 1][4][64];  // partial accumulators of waves 1..7
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = gridDim.x, wg = blockIdx.x;
    for (int l = 0; l < c.n_layers; ++l) {
        const OgcLayerArgs& a = c.layer[l];
        const bool first = l == 0, last = l + 1 == c.n_layers;
        const int nb = last ? ((a.N + 31) >> 5) : a.NB_out;
        const int blocks = m_blocks * nb;
        const int KP2 = a.KC >> 1;  // 32-byte k-steps
        for (int b = wg; b < blocks; b += G) {
            const int bm = b / nb, bn = b - bm * nb;
            typename AccT<DT>::type acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0;
            const uint8_t* wp = a.w + (size_t)bn * a.KC * 512 + lane * 16;
            const uint8_t* xp = a.x + (size_t)bm * a.KC * 512 + lane * 16;  // blocked input (layers after the first)
            const int row = bm * 32 + (lane & 31), kb0 = (lane >> 5) * 16;   // plain input (first layer)
            int kp = wave;
            for (; kp + (OGC_COOP_U - 1) * OGC_COOP_WAVES < KP2; kp += OGC_COOP_U * OGC_COOP_WAVES) {  // k-steps of this wave in flight
                v4i wf[OGC_COOP_U], xf[OGC_COOP_U];
#pragma unroll
                for (int u = 0; u < OGC_COOP_U; ++u) wf[u] = *(const v4i*)(wp + (size_t)(kp + u * OGC_COOP_WAVES) * 1024);
                if (first) {
#pragma unroll
                    for (int u = 0; u < OGC_COOP_U; ++u) xf[u] = load_plain_chunk<DT>(a, row, (kp + u * OGC_COOP_WAVES) * 32 + kb0);
                } else {
                    static_assert(OGC_COOP_U == 4, "the coherent load below takes four pieces");
                    const uint8_t* g = xp + (size_t)kp * 1024;
                    load16x4_coherent(g, g + OGC_COOP_WAVES * 1024, g + 2 * OGC_COOP_WAVES * 1024, g + 3 * OGC_COOP_WAVES * 1024, xf);
                }
#pragma unroll
                for (int u = 0; u < OGC_COOP_U; ++u) mma32<DT>(acc, wf[u], xf[u]);
            }
            for (; kp < KP2; kp += OGC_COOP_WAVES) {
                const v4i wf = *(const v4i*)(wp + (size_t)kp * 1024);
                const v4i xf = first ? load_plain_chunk<DT>(a, row, kp * 32 + kb0)
                                     : load16_coherent(xp + (size_t)kp * 1024);
                mma32<DT>(acc, wf, xf);
            }
            // k-slices of waves 1..7 to LDS, wave 0 adds them in ascending order (a fixed order: deterministic)
            if (wave > 0) partial_store<DT>(red, wave - 1, lane, acc);
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int w = 0; w < OGC_COOP_WAVES - 1; ++w) partial_add<DT>(red, w, lane, acc);
                if (last) epilogue_block<DT, 1>(acc, a, bn * 32, bm * 32, lane, (uint8_t*)nullptr);
                else epilogue_block<DT, 0>(acc, a, bn * 32, bm * 32, lane, GlobalY{a.y + (size_t)bm * a.KC_out * 512});
            }
            __syncthreads();  // red is reused by the next block
        }
        if (!last && !coop_grid_barrier(sync, (unsigned long long)(l + 1) * G + c.barrier_extra, c.barrier_budget,
                                        sync + OGC_SYNC_ERR_WORD, (int*)&red[0][0][0], tid))
            break;  // the wait gave up (recorded in the sync area): the rest of the chain is abandoned
    }
    // the last workgroup out resets the counters for the next run
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        const unsigned long long done = __hip_atomic_fetch_add(sync + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (done == (unsigned long long)G - 1) {
            __hip_atomic_store(sync, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(sync + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__global__ void ogc_zero_sync_kernel(unsigned long long* sync) {
    for (int i = threadIdx.x; i < OGC_SYNC_WORDS; i += blockDim.x) sync[i] = 0;
}

// ------------------------------------------------------------------------------------------------
// Cluster chain kernel: the fused chain kernel with every 32-row tile shared by `split` workgroups.  Each member
// keeps the whole tile's activations in LDS and computes every split-th group of eight channel blocks of each layer,
// so it streams 1/split of the weights (the fused kernel's time is one CU streaming ALL the weights);
// between layers the members write their channel blocks to the workspace, meet at a barrier of their own (a
// counter per tile) and copy the complete tile back into LDS.  The members of a tile sit on one XCD (workgroup b
// runs on XCD b%8): their exchange stays in that XCD's L2.  Visibility does not depend on that placement: stores are
// written through and the copy back uses system-scope loads, as in the cooperative kernel above, whose bounded
// barrier wait and counter reset this kernel shares.  sync[1]: workgroups finished; sync[2 + tile]: arrivals.
// ------------------------------------------------------------------------------------------------
template <int DT>
__global__ void __launch_bounds__(OGC_FUSED_THREADS) ogc_cluster_chain_kernel(const OgcChainArgs c, unsigned long long* sync) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = c.cluster_split;
    int tile, member;
    if (c.fused_xcds == 0) {  // members of a tile on consecutive workgroups: spread over the XCDs
        tile = blockIdx.x / S, member = blockIdx.x % S;
    } else {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        tile = (slot / S) * c.fused_xcds + xcd, member = slot % S;
        if (xcd >= c.fused_xcds || tile >= c.fused_tiles) return;
    }
    const int m0 = tile * 32;
    // the members' waves are numbered member-fastest: a layer with fewer channel blocks than waves still gives every
    // member its share (wave w of member j is wave w*S + j of the tile)
    const int vwave = wave * S + member, vwaves = S * OGC_FUSED_WAVES;
    uint8_t* buf0 = smem;
    uint8_t* buf1 = smem + c.lds_buf_bytes;
    {
        const OgcLayerArgs& a = c.layer[0];
        const int pieces = a.KC * 32;
        for (int p = tid; p < pieces; p += OGC_FUSED_THREADS) {
            const int mr = p & 31, kc = p >> 5;
            *(v4i*)(buf0 + (size_t)p * 16) = load_plain_chunk<DT>(a, m0 + mr, kc * 16);
        }
    }
    __syncthreads();
    unsigned long long* ctr = sync + (size_t)tile * OGC_SYNC_STRIDE;  // [0] arrivals, [1] members finished
    int barriers = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        const OgcLayerArgs& a = c.layer[l];
        const uint8_t* xin = (l & 1) ? buf1 : buf0;
        uint8_t* xout = (l & 1) ? buf0 : buf1;
        if (l + 1 < c.n_layers && ((c.cluster_whole_mask >> l) & 1)) {
            // a layer too small to be worth an exchange: every member computes all of it, as the fused kernel does
            fused_layer<DT, 0>(a, xin, xout, m0, wave, OGC_FUSED_WAVES, lane);
            __syncthreads();
        } else if (l + 1 < c.n_layers) {
            // the tile in blocked layout = its LDS image; a.y is the layer's exchange slot, in which every tile owns a
            // region at a fixed stride (not the layer's own row-block size: a tile two layers ahead of its neighbour
            // must not reach into the neighbour's region)
            uint8_t* ytile = a.y + (size_t)tile * c.cluster_tile_stride;
            fused_layer<DT, 0>(a, xin, GlobalY{ytile}, m0, vwave, vwaves, lane);
            // xout is free until the copy below fills it: its first bytes carry the barrier's verdict
            if (!coop_grid_barrier(ctr, (unsigned long long)(++barriers) * S + c.barrier_extra, c.barrier_budget,
                                   sync + OGC_SYNC_ERR_WORD, (int*)xout, tid))
                break;
            copy_tile_coherent(xout, ytile, a.KC_out * 32, tid);
            __syncthreads();
        } else {
            fused_layer<DT, 1>(a, xin, (uint8_t*)nullptr, m0, vwave, vwaves, lane);
        }
    }
    // the last member out resets its tile's counters for the next run (by then nobody waits on them)
    if (barriers > 0) {
        __syncthreads();
        if (tid == 0) {
            const unsigned long long done = __hip_atomic_fetch_add(ctr + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == (unsigned long long)S - 1) {
                __hip_atomic_store(ctr, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(ctr + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Cluster chain kernel with the reduction axis split inside a workgroup: the members of a tile take whole channel
// blocks (member j: blocks j, j + split, ...) and the eight waves of a member split K between them, as in the
// cooperative kernel, but with the activations read from the member's LDS copy of the tile instead of global
// memory.  For chains whose matrix work per block is large against its weight stream (fp32: a 32x32 block over
// K = 1024 is 3.4 us of one CU's MFMA rate), where splitting the channel blocks alone leaves most waves idle.
// One LDS activation buffer: a layer's input is dead once its members have met at the barrier, and the copy of the
// layer's output takes its place; the reduction scratch (waves 1..7, 28 KiB) follows it.  Every layer but the
// last is exchanged.
// ------------------------------------------------------------------------------------------------
#define OGC_KS_RED_BYTES ((OGC_FUSED_WAVES - 1) * 16 * 64 * 4)

template <int DT>
__global__ void __launch_bounds__(OGC_FUSED_THREADS) ogc_cluster_ksplit_chain_kernel(const OgcChainArgs c, unsigned long long* sync) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = c.cluster_split;
    int tile, member;
    if (c.fused_xcds == 0) {
        tile = blockIdx.x / S, member = blockIdx.x % S;
    } else {
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        tile = (slot / S) * c.fused_xcds + xcd, member = slot % S;
        if (xcd >= c.fused_xcds || tile >= c.fused_tiles) return;
    }
    const int m0 = tile * 32;
    uint8_t* buf = smem;
    v4i(*red)[4][64] = (v4i(*)[4][64])(smem + c.lds_buf_bytes);
    {
        const OgcLayerArgs& a = c.layer[0];
        const int pieces = a.KC * 32;
        for (int p = tid; p < pieces; p += OGC_FUSED_THREADS) {
            const int mr = p & 31, kc = p >> 5;
            *(v4i*)(buf + (size_t)p * 16) = load_plain_chunk<DT>(a, m0 + mr, kc * 16);
        }
    }
    __syncthreads();
    unsigned long long* ctr = sync + (size_t)tile * OGC_SYNC_STRIDE;  // [0] arrivals, [1] members finished
    int barriers = 0;
    v4i wfirst[4];
    bool have_first = false;
    for (int l = 0; l < c.n_layers; ++l) {
        const OgcLayerArgs& a = c.layer[l];
        const bool last = l + 1 == c.n_layers;
        const int nb = last ? ((a.N + 31) >> 5) : a.NB_out;
        const int KP2 = a.KC >> 1;  // 32-byte k-steps
        uint8_t* ytile = last ? nullptr : a.y + (size_t)tile * c.cluster_tile_stride;  // fixed stride: see the kernel above
        for (int bn = member; bn < nb; bn += S) {
            typename AccT<DT>::type acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0;
            const uint8_t* wp = a.w + (size_t)bn * a.KC * 512 + lane * 16;
            const uint8_t* xp = buf + lane * 16;
            int kp = wave;
            if (have_first) {  // this member's first block of the layer: its first weight group came in under the barrier
                have_first = false;
                v4i xf[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) xf[u] = *(const v4i*)(xp + (size_t)(kp + u * OGC_FUSED_WAVES) * 1024);
#pragma unroll
                for (int u = 0; u < 4; ++u) mma32<DT>(acc, wfirst[u], xf[u]);
                kp += 4 * OGC_FUSED_WAVES;
            }
            for (; kp + 3 * OGC_FUSED_WAVES < KP2; kp += 4 * OGC_FUSED_WAVES) {  // four k-steps of this wave in flight
                v4i wf[4], xf[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) wf[u] = *(const v4i*)(wp + (size_t)(kp + u * OGC_FUSED_WAVES) * 1024);
#pragma unroll
                for (int u = 0; u < 4; ++u) xf[u] = *(const v4i*)(xp + (size_t)(kp + u * OGC_FUSED_WAVES) * 1024);
#pragma unroll
                for (int u = 0; u < 4; ++u) mma32<DT>(acc, wf[u], xf[u]);
            }
            for (; kp < KP2; kp += OGC_FUSED_WAVES) mma32<DT>(acc, *(const v4i*)(wp + (size_t)kp * 1024), *(const v4i*)(xp + (size_t)kp * 1024));
            // k-slices of waves 1..7 to LDS, wave 0 adds them in ascending order (a fixed order: deterministic)
            if (wave > 0) partial_store<DT>(red, wave - 1, lane, acc);
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int w = 0; w < OGC_FUSED_WAVES - 1; ++w) partial_add<DT>(red, w, lane, acc);
                if (last) epilogue_block<DT, 1>(acc, a, bn * 32, m0, lane, (uint8_t*)nullptr);
                else epilogue_block<DT, 0>(acc, a, bn * 32, m0, lane, GlobalY{ytile});
            }
            __syncthreads();  // red is reused by the next block
        }
        if (!last) {
            // The barrier of the tile's members, with the next layer's first weight loads of this wave issued before it:
            // they do not depend on the exchange and arrive while the members wait for each other.  Only wave 0
            // has result stores to wait for; it issues its loads after that wait.
            if (wave == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            {
                const OgcLayerArgs& an = c.layer[l + 1];
                const int nbn = (l + 2 == c.n_layers) ? ((an.N + 31) >> 5) : an.NB_out;
                have_first = member < nbn && wave + 3 * OGC_FUSED_WAVES < (an.KC >> 1);
                if (have_first) {
                    const uint8_t* wn = an.w + (size_t)member * an.KC * 512 + lane * 16;
#pragma unroll
                    for (int u = 0; u < 4; ++u) wfirst[u] = *(const v4i*)(wn + (size_t)(wave + u * OGC_FUSED_WAVES) * 1024);
                }
            }
            ++barriers;
            __syncthreads();
            // bounded, as in the cooperative kernel's barrier; the reduction scratch is free here and carries the verdict
            if (!barrier_wait(ctr, (unsigned long long)barriers * S + c.barrier_extra, c.barrier_budget, sync + OGC_SYNC_ERR_WORD,
                              (int*)&red[0][0][0], tid))
                break;
            copy_tile_coherent(buf, ytile, a.KC_out * 32, tid);
            __syncthreads();
        }
    }
    if (barriers > 0) {
        __syncthreads();
        if (tid == 0) {
            const unsigned long long done = __hip_atomic_fetch_add(ctr + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == (unsigned long long)S - 1) {
                __hip_atomic_store(ctr, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(ctr + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// Second pass of a split-K layer: adds the partial accumulators of the k ranges in ascending order (a fixed
// order: the result does not depend on which workgroup finished first) and applies the ordinary epilogue.
// One wave per 32x32 block; the partial buffer holds every wave's accumulator registers as they were.
template <int DT, int OUT_PLAIN>
__global__ void __launch_bounds__(256) ogc_splitk_reduce_kernel(const OgcLayerArgs a, int nb, int total_blocks) {
    const int lane = threadIdx.x & 63;
    const int blk = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (blk >= total_blocks) return;
    const int bm = blk / nb, bn = blk - bm * nb;
    const int ranges = 1 << a.ksplit_log2;
    const size_t range_stride = (size_t)a.pmb * a.pnb * 4096;
    const uint8_t* src = a.partial + ((size_t)bm * a.pnb + bn) * 4096 + lane * 16;
    typename AccT<DT>::type acc;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if constexpr (DT == OGC_I8) {
            v4i sum = *(const v4i*)(src + q * 1024);
            for (int r = 1; r < ranges; ++r) sum += *(const v4i*)(src + r * range_stride + q * 1024);
            acc[4 * q] = sum.x, acc[4 * q + 1] = sum.y, acc[4 * q + 2] = sum.z, acc[4 * q + 3] = sum.w;
        } else {
            v4f sum = *(const v4f*)(src + q * 1024);
            for (int r = 1; r < ranges; ++r) sum += *(const v4f*)(src + r * range_stride + q * 1024);
            acc[4 * q] = sum.x, acc[4 * q + 1] = sum.y, acc[4 * q + 2] = sum.z, acc[4 * q + 3] = sum.w;
        }
    }
    if constexpr (OUT_PLAIN) epilogue_block<DT, 1>(acc, a, bn * 32, bm * 32, lane, (uint8_t*)nullptr);
    else epilogue_block<DT, 0>(acc, a, bn * 32, bm * 32, lane, GlobalY{a.y + (size_t)bm * a.KC_out * 512});
}

template <int DT> static int launch_splitk_reduce(int op, const OgcLayerArgs* a, hipStream_t stream) {
    const int nb = op ? (a->N + 31) / 32 : a->NB_out;
    const int total = ((a->M + 31) / 32) * nb;
    if (op) hipLaunchKernelGGL((ogc_splitk_reduce_kernel<DT, 1>), dim3((total + 3) / 4), dim3(256), 0, stream, *a, nb, total);
    else hipLaunchKernelGGL((ogc_splitk_reduce_kernel<DT, 0>), dim3((total + 3) / 4), dim3(256), 0, stream, *a, nb, total);
    return (int)hipGetLastError();
}

template <int DT, int TILE, int XP, int OP>
static int launch_layer_t(const OgcLayerArgs* a, hipStream_t stream) {
    const OgcTileInfo ti = tile_info_t<TILE>();
    auto kern = ogc_layer_kernel<DT, TILE, XP, OP>;
    static std::atomic<bool> attr_set{false};  // raising the LDS limit is idempotent; two threads at once only repeat it
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)ti.lds_bytes);
        if (e != hipSuccess) return (int)e;
        attr_set.store(true, std::memory_order_release);
    }
    const int nrows = OP ? a->N : a->NB_out * 32;
    const int tiles_n = (nrows + ti.bn - 1) / ti.bn;
    const int tiles_m = (a->M + ti.bm - 1) / ti.bm;
    const int total = tiles_n * tiles_m;
    const int per_xcd = (total + 7) / 8;
    hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(ti.threads), ti.lds_bytes, stream, *a, tiles_n, total, per_xcd);
    return (int)hipGetLastError();
}

template <int DT, int TILE>
static int launch_layer_io(int xp, int op, const OgcLayerArgs* a, hipStream_t s) {
    if (xp) return op ? launch_layer_t<DT, TILE, 1, 1>(a, s) : launch_layer_t<DT, TILE, 1, 0>(a, s);
    return op ? launch_layer_t<DT, TILE, 0, 1>(a, s) : launch_layer_t<DT, TILE, 0, 0>(a, s);
}

template <int DT>
static int launch_layer_tile(int tile, int xp, int op, const OgcLayerArgs* a, hipStream_t s) {
    switch (tile) {
    case OGC_TILE_BIG: return launch_layer_io<DT, OGC_TILE_BIG>(xp, op, a, s);
    case OGC_TILE_MID: return launch_layer_io<DT, OGC_TILE_MID>(xp, op, a, s);
    default: return launch_layer_io<DT, OGC_TILE_SMALL>(xp, op, a, s);
    }
}

template <int DT, int SHAPE, int XP, int OP, int EPI>
static int launch_dma_t(const OgcLayerArgs* a, hipStream_t stream) {
    typedef StreamCfg<SHAPE> C;
    auto kern = ogc_layer_dma_kernel<DT, SHAPE, XP, OP, EPI>;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
        if (e != hipSuccess) return (int)e;
        attr_set.store(true, std::memory_order_release);
    }
    // (a split-K launch always writes partials; NB_out == 0 marks the chain's last layer, whose width is N)
    const int nrows = (OP || (EPI == 2 && a->NB_out == 0)) ? a->N : a->NB_out * 32;
    const int tiles_n = ((nrows + C::BN - 1) / C::BN) << (EPI == 2 ? a->ksplit_log2 : 0);  // x k ranges when split
    const int tiles_m = (a->M + C::BM - 1) / C::BM;
    const int total = tiles_n * tiles_m;
    const int per_xcd = (total + 7) / 8;
    const int max_slots = SHAPE ? 32 : 64;  // 32 CUs per XCD, two resident workgroups per CU for the four-wave shape
    const int slots = per_xcd < max_slots ? per_xcd : max_slots;
    hipLaunchKernelGGL(kern, dim3(slots * 8), dim3(C::NT), C::LDS, stream, *a, tiles_n, total, per_xcd, slots);
    return (int)hipGetLastError();
}

template <int DT, int SHAPE, int EPI>
static int launch_dma_io(int xp, int op, const OgcLayerArgs* a, hipStream_t s) {
    if (xp) return op ? launch_dma_t<DT, SHAPE, 1, 1, EPI>(a, s) : launch_dma_t<DT, SHAPE, 1, 0, EPI>(a, s);
    return op ? launch_dma_t<DT, SHAPE, 0, 1, EPI>(a, s) : launch_dma_t<DT, SHAPE, 0, 0, EPI>(a, s);
}

// EPI = 1: quantized layer with ReLU and a requantized result (that epilogue only); 2: split-K partials, followed by the
// reduction pass that owns the epilogue; 3 / 4 (not the k-sliced shape, whose reduction across the k groups needs the
// registers): quantized layer without activation / with GELU and a requantized result; 0: everything else, activation and result type looked up at run time.  One epilogue per kernel
// is not a matter of a few branches: with all of them in one kernel the compiler runs out of the 80 registers it is left
// with and spills, and a reload from scratch memory in the code between the assembly blocks makes it wait for EVERY
// outstanding vector-memory operation, the ring's direct loads included (measured: 45 instead of 34 us per launch).
static int stream_epi(const OgcLayerArgs* a, bool k_sliced) {
    if (a->out_f32) return 0;
    if (a->act == OGC_ACT_RELU) return 1;
    if (!k_sliced && a->act == OGC_ACT_NONE) return 3;
    if (!k_sliced && a->act == OGC_ACT_GELU_TANH) return 4;
    return 0;
}
template <int DT, int SHAPE>
static int launch_dma_quant(int xp, int op, const OgcLayerArgs* a, hipStream_t s) {
    const int epi = stream_epi(a, SHAPE == 2);
    if (epi == 1) return launch_dma_io<DT, SHAPE, 1>(xp, op, a, s);
    if constexpr (SHAPE != 2) {
        if (epi == 3) return launch_dma_io<DT, SHAPE, 3>(xp, op, a, s);
        if (epi == 4) return launch_dma_io<DT, SHAPE, 4>(xp, op, a, s);
    }
    return launch_dma_io<DT, SHAPE, 0>(xp, op, a, s);
}
template <int SHAPE>
static int launch_dma_dtype(int dtype, int xp, int op, const OgcLayerArgs* a, hipStream_t s) {
    if constexpr (SHAPE == 2) {
        if (a->ksplit_log2 > 0) return (int)hipErrorInvalidValue;  // the plan never splits this shape between workgroups
        if (dtype == OGC_BF16) return launch_dma_io<OGC_BF16, 2, 0>(xp, op, a, s);
        if (dtype == OGC_I8) return launch_dma_quant<OGC_I8, 2>(xp, op, a, s);
        return (int)hipErrorInvalidValue;
    } else
    if (a->ksplit_log2 > 0) {
        int rc;
        if (dtype == OGC_BF16) rc = xp ? launch_dma_t<OGC_BF16, SHAPE, 1, 0, 2>(a, s) : launch_dma_t<OGC_BF16, SHAPE, 0, 0, 2>(a, s);
        else if (dtype == OGC_I8) rc = xp ? launch_dma_t<OGC_I8, SHAPE, 1, 0, 2>(a, s) : launch_dma_t<OGC_I8, SHAPE, 0, 0, 2>(a, s);
        else return (int)hipErrorInvalidValue;
        if (rc != 0) return rc;
        return dtype == OGC_BF16 ? launch_splitk_reduce<OGC_BF16>(op, a, s) : launch_splitk_reduce<OGC_I8>(op, a, s);
    }
    if (dtype == OGC_BF16) return launch_dma_io<OGC_BF16, SHAPE, 0>(xp, op, a, s);
    if (dtype == OGC_I8) return launch_dma_quant<OGC_I8, SHAPE>(xp, op, a, s);
    if constexpr (SHAPE == 1) {
        if (dtype == OGC_F8) return launch_dma_quant<OGC_F8, 1>(xp, op, a, s);  // E4M3: the eight-wave shape only
    }
    return (int)hipErrorInvalidValue;  // the plan never selects this kernel for fp32
}

extern "C" int ogc_launch_layer(int dtype, int tile, int x_plain, int out_plain, const OgcLayerArgs* a, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    if (tile == OGC_TILE_DMA || tile == OGC_TILE_DMA8 || tile == OGC_TILE_DMAK2) {
        if (x_plain && !a->x_vec_ok) {
            tile = OGC_TILE_MID;  // caller's x is not 16-byte aligned: same channel padding, register-staged loads
        } else {
            if (tile == OGC_TILE_DMA) return launch_dma_dtype<0>(dtype, x_plain, out_plain, a, s);
            if (tile == OGC_TILE_DMAK2) return launch_dma_dtype<2>(dtype, x_plain, out_plain, a, s);
            return launch_dma_dtype<1>(dtype, x_plain, out_plain, a, s);
        }
    }
    switch (dtype) {
    case OGC_F32: return launch_layer_tile<OGC_F32>(tile, x_plain, out_plain, a, s);
    case OGC_BF16: return launch_layer_tile<OGC_BF16>(tile, x_plain, out_plain, a, s);
    case OGC_F8: return launch_layer_tile<OGC_F8>(tile, x_plain, out_plain, a, s);
    default: return launch_layer_tile<OGC_I8>(tile, x_plain, out_plain, a, s);
    }
}

extern "C" size_t ogc_fused_lds_limit(void) { return 160 * 1024; }
extern "C" int ogc_fused_threads(void) { return OGC_FUSED_THREADS; }

template <int DT> static int launch_fused_t(const OgcChainArgs* c, int m_blocks, hipStream_t stream) {
    auto kern = ogc_fused_chain_kernel<DT>;
    const size_t lds = (size_t)2 * c->lds_buf_bytes;
    {   // the limit only ever grows; the lock keeps raising it and remembering it together
        static std::mutex mu;
        static size_t attr_max = 0;
        std::lock_guard<std::mutex> hold(mu);
        if (lds > attr_max) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return (int)e;
            attr_max = lds;
        }
    }
    OgcChainArgs args = *c;
    // Up to 16 row tiles per XCD before the next XCD is used: every XCD that takes part fetches all the weights
    // into its own L2, so a small batch on one XCD asks the fabric for them once instead of eight times
    // (measured 1-4 % faster as well; beyond 16 workgroups on an XCD it turns slower).
    int xcds = 1;
    while (xcds < 8 && m_blocks > 16 * xcds) xcds *= 2;
    args.fused_xcds = xcds;
    args.fused_tiles = m_blocks;
    const int grid = (m_blocks - 1) / xcds * 8 + (m_blocks - 1) % xcds + 1;  // up to the last tile's workgroup
    hipLaunchKernelGGL(kern, dim3(grid), dim3(OGC_FUSED_THREADS), lds, stream, args);
    return (int)hipGetLastError();
}

extern "C" int ogc_launch_fused(int dtype, const OgcChainArgs* c, int m_blocks, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    switch (dtype) {
    case OGC_F32: return launch_fused_t<OGC_F32>(c, m_blocks, s);
    case OGC_BF16: return launch_fused_t<OGC_BF16>(c, m_blocks, s);
    case OGC_F8: return launch_fused_t<OGC_F8>(c, m_blocks, s);
    default: return launch_fused_t<OGC_I8>(c, m_blocks, s);
    }
}

template <int DT> static int launch_coop_t(const OgcChainArgs* c, int m_blocks, int grid, void* sync, hipStream_t stream) {
    hipLaunchKernelGGL((ogc_coop_chain_kernel<DT>), dim3(grid), dim3(OGC_COOP_THREADS), 0, stream, *c, (unsigned long long*)sync, m_blocks);
    return (int)hipGetLastError();
}

// grid: workgroups to launch (at most one per CU, at most the largest number of 32x32 blocks of any layer)
extern "C" int ogc_launch_coop(int dtype, const OgcChainArgs* c, int m_blocks, int grid, void* sync, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    switch (dtype) {
    case OGC_F32: return launch_coop_t<OGC_F32>(c, m_blocks, grid, sync, s);
    case OGC_BF16: return launch_coop_t<OGC_BF16>(c, m_blocks, grid, sync, s);
    case OGC_F8: return launch_coop_t<OGC_F8>(c, m_blocks, grid, sync, s);
    default: return launch_coop_t<OGC_I8>(c, m_blocks, grid, sync, s);
    }
}

__global__ void ogc_zero_words_kernel(unsigned long long* w, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) w[i] = 0;
}
extern "C" int ogc_launch_zero_words(void* words, int n, void* stream) {
    hipLaunchKernelGGL(ogc_zero_words_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (unsigned long long*)words, n);
    return (int)hipGetLastError();
}

extern "C" int ogc_launch_zero_sync(void* sync, void* stream) {
    hipLaunchKernelGGL(ogc_zero_sync_kernel, dim3(1), dim3(512), 0, (hipStream_t)stream, (unsigned long long*)sync);
    return (int)hipGetLastError();
}

// XCDs a packed cluster launch uses: the fewest (a power of two) that keep at most 16 workgroups on each; -1 if
// the tiles do not fit one workgroup per CU.  A spread launch (consecutive workgroups, hence different XCDs, for the
// members of a tile) fits if there is a CU for every workgroup.
extern "C" int ogc_cluster_xcds(int m_blocks, int split, int spread) {
    if (split < 1 || m_blocks < 1 || m_blocks * OGC_SYNC_STRIDE > OGC_SYNC_WORDS) return -1;
    if (spread) return (long)m_blocks * split <= 256 ? 0 : -1;
    for (int xcds = 1; xcds <= 8; xcds *= 2) {
        const int per_xcd = (m_blocks + xcds - 1) / xcds * split;
        if (per_xcd <= 16 || (xcds == 8 && per_xcd <= 32)) return xcds;
    }
    return -1;
}

template <int DT, int KSPLIT> static int launch_cluster_t(const OgcChainArgs* c, int m_blocks, int split, int spread, int cus, void* sync, hipStream_t stream) {
    auto kern = KSPLIT ? ogc_cluster_ksplit_chain_kernel<DT> : ogc_cluster_chain_kernel<DT>;
    const size_t lds = KSPLIT ? (size_t)c->lds_buf_bytes + OGC_KS_RED_BYTES : (size_t)2 * c->lds_buf_bytes;
    {   // the limit only ever grows; the lock keeps raising it and remembering it together
        static std::mutex mu;
        static size_t attr_max = 0;
        std::lock_guard<std::mutex> hold(mu);
        if (lds > attr_max) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return (int)e;
            attr_max = lds;
        }
    }
    const int xcds = ogc_cluster_xcds(m_blocks, split, spread);
    // every member waits for the others of its tile: all of them need a CU at once (the plan assumed 256 CUs)
    if (xcds < 0 || (long)m_blocks * split > cus) return (int)hipErrorInvalidValue;
    OgcChainArgs args = *c;
    args.fused_xcds = xcds;  // 0: spread
    args.fused_tiles = m_blocks;
    args.cluster_split = split;
    const int grid = spread ? m_blocks * split : (m_blocks + xcds - 1) / xcds * split * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(OGC_FUSED_THREADS), lds, stream, args, (unsigned long long*)sync);
    return (int)hipGetLastError();
}

extern "C" size_t ogc_cluster_ksplit_lds_bytes(size_t lds_buf_bytes) { return lds_buf_bytes + OGC_KS_RED_BYTES; }

// ksplit: the kernel whose waves split K inside a member (one LDS buffer + reduction scratch) instead of the one
// whose waves take different channel blocks (two LDS buffers)
// cus: compute units of the device (every member of every tile needs one at the same time)
extern "C" int ogc_launch_cluster(int dtype, int ksplit, const OgcChainArgs* c, int m_blocks, int split, int spread, int cus,
                                  void* sync, void* stream) {
    hipStream_t s = (hipStream_t)stream;
    if (ksplit) {
        switch (dtype) {
        case OGC_F32: return launch_cluster_t<OGC_F32, 1>(c, m_blocks, split, spread, cus, sync, s);
        case OGC_BF16: return launch_cluster_t<OGC_BF16, 1>(c, m_blocks, split, spread, cus, sync, s);
        case OGC_F8: return launch_cluster_t<OGC_F8, 1>(c, m_blocks, split, spread, cus, sync, s);
        default: return launch_cluster_t<OGC_I8, 1>(c, m_blocks, split, spread, cus, sync, s);
        }
    }
    switch (dtype) {
    case OGC_F32: return launch_cluster_t<OGC_F32, 0>(c, m_blocks, split, spread, cus, sync, s);
    case OGC_BF16: return launch_cluster_t<OGC_BF16, 0>(c, m_blocks, split, spread, cus, sync, s);
    case OGC_F8: return launch_cluster_t<OGC_F8, 0>(c, m_blocks, split, spread, cus, sync, s);
    default: return launch_cluster_t<OGC_I8, 0>(c, m_blocks, split, spread, cus, sync, s);
    }
}

// ------------------------------------------------------------------------------------------------
// Workspace for callers that cannot allocate (ogc_mlp_run_static): a fixed array in the library's device image, one
// copy per GPU, held until the process ends.  In host code the array's name is only a stand-in: the device address
// comes from hipGetSymbolAddress, asked once per device with that device current, and only that address is ever
// handed to kernels.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[OGC_STATIC_SCRATCH_BYTES];

extern "C" int ogc_static_scratch(void** ptr) {
    enum { MAX_DEVICES = 64 };
    static std::mutex mu;
    static void* addr[MAX_DEVICES];  // zero-initialised: not asked yet
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= MAX_DEVICES) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p || ((uintptr_t)p & 255) != 0) return (int)hipErrorInvalidSymbol;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return 0;
}

extern "C" int ogc_device_cu_count(void) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return n;
}

static const char* chain_kernel_name(const char* const (&names)[4], int dtype) { return (dtype >= 0 && dtype < 4) ? names[dtype] : "?"; }
extern "C" const char* ogc_coop_kernel_name(int dtype) {
    static const char* const names[4] = {"ogc_coop_chain_kernel<0>", "ogc_coop_chain_kernel<1>", "ogc_coop_chain_kernel<2>", "ogc_coop_chain_kernel<3>"};
    return chain_kernel_name(names, dtype);
}
extern "C" const char* ogc_cluster_kernel_name(int dtype, int ksplit) {
    static const char* const ks[4] = {"ogc_cluster_ksplit_chain_kernel<0>", "ogc_cluster_ksplit_chain_kernel<1>",
                                      "ogc_cluster_ksplit_chain_kernel<2>", "ogc_cluster_ksplit_chain_kernel<3>"};
    static const char* const plain[4] = {"ogc_cluster_chain_kernel<0>", "ogc_cluster_chain_kernel<1>", "ogc_cluster_chain_kernel<2>",
                                         "ogc_cluster_chain_kernel<3>"};
    return ksplit ? chain_kernel_name(ks, dtype) : chain_kernel_name(plain, dtype);
}

extern "C" int ogc_launch_prepack_weights(const void* w, void* out, int K, int N, int KC, int NPw, int esz, void* stream) {
    const long long total = (long long)(NPw >> 5) * KC * 32;
    const int threads = 256;
    const long long blocks = (total + threads - 1) / threads;
    hipLaunchKernelGGL(ogc_prepack_weights_kernel, dim3((unsigned)blocks), dim3(threads), 0, (hipStream_t)stream,
                       (const uint8_t*)w, (uint8_t*)out, K, N, KC, NPw, esz);
    return (int)hipGetLastError();
}

extern "C" int ogc_launch_prepack_params(int dtype, const void* w, const float* w_scale, const float* bias, float in_scale,
                                         int in_zp, int K, int N, int NPw, float* scale_out, float* bias_out,
                                         int32_t* ncomp_out, void* stream) {
    hipLaunchKernelGGL(ogc_prepack_params_kernel, dim3((NPw + 63) / 64), dim3(64 * OGC_PARAMS_SLICES), 0, (hipStream_t)stream,
                       dtype, (const int8_t*)w, w_scale, bias, in_scale, in_zp, K, N, NPw, scale_out, bias_out, ncomp_out);
    return (int)hipGetLastError();
}

// Kernel names with their template arguments, spelled the way a kernel trace prints them.
extern "C" const char* ogc_layer_kernel_name(int dtype, int tile, int x_plain, int out_plain, int act, int out_f32, int split) {
    static char names[4][OGC_NUM_TILES][2][2][5][48];
    if (dtype < 0 || dtype > 3 || tile < 0 || tile >= OGC_NUM_TILES) return "?";
    const bool stream = tile == OGC_TILE_DMA || tile == OGC_TILE_DMA8 || tile == OGC_TILE_DMAK2;
    int epi = 0;
    if (stream && split) {
        epi = 2;
    } else if (stream && (dtype == OGC_I8 || dtype == OGC_F8)) {
        OgcLayerArgs probe;
        memset(&probe, 0, sizeof probe);
        probe.act = act, probe.out_f32 = out_f32;
        epi = stream_epi(&probe, tile == OGC_TILE_DMAK2);
    }
    if (epi == 2) out_plain = 0;
    char* n = names[dtype][tile][x_plain != 0][out_plain != 0][epi];
    if (!n[0]) {
        char tmp[48];
        if (stream)
            snprintf(tmp, sizeof tmp, "ogc_layer_dma_kernel<%d, %d, %d, %d, %d>", dtype,
                     tile == OGC_TILE_DMA8 ? 1 : (tile == OGC_TILE_DMAK2 ? 2 : 0), x_plain != 0, out_plain != 0, epi);
        else
            snprintf(tmp, sizeof tmp, "ogc_layer_kernel<%d, %d, %d, %d>", dtype, tile, x_plain != 0, out_plain != 0);
        memcpy(n, tmp, sizeof tmp);  // every writer stores the same bytes
    }
    return n;
}
extern "C" const char* ogc_fused_kernel_name(int dtype) {
    static const char* const names[4] = {"ogc_fused_chain_kernel<0>", "ogc_fused_chain_kernel<1>", "ogc_fused_chain_kernel<2>", "ogc_fused_chain_kernel<3>"};
    return chain_kernel_name(names, dtype);
}
