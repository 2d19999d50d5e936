/*
 * ogc_mha.h -- C ABI of the fused scaled dot-product attention subgraph for AMD MI355X (gfx950).
 *
 * The operation is the second workload of the oneDNN Graph Compiler paper (arxiv 2301.01333, Section VII,
 * Table I rows MHA-1..4): for every batch entry b and head h, with S tokens and head dimension d,
 *
 *     s[i][j] = sum_c q[i][c] * k[j][c]           batch matmul with the transposed keys
 *     s[i][j] = s[i][j] * scale                   the division by a scalar, as a multiply by its fp32 reciprocal
 *     s[i][j] = s[i][j] + mask[b][j]              addition of a mask (one value per key: a padding mask)
 *     p[i][:] = softmax_j(s[i][:])                decomposed and fused into the first matmul (fine-grain fusion)
 *     o[i][c] = sum_j p[i][j] * v[j][c]           second batch matmul, merged with the first (coarse-grain fusion)
 *
 * all in ONE kernel launch: the S x S scores and weights never leave the compute unit.
 *
 * Softmax forms (Section VII mentions a fast softmax without the max reduction):
 *   OGC_SOFTMAX_STABLE  subtracts the row maximum before exponentiating (a running maximum inside the kernel);
 *   OGC_SOFTMAX_FAST    exponentiates the scores as they are.  Same result wherever exp(s) stays finite in
 *                       fp32 (s < 88); the caller vouches for that.  Masked keys (large negative) are fine.
 *
 * Tensors are DEVICE pointers.  q, k, v, o hold element [b][h][i][c] at
 *     base + b*stride_b + h*stride_h + i*stride_s + c        (strides in elements, c contiguous)
 * so both [batch, seq, heads*d] (what a projection layer leaves: stride_b = S*H*d, stride_h = d, stride_s = H*d)
 * and [batch, heads, seq, d] work without a transpose pass.  Every stride must be a multiple of 16 bytes and
 * every base pointer 16-byte aligned.  mask is fp32 [batch][seq], finite values (use -10000, not -infinity), or
 * NULL.  o has q's dtype.  The library allocates nothing and keeps no state between calls.
 *
 * Arithmetic: OGC_F32 multiplies fp32 operands with fp32 accumulation throughout.  OGC_BF16 multiplies bf16
 * operands with fp32 accumulation; scores, exponentials and row sums are fp32; the softmax weights are rounded
 * to bf16 (nearest even) for the second matmul and o is rounded to bf16 once at the end.  OGC_I8 (Table I lists the
 * MHA rows as Int8 too) has an entry point of its own, ogc_mha_run_i8, because it needs quantization scales.
 *
 * Errors are return codes (ogc_status of ogc_mlp.h); every check happens before the launch.
 */
#ifndef OGC_MHA_H
#define OGC_MHA_H

#include "ogc_mlp.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { OGC_SOFTMAX_STABLE = 0, OGC_SOFTMAX_FAST = 1 } ogc_softmax_kind;

typedef struct ogc_mha_desc {
    int32_t dtype;      /* OGC_F32 or OGC_BF16 */
    int32_t batch;      /* > 0 */
    int32_t heads;      /* > 0; batch*heads <= 65535 */
    int32_t seq;        /* S > 0, any value (ragged tiles are handled inside), <= 65536 */
    int32_t head_dim;   /* d: 32, 64, 96 or 128 */
    int32_t softmax;    /* ogc_softmax_kind */
    float scale;        /* finite; 1/sqrt(d) for the usual attention */
    int64_t q_stride[3]; /* elements: batch, head, token */
    int64_t k_stride[3];
    int64_t v_stride[3];
    int64_t o_stride[3];
    int32_t query_groups; /* 0: the library's choice; 1 or 2: 32-query groups per wavefront, forced (tests, sweeps; 2 needs
                             OGC_BF16 and head_dim <= 64, otherwise 1 is taken) */
} ogc_mha_desc;

/* Checks a description without touching the device.
 * OGC_ERR_INVALID_ARG: NULL, bad enum, non-finite scale.  OGC_ERR_SHAPE: non-positive sizes, limits above.
 * OGC_ERR_UNSUPPORTED: OGC_I8 (see ogc_mha_run_i8), head_dim outside {32,64,96,128}.  OGC_ERR_ALIGNMENT: a stride that is not a
 * multiple of 16 bytes or is negative. */
ogc_status ogc_mha_validate(const ogc_mha_desc* desc);

/* Runs the subgraph: one asynchronous launch on `stream` (a hipStream_t, NULL = the default stream).
 * q, k, v: device, read only.  mask: device fp32 [batch][seq] or NULL.  o: device, written for all
 * batch*heads*seq*head_dim elements; must not overlap the inputs.
 * Returns ogc_mha_validate's codes, OGC_ERR_INVALID_ARG for a NULL tensor, OGC_ERR_ALIGNMENT for a base pointer
 * that is not 16-byte aligned, OGC_ERR_DEVICE if the launch failed. */
ogc_status ogc_mha_run(const ogc_mha_desc* desc, const void* q, const void* k, const void* v, const float* mask, void* o,
                       void* stream);

/* Name of the kernel instantiation ogc_mha_run launches for this description (has_mask: whether the run passes a
 * mask), as a profiler's kernel trace prints it (static storage), or NULL for an invalid description.  A run
 * without a mask whose sequence is a whole number of key blocks (bf16: 64, fp32: 32) and whose scale is
 * positive takes a variant that spends no per-key addend; bf16 with head_dim <= 64 and seq >= 256 takes one in
 * which a wavefront owns 64 queries instead of 32 (the last template argument; desc->query_groups forces either). */
const char* ogc_mha_kernel_name(const ogc_mha_desc* desc, int32_t has_mask);

/* Quantization scales of the Int8 attention: real value = scale * integer, zero point 0 for all four tensors
 * (a batch matmul has no constant operand into which a zero point could be folded, Section V). */
typedef struct ogc_mha_quant {
    float q_scale, k_scale, v_scale, o_scale; /* > 0, finite */
} ogc_mha_quant;

/* Int8 rows of Table I (Section VII; low-precision conversion of Section V).  q, k, v, o: int8, same strides and
 * alignment rules as above (strides in elements = bytes).  Per batch entry, head and query i:
 *     S[j] = sum_c q[i][c] k[j][c]                          int32, exact
 *     s[j] = S[j] * (q_scale*k_scale*scale) + mask[j]       fp32
 *     P[j] = rne(127 * exp(s[j] - max_j s[j]))              softmax numerators quantized to 7 bits unsigned
 *     A[c] = sum_j P[j] v[j][c],  L = sum_j P[j]            int32, exact
 *     o[c] = clamp(rne((float(A[c]) / float(L)) * (v_scale / o_scale)), -128, 127)
 *            (int -> float, IEEE divide, multiply by the fp32 quotient v_scale / o_scale, each rounded to nearest even)
 * Everything after P is exact integer arithmetic and three fp32 operations, reproducible bit for bit; P itself can
 * differ by one step from another implementation's where 127 * exp(..) lies within rounding error of a tie.
 * desc->dtype must be OGC_I8 and desc->softmax OGC_SOFTMAX_STABLE (the numerators are quantized against the row
 * maximum; OGC_SOFTMAX_FAST returns OGC_ERR_UNSUPPORTED).  Other codes as ogc_mha_validate / ogc_mha_run, plus
 * OGC_ERR_INVALID_ARG for a NULL quant or a scale that is not positive and finite.  One asynchronous launch. */
ogc_status ogc_mha_i8_validate(const ogc_mha_desc* desc, const ogc_mha_quant* quant);
ogc_status ogc_mha_run_i8(const ogc_mha_desc* desc, const ogc_mha_quant* quant, const void* q, const void* k, const void* v,
                          const float* mask, void* o, void* stream);
/* Kernel instantiation ogc_mha_run_i8 launches for this description, as a kernel trace prints it, or NULL. */
const char* ogc_mha_i8_kernel_name(const ogc_mha_desc* desc);

#ifdef __cplusplus
}
#endif
#endif
