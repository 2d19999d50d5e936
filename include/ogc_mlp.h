/*
 * ogc_mlp.h — C ABI of the MI355X (gfx950) fused-MLP library.
 *
 * The library runs a chain of MatMul + bias + activation layers ("MLP subgraph", arxiv 2301.01333
 * Section VII) as fused GPU kernels: for layer l = 0..L-1, Y_l[M,N_l] = post_ops(X_l[M,K_l] W_l[K_l,N_l])
 * with X_{l+1} = Y_l.  fp32, bf16 and int8 (u8 activations x s8 per-output-channel weights, int32
 * accumulation, dequantize / requantize as fused post-ops) are supported.
 *
 * Conventions common to every entry point
 *   - All shapes, dtypes, activations and quantization parameters are static: fixed when the plan is
 *     made (the paper specialises for static shapes and folds quantization constants, Sections I, V).
 *   - Tensors at the boundary are plain row-major (as in the evaluation set-up of Section VII, where the
 *     graph's inputs and outputs keep the plain layout) unless the description asks for the blocked layout (ogc_layout), which lets chains hand
 *     activations to each other the way the layers of one chain do.  Weights are [K,N] row-major (B[K,N] of
 *     Section III).  Otherwise blocked layouts exist only inside the packed blob and the workspace.
 *   - "dev" pointers are device (HBM) addresses on the current HIP device; "host" pointers are ordinary
 *     process memory.  The library never allocates, frees or retains device memory: x, y, raw weights,
 *     packed and workspace are owned by the caller.  The plan is host memory owned by the library until
 *     ogc_mlp_destroy.
 *   - ogc_mlp_prepack_weights and ogc_mlp_run only enqueue work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and return without synchronising.
 *   - Errors are return codes; nothing throws or aborts across this boundary.  Every argument check
 *     happens before the first launch, so a call that returns an argument error has touched nothing.
 *   - A plan may be used from several host threads; concurrent ogc_mlp_run calls on different streams
 *     need distinct workspace buffers.
 */
#ifndef OGC_MLP_H
#define OGC_MLP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OGC_OK = 0,
    OGC_ERR_INVALID_ARG = -1,   /* NULL where a pointer is required, bad enum value, bad quant parameter */
    OGC_ERR_UNSUPPORTED = -2,   /* legal description the kernels do not cover (see ogc_mlp_plan) */
    OGC_ERR_SHAPE = -3,         /* non-positive or inconsistent dimensions */
    OGC_ERR_ALIGNMENT = -4,     /* packed / workspace pointer not 256-byte aligned, x / y not element aligned */
    OGC_ERR_WORKSPACE = -5,     /* workspace is NULL although ogc_mlp_workspace_bytes() > 0 */
    OGC_ERR_NOT_PREPACKED = -6, /* ogc_mlp_run before any ogc_mlp_prepack_weights on this plan */
    OGC_ERR_DEVICE = -7,        /* the HIP runtime reported an error at launch */
    OGC_ERR_TIMEOUT = -8        /* ogc_mlp_check / ogc_mlp_run_profiled: a barrier wait of the cooperative mode gave up */
} ogc_status;

typedef enum { OGC_F32 = 0, OGC_BF16 = 1, OGC_I8 = 2, OGC_F8 = 3 } ogc_dtype;
/* OGC_I8: u8 activations x s8 weights.  OGC_F8: 8-bit floats in the OCP E4M3 encoding (1 sign, 4 exponent bits with bias 7,
 * 3 mantissa bits, no infinities, S.1111.111 = NaN, largest finite value 448), activations and weights alike. */
typedef enum { OGC_ACT_NONE = 0, OGC_ACT_RELU = 1, OGC_ACT_GELU_TANH = 2, OGC_ACT_SIGMOID = 3 } ogc_act;
typedef enum { OGC_OUT_SAME = 0, OGC_OUT_F32 = 1 } ogc_out_kind;
typedef enum { OGC_MODE_AUTO = 0, OGC_MODE_PER_LAYER = 1, OGC_MODE_FUSED = 2, OGC_MODE_COOP = 3 } ogc_mode;
/* Layout of x / y at the boundary.  OGC_LAYOUT_BLOCKED is the library's operand layout (the blocked layout of
 * Section III, as propagated between the layers of a chain, Section V): with it one chain's y is the next
 * chain's x without the round trip through the plain layout.  A blocked tensor of m rows and c columns holds
 * round_up(m,256) rows of c padded to a multiple of 64 (u8, E4M3) or 32 (bf16, fp32) elements, as
 * [rows/32][row bytes/16][32 rows][16 bytes]; u8 values are stored with 128 subtracted.  Its size is ogc_mlp_blocked_bytes(); only a chain of this library should write it. */
typedef enum { OGC_LAYOUT_PLAIN = 0, OGC_LAYOUT_BLOCKED = 1 } ogc_layout;

/* One layer: [M,k] x [k,n] -> [M,n].
 * Post-ops, in this order (fine-grain fusion of the matmul's successors, Section V):
 *   float dtypes: y = acc + bias[n]; y = act(y); last layer with residual: y += x0[m,n]; round to dtype.
 *   OGC_I8 (low-precision conversion + compensated weight, Section V; scheme of Section VII):
 *       acc2 = sum_k x_q*w_q - in_zp*sum_k w_q   (int32, exact)
 *       y    = fma((float)acc2, in_scale*w_scale[n], bias[n])      (no bias: plain product)
 *       y    = act(y)
 *       out == OGC_OUT_F32: store y as fp32 (last layer only);
 *       else q = clamp(rne(y * (1.0f/out_scale)) + out_zp, 0, 255) stored as u8.
 *   OGC_F8 (the same scheme with E4M3 operands; the format is signed, so there is no zero point and no compensation;
 *   not in the paper, whose low-precision type is int8):
 *       acc  = sum_k x8*w8                     (exact products, added by the matrix unit: fp32 result, but the
 *                                               products of one instruction are aligned to the largest and about
 *                                               13 bits below it are kept)
 *       y    = fma(acc, in_scale*w_scale[n], bias[n]) ; y = act(y)
 *       out == OGC_OUT_F32: store y as fp32 (last layer only);
 *       else the E4M3 code nearest to y * (1.0f/out_scale), ties to the even mantissa, saturating at +-448
 *       (never NaN from overflow; a NaN value stays NaN).
 *   acc therefore agrees with the exact sum to about 2^-12 of the largest product, not to fp32 rounding: a
 *   requantized code differs from an exact-sum reference where that much moves the value across a rounding boundary.
 * For OGC_I8 and OGC_F8 the caller sets in_scale (and in_zp) of layer l+1 equal to out_scale (out_zp) of layer l. */
typedef struct {
    int32_t k, n;          /* > 0; k of layer l+1 must equal n of layer l; OGC_I8: k <= 65536 */
    int32_t has_bias;      /* 0 or 1; bias is fp32[n] for every dtype */
    int32_t act;           /* ogc_act */
    float in_scale;        /* OGC_I8, OGC_F8: a_s > 0, finite.  Ignored otherwise */
    int32_t in_zp;         /* OGC_I8: a_z in [0,255]; OGC_F8: must be 0 */
    float out_scale;       /* OGC_I8, OGC_F8 with OGC_OUT_SAME: c_s > 0, finite */
    int32_t out_zp;        /* OGC_I8 with OGC_OUT_SAME: c_z in [0,255]; OGC_F8: must be 0 */
    int32_t out;           /* ogc_out_kind; OGC_OUT_F32 only for OGC_I8 / OGC_F8 and only on the last layer */
} ogc_layer_desc;

typedef struct {
    int32_t dtype;                 /* ogc_dtype */
    int32_t m;                     /* batch rows, > 0 */
    int32_t n_layers;              /* 1..16 */
    const ogc_layer_desc* layers;  /* host, n_layers entries; copied by ogc_mlp_plan */
    int32_t ld_x, ld_y;            /* row strides of x and y in elements; ld_x >= k0, ld_y >= n_last */
    int32_t residual;              /* 1: last layer adds x (float dtypes only; requires n_last == k0) */
    int32_t mode;                  /* ogc_mode */
    int32_t x_layout, y_layout;    /* ogc_layout.  Blocked: per-layer kernels only (OGC_MODE_FUSED is refused), no
                                      residual with a blocked x, no OGC_OUT_F32 with a blocked y; ld_x / ld_y
                                      are ignored for a blocked tensor */
} ogc_mlp_desc;

typedef struct ogc_mlp_plan_s* ogc_mlp_plan_t;

/* Makes a plan from a static description: validates it, chooses between the fused-chain kernel (one
 * workgroup keeps its batch tile's activations in LDS across all layers: coarse-grain fusion, Section V)
 * and per-layer kernels with workspace buffer reuse (Section VI), picks tile shapes (the role of the
 * template-parameter heuristic, Section III) and lays out the packed blob and the workspace.
 * Host only: no device call is made.  *out_plan is written only on OGC_OK.
 * OGC_MODE_COOP is the small-batch mode: one launch in which several workgroups share the work of a row tile
 * (multi-core loop and k-slicing, Section III) and meet at barriers between layers.  It has three kernels, and the
 * plan takes the one with the lowest estimate: (a) all CUs share each layer's 32x32 output blocks, the waves of a
 * workgroup split the reduction axis, device-wide barrier; (b) the cluster kernel: 2, 4, 8 or 16 workgroups per
 * 32-row tile, each keeps the tile in LDS and streams its share of the weights, the tile's members exchange their
 * channel blocks through the workspace at a barrier of their own (int8 and bf16 chains whose widest row fits LDS
 * twice); (c) its k-split variant: 2 to 32 members per tile take whole channel blocks, the waves of a member split
 * the reduction axis as in (a) but read the activations from the member's LDS copy of the tile (any dtype; the
 * widest row has to fit LDS once).
 * The mode needs the workspace and keeps barrier counters in the packed blob (16 KiB at its end), so runs that
 * share a packed blob must not overlap in time; all its workgroups must be resident at once (the grid is at most
 * one per CU), so it is meant for a device that is not kept busy by other kernels for seconds: the barrier wait
 * is bounded (about 2^22 polls).  A wait that gives up does not hang: the workgroup records the fact in the packed
 * blob's sync area and abandons the rest of the chain, and so do the workgroups that wait for it; y is then invalid.
 * ogc_mlp_run cannot report that (it returns before the kernel runs): call ogc_mlp_check after the run, or use
 * ogc_mlp_run_profiled, which includes the check.  The plan sizes the cluster kernels for the 256 CUs of
 * this part; on a device with fewer CUs than a launch has workgroups ogc_mlp_run returns OGC_ERR_DEVICE.
 * OGC_MODE_AUTO takes the mode with the lowest estimate of the modes' fitted cost models (ogc_mlp_mode_estimates); a
 * single-launch mode wins ties within 7 %.  In per-layer mode each layer's tile and k-split are the candidate with
 * the lowest estimate (ogc_mlp_estimated_us): the scoring heuristic of Section III, no tuning run.
 * OGC_ERR_UNSUPPORTED: OGC_MODE_FUSED requested but a layer is too wide for the LDS activation tile; a blocked
 * x or y with a mode other than per-layer.
 * The plan depends on the description alone (nothing is read from the process environment). */
ogc_status ogc_mlp_plan(const ogc_mlp_desc* desc /*host*/, ogc_mlp_plan_t* out_plan /*host*/);

/* Forced choices for ogc_mlp_plan_with_overrides; -1 in a field leaves that choice to the cost model.  For tests,
 * sweeps and the calibration of the cost models (every candidate of Section III's heuristic can be timed by itself). */
typedef struct {
    int32_t tile;            /* per-layer mode: tile configuration of every layer, 0..5 (0-2 register-staged 256x256 /
                                128x128 / 64x32 channels x rows; 3 / 4 the four- / eight-wave stream tile, 128x256 /
                                256x256; 5 the k-sliced stream tile: 128x128, two groups of four waves take alternate
                                k-steps and add up in LDS at the end of a tile); a stream tile falls back to 1 on a layer
                                the stream kernel cannot run (5 also where the number of 64-byte k-steps is odd;
                                OGC_F8 has stream tile 4 only, 3 and 5 fall back) */
    int32_t ksplit_log2;     /* per-layer mode: log2 of the number of k ranges of every layer on stream tile 3 or 4, 0..3
                                (ignored for OGC_F8) */
    int32_t cluster_split;   /* cooperative mode: 0 = kernel (a); n = kernel (b) with n workgroups per row tile where
                                they fit (any dtype) */
    int32_t cluster_ksplit;  /* cooperative mode: 1 together with cluster_split = n: kernel (c) with n members;
                                0: kernel (c) is never chosen */
    int32_t cluster_whole;   /* kernel (b): 0 = exchange after every layer, also the small ones the model would have
                                every member compute whole */
} ogc_plan_overrides;

/* ogc_mlp_plan with forced choices (overrides may be NULL: identical to ogc_mlp_plan).
 * OGC_ERR_INVALID_ARG also for a field outside its range. */
ogc_status ogc_mlp_plan_with_overrides(const ogc_mlp_desc* desc /*host*/, const ogc_plan_overrides* overrides /*host*/,
                                       ogc_mlp_plan_t* out_plan /*host*/);

/* Size of the packed-weights blob (blocked weights + per-channel parameters of every layer). */
ogc_status ogc_mlp_packed_bytes(ogc_mlp_plan_t plan, size_t* bytes /*host*/);

/* Bytes of the blocked x (which = 0) or y (which = 1) of this plan; 0 if that tensor is plain.  The buffer
 * must be 256-byte aligned. */
ogc_status ogc_mlp_blocked_bytes(ogc_mlp_plan_t plan, int32_t which, size_t* bytes /*host*/);

/* Size of the workspace ogc_mlp_run needs (0 for the fused-chain kernel).  Per-layer mode: the
 * intermediate activations share slots assigned by life span (a chain needs two), followed by the partial
 * accumulators of a layer whose reduction axis the plan splits into ranges (k-slicing, Section III). */
ogc_status ogc_mlp_workspace_bytes(ogc_mlp_plan_t plan, size_t* bytes /*host*/);

/* Which kernel family the plan chose: *mode is OGC_MODE_PER_LAYER, OGC_MODE_FUSED or OGC_MODE_COOP. */
ogc_status ogc_mlp_chosen_mode(ogc_mlp_plan_t plan, int32_t* mode /*host*/);

/* Buffer-reuse result for layer `layer`'s output (Section VI, memory buffer optimisation): *slot is the
 * workspace slot index (-1 = the caller's y, or LDS in fused mode), *offset its byte offset in workspace. */
ogc_status ogc_mlp_buffer_assignment(ogc_mlp_plan_t plan, int32_t layer, int32_t* slot /*host*/, size_t* offset /*host*/);

/* Constant-weight preprocessing (Section V): reorders every layer's plain [k,n] weights into the blocked
 * MFMA operand layout (zero padded) and precomputes everything that depends only on constants: for
 * OGC_I8 the per-channel combined scale in_scale*w_scale[n] and the zero-point compensation from the
 * column sums of w_q; bias is copied (zero padded).  Call once per weight set; raw weights may be
 * released once the stream has passed this call.
 *   w       host array of n_layers dev pointers: fp32 / bf16 / s8 weights, plain [k,n] row-major, contiguous
 *   bias    host array of n_layers dev pointers to fp32[n] (entry may be NULL where has_bias == 0);
 *           the array itself may be NULL if no layer has a bias
 *   w_scale OGC_I8, OGC_F8: host array of n_layers dev pointers to fp32[n] (> 0); otherwise NULL
 *   packed  dev, ogc_mlp_packed_bytes() bytes, 256-byte aligned; fully overwritten */
ogc_status ogc_mlp_prepack_weights(ogc_mlp_plan_t plan, const void* const* w, const float* const* bias,
                                   const float* const* w_scale, void* packed, void* stream);

/* Runs the chain: x[m, k0] (row stride ld_x) -> y[m, n_last] (row stride ld_y), both dev, plain row-major,
 * element type of the plan's dtype (u8 for OGC_I8, E4M3 bytes for OGC_F8; fp32 y if the last layer has OGC_OUT_F32).
 * (A blocked x or y, see ogc_layout, is a buffer of ogc_mlp_blocked_bytes() bytes instead.)
 * x and y must not overlap.  packed is the blob written by ogc_mlp_prepack_weights for this plan;
 * workspace is dev, 256-byte aligned, ogc_mlp_workspace_bytes() bytes (may be NULL when that is 0) and
 * holds no state between calls.  In the cooperative mode a run can come out invalid without an error here
 * (see ogc_mlp_plan and ogc_mlp_check). */
ogc_status ogc_mlp_run(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* workspace, void* stream);

/* ogc_mlp_run for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the workspace is a fixed array inside the library's device image, 8 MiB per GPU
 * (ogc_mlp_static_workspace_limit), held from the library's load until the process ends.  The call allocates nothing
 * and frees nothing; x, y and packed are the caller's as in ogc_mlp_run.  The array's device address is looked up
 * once per device, at the first call made with that device current.
 * OGC_ERR_WORKSPACE: the plan needs more than the limit (ogc_mlp_workspace_bytes); nothing is launched.
 * Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (different streams, or
 * different plans) race on it; the array keeps the last call's contents, which no later call relies on (every
 * intermediate and every split-K partial is written before it is read). */
ogc_status ogc_mlp_run_static(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* stream);

/* The size in bytes of the static workspace behind ogc_mlp_run_static. */
size_t ogc_mlp_static_workspace_limit(void);

/* The quantize and dequantize nodes of the low-precision graph (Section V) for OGC_F8 tensors at the boundary of a
 * chain: out[i] = E4M3(x[i] * (1.0f/scale)), nearest with ties to the even mantissa, saturating at +-448, NaN kept
 * (exactly a layer's requantized output); and out[i] = value(x[i]) * scale.  x, out: device, n elements, contiguous;
 * fp32 pointers 4-byte aligned (OGC_ERR_ALIGNMENT); scale > 0 and finite for quantize, finite for dequantize
 * (OGC_ERR_INVALID_ARG).  n == 0 is a no-op.  Asynchronous on `stream`. */
ogc_status ogc_quantize_e4m3(const float* x /*device*/, uint8_t* out /*device*/, size_t n, float scale, void* stream);
ogc_status ogc_dequantize_e4m3(const uint8_t* x /*device*/, float* out /*device*/, size_t n, float scale, void* stream);

/* Diagnostic run: ogc_mlp_run, with every workgroup of the stream kernel (per-layer mode, tiles 3-5) recording when it
 * ran on two clocks: the 100 MHz wall clock and the shader cycle counter, whose rate is the clock the chip actually gives
 * the kernel (the published peaks assume 2.4 GHz; under matrix-instruction load the power limit sets less).  clocks:
 * device, 8-byte aligned, ogc_mlp_num_launches() x ogc_mlp_clock_words_per_launch() 64-bit words; launch l, workgroup g
 * writes words [l * words_per_launch + 4 g .. + 3] = wall clock at start, cycle counter at start, wall clock at end,
 * cycle counter at end (of the workgroup's first wavefront).  Launches of other kernels and workgroups that do not exist
 * leave their words as they are: clear the buffer first.  The section on measurement (Section VII times whole operations;
 * this says at what clock) is what it serves; `bench.py` reports it.
 * OGC_ERR_INVALID_ARG: NULL clocks; OGC_ERR_ALIGNMENT: clocks not 8-byte aligned; otherwise as ogc_mlp_run. */
ogc_status ogc_mlp_run_clocked(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* workspace, void* stream,
                               int64_t* clocks /*device*/);
size_t ogc_mlp_clock_words_per_launch(void);

/* Number of timed launch steps of one ogc_mlp_run: 1 for the fused-chain kernel, n_layers otherwise (a layer
 * whose reduction axis is split runs two kernels, the k ranges and the pass that adds them, and counts as one). */
ogc_status ogc_mlp_num_launches(ogc_mlp_plan_t plan, int32_t* n /*host*/);

/* ogc_mlp_run with a HIP event recorded on `stream` around every launch; waits for the last one and writes
 * each launch's duration in milliseconds to launch_ms[0 .. ogc_mlp_num_launches()-1] (host).  This is the
 * per-operation measurement of Section VII (layers timed separately while still run back to back as a
 * chain).  Unlike ogc_mlp_run it synchronises with the stream and creates/destroys HIP events, and it ends with
 * ogc_mlp_check (OGC_ERR_TIMEOUT if a barrier wait gave up). */
ogc_status ogc_mlp_run_profiled(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* workspace,
                                void* stream, float* launch_ms /*host*/);

/* Tells whether a barrier wait of the cooperative mode gave up in any run on `packed` since the last check
 * (Section III's multi-core template needs all cores at the barrier; on a shared device they may not all be resident
 * in time).  Waits for `stream`, reads one word of the packed blob's sync area, and, if it is set, clears the sync
 * area and returns OGC_ERR_TIMEOUT: the y of that run is invalid and the run may simply be repeated.  OGC_OK
 * otherwise, and at once for plans in another mode.  packed: dev, the blob this plan's runs used.
 * OGC_ERR_INVALID_ARG: NULL plan or packed.  OGC_ERR_DEVICE: the runtime failed. */
ogc_status ogc_mlp_check(ogc_mlp_plan_t plan, const void* packed, void* stream);

/* Test hook for the give-up path of the cooperative mode's barriers: later runs of this plan poll `budget` times
 * (>= 1; default about 2^22) and wait for `extra_target` arrivals more than will ever come (default 0).  With
 * extra_target = 1 every workgroup gives up at its first barrier after `budget` polls and exits normally, which is
 * what ogc_mlp_check must then report.  Host only. */
ogc_status ogc_mlp_test_barrier(ogc_mlp_plan_t plan, int32_t budget, int32_t extra_target);

/* Cooperative mode, cluster kernels: *members = workgroups per 32-row tile (0: not a cluster kernel), *ksplit = 1 for
 * kernel (c), *whole_mask bit l = layer l is computed whole by every member (no exchange), *tile_stride = bytes
 * between the exchange regions of two row tiles inside a workspace slot.  Together with ogc_mlp_buffer_assignment
 * this is the workspace layout of Section VI's buffer reuse as the cluster kernels use it: every tile owns
 * [slot offset + tile*tile_stride, + row-block bytes of the layer) and consecutive exchanged layers alternate
 * between two slots.  Host only; all pointers host, none NULL. */
ogc_status ogc_mlp_cluster_layout(ogc_mlp_plan_t plan, int32_t* members, int32_t* ksplit, uint32_t* whole_mask,
                                  size_t* tile_stride);

/* Releases the plan (NULL is ignored). */
void ogc_mlp_destroy(ogc_mlp_plan_t plan);

/* Static, NUL-terminated description of a status code. */
const char* ogc_status_string(ogc_status s);

/* The plan's cost-model estimate, in microseconds, of layer `layer`'s launch (both launches of a layer whose
 * reduction axis is split), the figure by which ogc_mlp_plan chose that layer's tile and split (Section III: the
 * heuristic scores candidate template parameters, no tuning run).  *us = -1 when the layer was not chosen by the
 * model: fused / cooperative mode, OGC_F32, a forced tile of a kind the model does not cover.  Host only.
 * OGC_ERR_INVALID_ARG: NULL plan or us, layer out of range. */
ogc_status ogc_mlp_estimated_us(ogc_mlp_plan_t plan, int32_t layer, float* us);

/* The cost models' estimates of the whole chain in microseconds, by which OGC_MODE_AUTO chose the mode:
 * us[0] layer by layer (sum of the layers' estimates), us[1] the fused whole-chain kernel, us[2] the cooperative
 * mode (the lowest of its kernels' estimates); -1 where a mode is not admissible (fused: the widest layer does not fit LDS, or bf16 / fp32 weights
 * beyond 2.5 MB; cooperative: a single layer, blocked tensors at the boundary) or not modelled.  Host only.
 * OGC_ERR_INVALID_ARG: NULL plan or us. */
ogc_status ogc_mlp_mode_estimates(ogc_mlp_plan_t plan, float us[3]);

/* Name, with template arguments as a kernel trace prints them, of the kernel that ogc_mlp_run launches for
 * layer `layer` (fused mode: the same name for every layer; a split layer: its first kernel), for matching
 * profiler output.  Returns NULL on a bad argument. */
const char* ogc_mlp_kernel_name(ogc_mlp_plan_t plan, int32_t layer);

#ifdef __cplusplus
}
#endif
#endif /* OGC_MLP_H */
