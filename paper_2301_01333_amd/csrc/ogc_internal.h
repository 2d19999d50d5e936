// Internal declarations shared by the host-side plan code and the gfx950 kernels.
// Not part of the public ABI (that is include/ogc_mlp.h).
#ifndef OGC_INTERNAL_H
#define OGC_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#include "ogc_mlp.h"

// ------------------------------------------------------------------------------------------------
// Blocked operand layout ("KB16"), used for packed weights and for intermediate activations.
//
// A matrix with R rows (weights: output channel n; activations: batch row m) and a reduction axis of
// KPB bytes per row (K elements zero-padded so that KPB is a multiple of 64) is stored as
//     [R/32][KPB/16][32 rows][16 bytes]
// i.e. byte (r, kb) lives at ((r/32)*(KPB/16) + kb/16)*512 + (r%32)*16 + kb%16.
// Two consecutive 512-byte slabs are exactly one 32x32-MFMA operand in register order: lane l of a
// wavefront owns the 16 bytes at l*16 (row l%32, k-half l/32), for v_mfma_i32_32x32x32_i8,
// v_mfma_f32_32x32x16_bf16 and four v_mfma_f32_32x32x2_f32 steps alike.  This is the GPU analogue of
// the paper's blocked layout A[M/MB, K/KB, MB, KB] (Section III) with MB=32, KB=16 bytes.
// u8 activations are held internally as s8 with 128 subtracted (x ^ 0x80), which is what the signed
// int8 MFMA consumes; the constant 128 is folded into the zero-point compensation.
// ------------------------------------------------------------------------------------------------

#define OGC_MAX_LAYERS 16

struct OgcLayerArgs {
    const uint8_t* w;      // packed weights, KB16 layout, rows = padded N, zero padded
    const float* scale;    // I8: in_scale*w_scale[n] (0 in the padding); unused otherwise
    const float* bias;     // fp32, padded with zeros; all zeros when the layer has no bias
    const int32_t* ncomp;  // I8: -(in_zp-128)*sum_k w_q[k,n]; read only if has_comp
    const uint8_t* x;      // input: plain row-major (first layer) or KB16 workspace buffer
    uint8_t* y;            // output: KB16 workspace buffer, or the caller's plain y (last layer)
    const uint8_t* res;    // plain x0 for the residual add, or NULL
    long long ldx_bytes, ldy_bytes, ldres_bytes;  // plain row strides in bytes
    int32_t M, K, N;       // logical sizes of this layer
    int32_t KC;            // 16-byte chunks per padded input row (KPB/16), a multiple of 4
    int32_t KC_out;        // KB16 output: chunks per row of the next layer's input
    int32_t NB_out;        // KB16 output: number of 32-channel blocks to write
    int32_t act;           // ogc_act
    int32_t has_comp;      // I8: in_zp != 128
    int32_t out_f32;       // I8 last layer: store fp32
    int32_t x_vec_ok;      // plain x: base and stride 16-byte aligned and K*elt a multiple of 16
    int32_t y_vec_ok;      // plain y: base and stride 16-byte aligned
    int32_t res_vec_ok;
    float inv_cs;          // I8: 1.0f/out_scale
    float zp_out;          // I8: (float)out_zp
    int32_t has_bias;
    float q_hi;            // I8: 255 - out_zp
    uint32_t q_add, q_xor; // I8: packed-byte zero-point add and u8 -> internal s8 flip for four results at once
    // Split-K (stream kernel only): the reduction axis is cut into 1 << ksplit_log2 equal ranges, each computed by
    // its own workgroup, which writes its raw accumulators to `partial`; a second kernel adds the ranges in a
    // fixed order and applies the epilogue.  Partial layout: [range][M block of 32][N block of 32][4][64 lanes]
    // x 16 bytes, i.e. each wave stores its accumulator registers as they are.
    int32_t ksplit_log2;
    uint8_t* partial;
    int32_t pmb, pnb;      // 32-row / 32-channel blocks per range in `partial`
    // Stream kernel, diagnostic runs only (NULL otherwise): every workgroup's first thread stores the 100 MHz wall clock and
    // the shader cycle counter at its start and at its end, four 64-bit words per workgroup (ogc_mlp_run_clocked)
    long long* clocks;
};

struct OgcChainArgs {
    int32_t n_layers;
    int32_t lds_buf_bytes;  // size of one LDS activation buffer
    int32_t fused_xcds;     // fused and cluster kernels: row tiles are dealt to this many of the 8 XCDs (workgroup b runs on
                            // XCD b%8); cluster kernel, 0: a tile's members are consecutive workgroups instead
    int32_t fused_tiles;    // fused and cluster kernels: number of 32-row tiles
    int32_t cluster_split;  // cluster kernel: workgroups that share a row tile
    uint32_t cluster_whole_mask;  // cluster kernel: bit l set = every member computes the whole of layer l (no exchange)
    uint32_t cluster_tile_stride; // cluster kernels: bytes between the exchange regions of two row tiles inside a workspace
                                  // slot (the widest exchanged row block: the same for every layer, so that the regions
                                  // of different tiles never overlap whichever layers the tiles are at)
    int32_t barrier_budget;       // cooperative and cluster kernels: polls before a barrier wait gives up
    int32_t barrier_extra;        // added to every barrier's target; 0 except in the test of the give-up path
    OgcLayerArgs layer[OGC_MAX_LAYERS];
};

#define OGC_CLOCK_WORDS_PER_LAUNCH 2048  // ogc_mlp_run_clocked: 64-bit words per launch (at most 512 workgroups x 4)
#define OGC_STATIC_SCRATCH_BYTES (8u << 20)  // the library's own workspace for ogc_mlp_run_static, per GPU

#define OGC_SYNC_STRIDE 16    // 64-bit words between the counters of two row tiles: a 128-byte line each
#define OGC_SYNC_WORDS 2048   // 64-bit words at the end of the packed blob (cooperative and cluster kernels)
#define OGC_SYNC_ERR_WORD 2   // set to 1 by a workgroup whose barrier wait gave up; read and cleared by ogc_mlp_check
#define OGC_BARRIER_BUDGET (1 << 22)

enum { OGC_TILE_BIG = 0, OGC_TILE_MID = 1, OGC_TILE_SMALL = 2, OGC_TILE_DMA = 3, OGC_TILE_DMA8 = 4, OGC_TILE_DMAK2 = 5, OGC_NUM_TILES = 6 };

struct OgcTileInfo {
    int bn, bm, threads;
    size_t lds_bytes;
};

#ifdef __cplusplus
extern "C" {
#endif
// Launchers implemented next to the kernels.  All return a hipError_t value cast to int.
OgcTileInfo ogc_tile_info(int tile);
int ogc_launch_layer(int dtype, int tile, int x_plain, int out_plain, const OgcLayerArgs* a, void* stream);
int ogc_launch_fused(int dtype, const OgcChainArgs* c, int m_blocks, void* stream);
int ogc_launch_coop(int dtype, const OgcChainArgs* c, int m_blocks, int grid, void* sync, void* stream);
int ogc_launch_zero_sync(void* sync, void* stream);
int ogc_launch_zero_words(void* words, int n, void* stream);
int ogc_cluster_xcds(int m_blocks, int split, int spread);
int ogc_launch_cluster(int dtype, int ksplit, const OgcChainArgs* c, int m_blocks, int split, int spread, int cus, void* sync,
                       void* stream);
size_t ogc_cluster_ksplit_lds_bytes(size_t lds_buf_bytes);
int ogc_device_cu_count(void);
int ogc_static_scratch(void** ptr);  // device address of the static workspace on the current device (asked once per device)
const char* ogc_coop_kernel_name(int dtype);
const char* ogc_cluster_kernel_name(int dtype, int ksplit);
int ogc_launch_prepack_weights(const void* w, void* out, int K, int N, int KC, int NPw, int esz, void* stream);
int ogc_launch_prepack_params(int dtype, const void* w, const float* w_scale, const float* bias, float in_scale, int in_zp,
                              int K, int N, int NPw, float* scale_out, float* bias_out, int32_t* ncomp_out, void* stream);
int ogc_launch_quantize_e4m3(const float* x, uint8_t* out, size_t n, float inv_scale, void* stream);
int ogc_launch_dequantize_e4m3(const uint8_t* x, float* out, size_t n, float scale, void* stream);
const char* ogc_layer_kernel_name(int dtype, int tile, int x_plain, int out_plain, int act, int out_f32, int split);
const char* ogc_fused_kernel_name(int dtype);
size_t ogc_fused_lds_limit(void);
int ogc_fused_threads(void);
#ifdef __cplusplus
}
#endif

#endif
