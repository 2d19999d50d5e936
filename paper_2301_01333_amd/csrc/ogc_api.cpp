// Host side of the fused-MLP library: plan construction (validation, kernel-family and tile choice,
// packed-blob and workspace layout, buffer reuse) and the C ABI declared in include/ogc_mlp.h.
// No device memory is allocated here and no device call is made outside prepack / run.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include <hip/hip_runtime_api.h>

#include "ogc_internal.h"

namespace {

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct LayerPlan {
    ogc_layer_desc d;
    int kp;           // padded K (elements) of this layer's input
    int kc;           // 16-byte chunks per input row
    int npw;          // padded rows of the packed weights
    int nb_out;       // 32-channel blocks written to a KB16 output (0 for the last layer)
    int kc_out;       // chunks per row of the KB16 output
    int tile;         // per-layer mode: tile configuration
    int ksplit_log2;  // stream tiles only: the reduction axis is cut into 1 << ksplit_log2 ranges (0: not split)
    double est_us;    // the cost model's estimate for this layer's launch(es); < 0: not modelled
    size_t w_off, scale_off, bias_off, ncomp_off;  // offsets in the packed blob
    int out_slot;     // workspace slot of the output (-1: caller's y / LDS)
    size_t out_off;   // byte offset of that slot in the workspace
    float inv_cs;
};

}  // namespace

struct ogc_mlp_plan_s {
    ogc_mlp_desc desc;
    std::vector<LayerPlan> layers;
    int esz;
    int mode;  // OGC_MODE_PER_LAYER, OGC_MODE_FUSED or OGC_MODE_COOP
    double mode_us[3];  // the cost models' estimates of the whole chain: per layer, fused, cooperative (< 0: n/a)
    int mp;    // padded batch rows of the workspace buffers
    size_t packed_bytes, workspace_bytes;
    int lds_buf_bytes;  // fused mode
    size_t partial_off, partial_bytes;  // split-K partial accumulators, after the activation slots
    size_t sync_off;                    // cooperative mode: counters at the end of the packed blob
    int cluster_split;                  // cooperative mode: 0 = blocks dealt to all workgroups, n = n workgroups per row tile
    int cluster_spread;                 // cluster kernel: a tile's members on different XCDs (weights beyond one L2)
    int cluster_ksplit;                 // cluster kernel: the waves of a member split K (one LDS buffer) instead of the channel blocks
    uint32_t cluster_whole_mask;        // channel-split cluster kernel: layers every member computes whole (no exchange)
    size_t cluster_tile_stride;         // cluster kernels: bytes between two row tiles' regions inside an exchange slot
    ogc_plan_overrides ov;              // forced choices (-1: the cost model's)
    std::vector<size_t> slot_off, slot_size;
    std::atomic<int> prepacked;
    std::atomic<int> cu_count;          // compute units of the device, asked once at the first cooperative run (0: not yet)
    std::atomic<int> barrier_budget, barrier_extra;  // cooperative barriers: polls before giving up, test-only target offset
};

namespace {

// Memory-buffer reuse across the chain (Section VI): life-span analysis over the topologically ordered
// fused ops; an intermediate buffer is reclaimable once its single consumer has run; among the free
// buffers the most recently used one is taken (its lines are the likeliest to still be in cache).
void assign_buffers(ogc_mlp_plan_s* p) {
    const int L = (int)p->layers.size();
    struct Slot { size_t size; int last_use; int busy_until; };
    std::vector<Slot> slots;
    for (int l = 0; l < L; ++l) p->layers[l].out_slot = -1;
    for (int l = 0; l + 1 < L; ++l) {
        const size_t need = (size_t)p->mp * p->layers[l + 1].kc * 16;
        // tensor l is produced by step l and consumed by step l+1: its buffer is busy through step l+1.
        int best = -1;
        for (int s = 0; s < (int)slots.size(); ++s)
            if (slots[s].busy_until < l && (best < 0 || slots[s].last_use > slots[best].last_use)) best = s;
        if (best < 0) {
            slots.push_back({0, -1, -1});
            best = (int)slots.size() - 1;
        }
        if (slots[best].size < need) slots[best].size = need;
        slots[best].busy_until = l + 1;
        slots[best].last_use = l + 1;
        p->layers[l].out_slot = best;
    }
    size_t off = 0;
    p->slot_off.clear();
    p->slot_size.clear();
    for (auto& s : slots) {
        p->slot_off.push_back(off);
        p->slot_size.push_back(s.size);
        off += round_up(s.size, 256);
    }
    p->workspace_bytes = off;
    for (int l = 0; l + 1 < L; ++l) p->layers[l].out_off = p->slot_off[p->layers[l].out_slot];
}

// ---- Plan-time cost model for a per-layer launch (the role of the template-parameter heuristic of Section III:
// propose a split of the output among the cores for load balance and a tile for kernel efficiency, score, take the
// best; no tuning run).  A candidate is a tile configuration and, for the stream tiles, a cut of the reduction
// axis into 1 << ks ranges (the paper's k-slicing).  Its time in microseconds is modelled as
//
//     W      = tiles * 2^ks workgroups of k = KT >> ks steps (a step is 64 bytes of K per row)
//     lone   = (c + d*k) * (1 + g*min(1, W/CUs))        one workgroup's latency, stretched as the chip fills up
//     stream = l0 + rounds * (a + b*k [+ px if split])   a CU's share of the work at full load,
//              rounds = (ceil(W/CUs) + W/CUs) / 2        (between whole rounds and perfect balance)
//     t      = max(lone, stream) [+ r0 + r2*2^ks + r1*(2^ks + 1)*Mp*Np*4 bytes/1e6 for the pass over the partials]
//
// with the constants fitted (least squares on log time, candidates near the fastest weighted double) to timed launches
// of mid-chain layers on an MI355X: K and N from 256 to 8192, batch 32 to 32768, every tile, splits 1 to 8.  The
// generated table file states the number of launches, the rms error and how far the model's pick is from the fastest
// candidate measured (about 1 % in the geometric mean).  The constants include the launch; activation and bias costs are left out (the same for
// every candidate to first order).
struct TileCost {
    float c, d, a, b, g;
};
struct CostTable {
    TileCost t[OGC_NUM_TILES];  // indexed by tile id; OGC_TILE_BIG is not a candidate
    float r0, r1, r2, px, l0;
};
// kCostI8, kCostBf16, kCostF32 (fp32 runs on the register-staged tiles only, never split): written by
// paper_2301_01333_amd/calibration/fit_layers.py from the measured launches in
// paper_2301_01333_amd/calibration/data/layer_times.csv (a test refits and compares)
#include "ogc_cost_layers.inc"

// m rows x n channels, kt = 64-byte steps of the (padded) reduction axis.
double estimate_layer_us(int dtype, int m, int n, int kt, int tile, int ks) {
    const CostTable& ct = (dtype == OGC_I8 || dtype == OGC_F8) ? kCostI8 : (dtype == OGC_BF16 ? kCostBf16 : kCostF32);
    const TileCost& tc = ct.t[tile];
    const OgcTileInfo ti = ogc_tile_info(tile);
    const double cus = 256.0;
    const double tiles = (double)((m + ti.bm - 1) / ti.bm) * ((n + ti.bn - 1) / ti.bn);
    const double w = tiles * (1 << ks), k = (double)(kt >> ks);
    const double lone = (tc.c + tc.d * k) * (1.0 + tc.g * std::min(1.0, w / cus));
    const double rounds = 0.5 * (std::ceil(w / cus) + w / cus);
    double t = std::max(lone, ct.l0 + rounds * (tc.a + tc.b * k + (ks ? ct.px : 0.0f)));
    if (ks) {
        const double mp = (double)round_up((size_t)m, 256), np = (double)round_up((size_t)n, 256);
        t += ct.r0 + ct.r2 * (1 << ks) + ct.r1 * ((1 << ks) + 1) * mp * np * 4.0 / 1e6;
    }
    return t;
}

// Picks tile and split for one layer.  dma_ok: the stream kernel can run this layer (int8 / bf16, no sigmoid,
// input zero point 128, and a first layer whose plain rows are 16-byte aligned without K padding); other layers
// choose among the register-staged tiles.  forced / forced_split (-1: none) come from ogc_mlp_plan_with_overrides.
void choose_tile_and_split(int dtype, int m, int n, int kt, bool dma_ok, int forced, int forced_split, int* tile_out, int* ks_out,
                           double* us_out) {
    auto tiles = [&](int t) {
        const OgcTileInfo ti = ogc_tile_info(t);
        return (long)((m + ti.bm - 1) / ti.bm) * ((n + ti.bn - 1) / ti.bn);
    };
    auto split_ok = [&](int ks) { return ks >= 0 && ks <= 3 && kt % (1 << ks) == 0 && (kt >> ks) >= 4; };
    int tile = -1, ks = 0;
    const bool f8 = dtype == OGC_F8;  // E4M3: of the stream shapes only the eight-wave one, never split along K
    if (forced >= 0 && forced < OGC_NUM_TILES)
        tile = ((forced == OGC_TILE_DMA || forced == OGC_TILE_DMA8 || forced == OGC_TILE_DMAK2) && !dma_ok) ? OGC_TILE_MID : forced;
    if (f8 && (tile == OGC_TILE_DMA || tile == OGC_TILE_DMAK2)) tile = OGC_TILE_MID;
    if (tile == OGC_TILE_DMAK2 && kt % 2 != 0) tile = OGC_TILE_MID;  // its stages hold two k-steps
    const bool stream = tile == OGC_TILE_DMA || tile == OGC_TILE_DMA8;  // (the k-sliced shape is never split between workgroups)
    if (tile >= 0) {
        if (stream && !f8 && forced_split > 0 && forced_split <= 3 && kt % (1 << forced_split) == 0) ks = forced_split;
    } else {
        double best = 0.0;
        // the 256x256 register-staged tile is timed for fp32 only; the stream tiles replace it for int8 / bf16
        const int cands[6] = {OGC_TILE_SMALL, OGC_TILE_MID, dtype == OGC_F32 ? OGC_TILE_BIG : -1, (dma_ok && !f8) ? OGC_TILE_DMA : -1,
                              dma_ok ? OGC_TILE_DMA8 : -1, (dma_ok && !f8 && kt % 2 == 0) ? OGC_TILE_DMAK2 : -1};
        for (int c = 0; c < 6; ++c) {
            if (cands[c] < 0) continue;
            const bool st = (cands[c] == OGC_TILE_DMA || cands[c] == OGC_TILE_DMA8) && !f8;
            if (forced_split > 0 && !st && dma_ok) continue;  // a forced split needs a stream tile
            for (int s = 0; s <= (st ? 3 : 0); ++s) {
                if (forced_split >= 0 && st && s != forced_split) continue;
                if (s > 0 && !(forced_split > 0 ? kt % (1 << s) == 0 : split_ok(s))) continue;
                const double us = estimate_layer_us(dtype, m, n, kt, cands[c], s);
                if (tile < 0 || us < best) best = us, tile = cands[c], ks = s;
            }
        }
    }
    if (tile < 0) tile = tiles(OGC_TILE_MID) >= 128 ? OGC_TILE_MID : OGC_TILE_SMALL;  // nothing admissible was forced
    *tile_out = tile;
    *ks_out = ks;
    const bool timed = dtype == OGC_F32 ? (tile <= OGC_TILE_SMALL) : (tile != OGC_TILE_BIG);
    *us_out = timed ? estimate_layer_us(dtype, m, n, kt, tile, ks) : -1.0;
}

// ---- Whole-chain models of the other two modes, fitted to 357 timed chains (12 shapes, batch 32..16384, three
// dtypes; 2-10 % rms).  A chain run layer by layer costs the sum of its layers' estimates less the event overhead
// each of those carries from the way it was timed.
constexpr double kProfiledLaunchExtraUs = 2.0;
// The E4M3 path has no constants of its own: it moves the same bytes as int8 through the same kernels, and the chains
// these models decide between are bound by weight streaming and launch latency, so it borrows the int8 constants.
inline int model_dtype(int dtype) { return dtype == OGC_F8 ? OGC_I8 : dtype; }
struct FusedCost { float f0, per_mb, per_layer, fill, per_block; };
struct CoopCost { float c0, barrier, block, step, fill; };
struct ClusterCost { float c0, per_mb, group, per_layer, barrier, copy_mb, fill, all_mb; };
struct KsplitCost { float c0, block, step, barrier, copy_mb, fill, all_mb; };
// kFused, kCoop, kCluster, kKsplit: written by paper_2301_01333_amd/calibration/fit_chains.py from the chains timed in
// paper_2301_01333_amd/calibration/data/chain_times.csv (a test refits and compares)
#include "ogc_cost_chains.inc"

// One workgroup per 32 rows streams every weight: flat in the batch up to 8192 rows (256 CUs), then in rounds.
double estimate_fused_us(const ogc_mlp_plan_s* p) {
    const FusedCost& c = kFused[model_dtype(p->desc.dtype)];
    const double m = p->desc.m, rounds = std::max(1.0, m / 8192.0);
    double sum = 0.0;
    for (const LayerPlan& lp : p->layers) {
        // a wave takes every eighth 32-channel block: per_block is what a block costs besides its weight stream
        // (first loads, epilogue), which counts for wide layers over a short K
        const int nb = lp.nb_out > 0 ? lp.nb_out : (lp.d.n + 31) / 32;
        sum += c.per_mb * ((double)lp.kp * p->esz * nb * 32.0) / 1e6 + c.per_layer + c.per_block * ((nb + 7) / 8);
    }
    return c.f0 + rounds * sum * (1.0 + c.fill * std::min(1.0, m / 8192.0));
}

// Every CU takes 32x32 blocks of the current layer, a device-wide barrier between layers.
double estimate_coop_us(const ogc_mlp_plan_s* p) {
    const CoopCost& c = kCoop[model_dtype(p->desc.dtype)];
    const double mb = (p->desc.m + 31) / 32;
    double most = 0.0;
    for (const LayerPlan& lp : p->layers) most = std::max(most, mb * ((lp.d.n + 31) / 32));
    const double g = std::min(256.0, most);
    double t = c.c0;
    for (const LayerPlan& lp : p->layers) {
        const double blocks = mb * ((lp.d.n + 31) / 32), rounds = 0.5 * (std::ceil(blocks / g) + blocks / g);
        t += c.barrier + rounds * (c.block + c.step * ((double)lp.kp * p->esz / 32.0));
    }
    return t * (1.0 + c.fill * std::min(1.0, most / 256.0));
}

// The cluster kernel: `split` workgroups per 32-row tile, each streaming 1/split of the weights; after every layer
// but the last, a barrier of the tile's members and a copy of the whole tile back into LDS.  Fitted like the other
// mode models (chains of 2-5 layers, 64-4096 wide, 32-2048 rows, splits 2-16; rms error 8 %, worst 34 %: wide bf16
// layers at 1024 rows, underestimated).  The fp32 row serves forced splits only: the kernel has no split along K,
// an fp32 chain is bound by one CU's MFMA rate in it, and the plan does not offer it fp32 chains.

// One layer of the cluster kernel: the busiest member's weight stream, and the exchange if the layer is split.
double cluster_layer_us(const ogc_mlp_plan_s* p, int l, int split, bool whole) {
    const ClusterCost& c = kCluster[model_dtype(p->desc.dtype)];
    const int L = (int)p->layers.size(), waves = 8 * (whole ? 1 : split);
    const LayerPlan& lp = p->layers[l];
    const bool last = l == L - 1;
    const int nb = last ? (lp.d.n + 31) / 32 : lp.nb_out;
    const double kb = (double)lp.kp * p->esz;  // bytes of a row of the layer's input
    int wg = 0;                                // channel blocks of the busiest member (its wave w is wave w*stride)
    const int stride = whole ? 1 : split;
    for (int w = 0; w < 8 && w * stride < nb; ++w) wg += (nb - w * stride + waves - 1) / waves;
    const int per_wave = (nb + waves - 1) / waves;
    double t = c.per_mb * kb * 32.0 * wg / 1e6 + c.group * std::ceil(kb / 128.0) * ((per_wave + 3) / 4) + c.per_layer;
    if (!last && !whole) t += c.barrier + c.copy_mb * ((double)p->layers[l + 1].kp * p->esz * 32.0) / 1e6;
    return t;
}

// Bit l set: layer l is so small that every member computing all of it costs less than splitting it and
// exchanging the result.  The last layer is always split (nothing follows it, so no exchange either).
uint32_t cluster_whole_layers(const ogc_mlp_plan_s* p, int split) {
    uint32_t mask = 0;
    const int L = (int)p->layers.size();
    if (p->ov.cluster_whole == 0) return 0;  // override: split every layer
    for (int l = 0; l + 1 < L; ++l)
        if (cluster_layer_us(p, l, split, true) < cluster_layer_us(p, l, split, false)) mask |= 1u << l;
    return mask;
}

double estimate_cluster_us(const ogc_mlp_plan_s* p, int split) {
    const ClusterCost& c = kCluster[model_dtype(p->desc.dtype)];
    const int L = (int)p->layers.size();
    const double tiles = (p->desc.m + 31) / 32;
    const uint32_t whole = cluster_whole_layers(p, split);
    double t = c.c0, all_mb = 0.0;
    for (int l = 0; l < L; ++l) {
        const LayerPlan& lp = p->layers[l];
        const int nb = l == L - 1 ? (lp.d.n + 31) / 32 : lp.nb_out;
        const bool w = (whole >> l) & 1;
        t += cluster_layer_us(p, l, split, w);
        all_mb += (double)lp.kp * p->esz * 32.0 * nb / 1e6 * (w ? split : 1);
    }
    // every tile streams all the weights through the L2s: the aggregate term counts beyond a few dozen tiles
    return t * (1.0 + c.fill * std::min(1.0, tiles * split / 256.0)) + c.all_mb * tiles * all_mb;
}

// The cluster kernel whose waves split K inside a member: member j of S takes the channel blocks j, j + S, ... one
// after the other (rounds), each over the whole of K on its eight waves; every layer but the last is exchanged.
// 899 timed chains (the 12 calibration shapes, batch 32-2048, splits 2-32, three dtypes): 4-6 % rms, worst 22 %.
double estimate_cluster_ksplit_us(const ogc_mlp_plan_s* p, int split) {
    const KsplitCost& c = kKsplit[model_dtype(p->desc.dtype)];
    const int L = (int)p->layers.size();
    const double tiles = (p->desc.m + 31) / 32;
    double t = c.c0, all_mb = 0.0;
    for (int l = 0; l < L; ++l) {
        const LayerPlan& lp = p->layers[l];
        const bool last = l == L - 1;
        const int nb = last ? (lp.d.n + 31) / 32 : lp.nb_out;
        const double kb = (double)lp.kp * p->esz;
        t += ((nb + split - 1) / split) * (c.block + c.step * kb / 256.0);  // kb/32 k-steps over eight waves
        if (!last) t += c.barrier + c.copy_mb * ((double)p->layers[l + 1].kp * p->esz * 32.0) / 1e6;
        all_mb += kb * 32.0 * nb / 1e6;
    }
    return t * (1.0 + c.fill * std::min(1.0, tiles * split / 256.0)) + c.all_mb * tiles * all_mb;
}

// Workspace of the cluster kernels.  The members of a row tile exchange a layer's output through the workspace and are
// synchronised only among themselves, so two tiles may be several layers apart.  Every tile therefore owns a private
// region at a fixed stride (the widest exchanged row block) in each of two slots, and the slots alternate per EXCHANGED
// layer (a layer that every member computes whole needs no slot and no barrier).  Inside a tile two slots suffice: a
// member writes exchange e+2 only after the barrier of exchange e+1, which every member reaches only after it has
// copied exchange e out of the slot that e+2 reuses.  (Life-span reuse as in assign_buffers, Section VI, applied per tile.)
void assign_cluster_buffers(ogc_mlp_plan_s* p) {
    const int L = (int)p->layers.size();
    p->cluster_whole_mask = p->cluster_ksplit ? 0u : cluster_whole_layers(p, p->cluster_split);
    size_t stride = 0;
    for (int l = 0; l + 1 < L; ++l)
        if (!((p->cluster_whole_mask >> l) & 1)) stride = std::max(stride, (size_t)p->layers[l].kc_out * 512);
    stride = round_up(stride, 256);
    const size_t tiles = (size_t)(p->desc.m + 31) / 32, slot_bytes = tiles * stride;
    p->cluster_tile_stride = stride;
    p->slot_off.assign({0, slot_bytes});
    p->slot_size.assign({slot_bytes, slot_bytes});
    int exchanges = 0;
    for (int l = 0; l < L; ++l) {
        LayerPlan& lp = p->layers[l];
        if (l + 1 < L && !((p->cluster_whole_mask >> l) & 1)) {
            lp.out_slot = exchanges++ & 1;
            lp.out_off = p->slot_off[lp.out_slot];
        } else {
            lp.out_slot = -1;
            lp.out_off = 0;
        }
    }
    p->workspace_bytes = exchanges > 1 ? 2 * slot_bytes : (exchanges == 1 ? slot_bytes : 0);
}

ogc_status validate(const ogc_mlp_desc* d) {
    if (!d || !d->layers) return OGC_ERR_INVALID_ARG;
    if (d->dtype != OGC_F32 && d->dtype != OGC_BF16 && d->dtype != OGC_I8 && d->dtype != OGC_F8) return OGC_ERR_INVALID_ARG;
    const bool quant = d->dtype == OGC_I8 || d->dtype == OGC_F8;
    if (d->mode != OGC_MODE_AUTO && d->mode != OGC_MODE_PER_LAYER && d->mode != OGC_MODE_FUSED && d->mode != OGC_MODE_COOP)
        return OGC_ERR_INVALID_ARG;
    if (d->n_layers < 1 || d->n_layers > OGC_MAX_LAYERS) return OGC_ERR_SHAPE;
    if (d->m < 1) return OGC_ERR_SHAPE;
    if (d->residual != 0 && d->residual != 1) return OGC_ERR_INVALID_ARG;
    if ((d->x_layout != OGC_LAYOUT_PLAIN && d->x_layout != OGC_LAYOUT_BLOCKED) ||
        (d->y_layout != OGC_LAYOUT_PLAIN && d->y_layout != OGC_LAYOUT_BLOCKED))
        return OGC_ERR_INVALID_ARG;
    if (d->x_layout == OGC_LAYOUT_BLOCKED && d->residual) return OGC_ERR_UNSUPPORTED;  // the residual reads plain x
    if ((d->x_layout == OGC_LAYOUT_BLOCKED || d->y_layout == OGC_LAYOUT_BLOCKED) &&
        (d->mode == OGC_MODE_FUSED || d->mode == OGC_MODE_COOP))
        return OGC_ERR_UNSUPPORTED;
    for (int l = 0; l < d->n_layers; ++l) {
        const ogc_layer_desc& y = d->layers[l];
        if (y.k < 1 || y.n < 1) return OGC_ERR_SHAPE;
        if (l > 0 && y.k != d->layers[l - 1].n) return OGC_ERR_SHAPE;
        if (y.has_bias != 0 && y.has_bias != 1) return OGC_ERR_INVALID_ARG;
        if (y.act < OGC_ACT_NONE || y.act > OGC_ACT_SIGMOID) return OGC_ERR_INVALID_ARG;
        if (y.out != OGC_OUT_SAME && y.out != OGC_OUT_F32) return OGC_ERR_INVALID_ARG;
        if (y.out == OGC_OUT_F32 && (!quant || l != d->n_layers - 1)) return OGC_ERR_INVALID_ARG;
        if (y.out == OGC_OUT_F32 && d->y_layout == OGC_LAYOUT_BLOCKED) return OGC_ERR_INVALID_ARG;
        if (d->dtype == OGC_I8) {
            if (y.k > 65536) return OGC_ERR_SHAPE;
            if (!(y.in_scale > 0.0f) || !std::isfinite(y.in_scale)) return OGC_ERR_INVALID_ARG;
            if (y.in_zp < 0 || y.in_zp > 255) return OGC_ERR_INVALID_ARG;
            if (y.out == OGC_OUT_SAME) {
                if (!(y.out_scale > 0.0f) || !std::isfinite(y.out_scale)) return OGC_ERR_INVALID_ARG;
                if (y.out_zp < 0 || y.out_zp > 255) return OGC_ERR_INVALID_ARG;
            }
        }
        if (d->dtype == OGC_F8) {  // a signed format: scales only, the zero-point fields must be left at 0
            if (!(y.in_scale > 0.0f) || !std::isfinite(y.in_scale) || y.in_zp != 0) return OGC_ERR_INVALID_ARG;
            if (y.out == OGC_OUT_SAME && (!(y.out_scale > 0.0f) || !std::isfinite(y.out_scale) || y.out_zp != 0)) return OGC_ERR_INVALID_ARG;
        }
    }
    const int k0 = d->layers[0].k, nl = d->layers[d->n_layers - 1].n;
    if (d->x_layout == OGC_LAYOUT_PLAIN && d->ld_x < k0) return OGC_ERR_SHAPE;
    if (d->y_layout == OGC_LAYOUT_PLAIN && d->ld_y < nl) return OGC_ERR_SHAPE;
    if (d->residual) {
        if (quant) return OGC_ERR_INVALID_ARG;
        if (nl != k0) return OGC_ERR_SHAPE;
    }
    return OGC_OK;
}

void fill_args(const ogc_mlp_plan_s* p, int l, const uint8_t* packed, OgcLayerArgs* a) {
    const LayerPlan& lp = p->layers[l];
    std::memset(a, 0, sizeof(*a));
    a->w = packed + lp.w_off;
    a->scale = (const float*)(packed + lp.scale_off);
    a->bias = (const float*)(packed + lp.bias_off);
    a->ncomp = (const int32_t*)(packed + lp.ncomp_off);
    a->M = p->desc.m;
    a->K = lp.d.k;
    a->N = lp.d.n;
    a->KC = lp.kc;
    a->KC_out = lp.kc_out;
    a->NB_out = lp.nb_out;
    a->act = lp.d.act;
    a->has_comp = (p->desc.dtype == OGC_I8 && lp.d.in_zp != 128) ? 1 : 0;
    a->out_f32 = (lp.d.out == OGC_OUT_F32) ? 1 : 0;
    a->inv_cs = lp.inv_cs;
    a->zp_out = (float)lp.d.out_zp;
    a->has_bias = lp.d.has_bias;
    a->q_hi = 255.0f - (float)lp.d.out_zp;
    // the result stays in the s8-with-128-subtracted form: every layer but the last, and a blocked y
    const bool internal = l + 1 < (int)p->layers.size() || p->desc.y_layout == OGC_LAYOUT_BLOCKED;
    if (internal && lp.d.out_zp == 128) {
        a->q_add = 0;
        a->q_xor = 0;
    } else {
        a->q_add = (uint32_t)lp.d.out_zp * 0x01010101u;
        a->q_xor = internal ? 0x80808080u : 0u;
    }
}

}  // namespace

extern "C" {

ogc_status ogc_mlp_plan(const ogc_mlp_desc* desc, ogc_mlp_plan_t* out_plan) {
    return ogc_mlp_plan_with_overrides(desc, nullptr, out_plan);
}

ogc_status ogc_mlp_plan_with_overrides(const ogc_mlp_desc* desc, const ogc_plan_overrides* overrides, ogc_mlp_plan_t* out_plan) {
    if (!out_plan) return OGC_ERR_INVALID_ARG;
    ogc_status st = validate(desc);
    if (st != OGC_OK) return st;
    const ogc_plan_overrides none = {-1, -1, -1, -1, -1};
    const ogc_plan_overrides ov = overrides ? *overrides : none;
    if (ov.tile < -1 || ov.tile >= OGC_NUM_TILES || ov.ksplit_log2 < -1 || ov.ksplit_log2 > 3 || ov.cluster_split < -1 ||
        ov.cluster_split > 32 || ov.cluster_ksplit < -1 || ov.cluster_ksplit > 1 || ov.cluster_whole < -1 || ov.cluster_whole > 1)
        return OGC_ERR_INVALID_ARG;
    ogc_mlp_plan_s* p = new (std::nothrow) ogc_mlp_plan_s();
    if (!p) return OGC_ERR_INVALID_ARG;
    p->desc = *desc;
    p->desc.layers = nullptr;
    p->ov = ov;
    p->prepacked.store(0);
    p->cu_count.store(0);
    p->barrier_budget.store(OGC_BARRIER_BUDGET);
    p->barrier_extra.store(0);
    const int L = desc->n_layers;
    const int esz = desc->dtype == OGC_F32 ? 4 : (desc->dtype == OGC_BF16 ? 2 : 1);
    p->esz = esz;
    const bool quant = desc->dtype == OGC_I8 || desc->dtype == OGC_F8;
    const int kgran = quant ? 64 : 32;  // padded K granularity in elements (>= 64 bytes)
    p->layers.resize(L);
    int max_kc = 0;
    for (int l = 0; l < L; ++l) {
        LayerPlan& lp = p->layers[l];
        lp.d = desc->layers[l];
        lp.kp = (int)round_up((size_t)lp.d.k, kgran);
        lp.kc = lp.kp * esz / 16;
        if (lp.kc > max_kc) max_kc = lp.kc;
        lp.inv_cs = (quant && lp.d.out == OGC_OUT_SAME) ? 1.0f / lp.d.out_scale : 0.0f;
    }
    for (int l = 0; l < L; ++l) {
        LayerPlan& lp = p->layers[l];
        if (l + 1 < L) {
            lp.nb_out = p->layers[l + 1].kp / 32;
            lp.kc_out = p->layers[l + 1].kc;
        } else if (desc->y_layout == OGC_LAYOUT_BLOCKED) {
            const int kp_y = (int)round_up((size_t)lp.d.n, kgran);  // as the next chain's first layer will pad it
            lp.nb_out = kp_y / 32;
            lp.kc_out = kp_y * esz / 16;
        } else {
            lp.nb_out = 0;
            lp.kc_out = 0;
        }
    }
    // Kernel family.  The fused-chain kernel needs two LDS activation buffers of 32 rows x widest padded row.
    const size_t lds_need = (size_t)2 * max_kc * 512;
    const bool fused_fits = lds_need <= ogc_fused_lds_limit();
    size_t wbytes = 0;
    for (int l = 0; l < L; ++l) wbytes += (size_t)p->layers[l].kp * esz * p->layers[l].d.n;
    int mode = desc->mode;
    const bool blocked_io = desc->x_layout == OGC_LAYOUT_BLOCKED || desc->y_layout == OGC_LAYOUT_BLOCKED;
    if (mode == OGC_MODE_AUTO && blocked_io) mode = OGC_MODE_PER_LAYER;
    if (mode == OGC_MODE_FUSED && !fused_fits) {
        delete p;
        return OGC_ERR_UNSUPPORTED;
    }
    // Per-layer candidates first: tile, split and the model's estimate of every layer (used if the chain runs layer
    // by layer, and to decide whether it should).
    double per_us = 0.0;
    bool per_timed = true;
    for (int l = 0; l < L; ++l) {
        LayerPlan& lp = p->layers[l];
        const int rows = lp.nb_out * 32 > lp.d.n ? lp.nb_out * 32 : lp.d.n;
        // the stream kernel keeps its accumulators in fixed registers: no out-of-line calls (sigmoid) in it
        const bool dma_ok = desc->dtype != OGC_F32 && lp.d.act != OGC_ACT_SIGMOID &&
                            !(desc->dtype == OGC_I8 && lp.d.in_zp != 128) &&
                            (l > 0 || desc->x_layout == OGC_LAYOUT_BLOCKED ||
                             (((long long)desc->ld_x * esz) % 16 == 0 && lp.kp == lp.d.k));
        choose_tile_and_split(desc->dtype, desc->m, rows, lp.kc / 4, dma_ok, p->ov.tile, p->ov.ksplit_log2, &lp.tile, &lp.ksplit_log2,
                              &lp.est_us);
        if (lp.est_us < 0) per_timed = false;
        per_us += lp.est_us - kProfiledLaunchExtraUs;
    }
    p->mode_us[0] = per_timed ? per_us : -1.0;
    p->mode_us[1] = (fused_fits && (quant || wbytes <= (size_t)2600000)) ? estimate_fused_us(p) : -1.0;
    p->mode_us[2] = (!blocked_io && L > 1) ? estimate_coop_us(p) : -1.0;
    // The cooperative mode has two kernels: blocks dealt to all workgroups (above), or a few workgroups per row tile
    // (the cluster kernel).  The split with the lowest estimate competes; the cluster_split override forces one (0: never).
    p->cluster_split = p->cluster_ksplit = 0;
    p->cluster_spread = wbytes > (size_t)3000000;  // weights beyond one XCD's L2: a tile's members on different XCDs
    const bool ksplit_fits = ogc_cluster_ksplit_lds_bytes((size_t)max_kc * 512) <= ogc_fused_lds_limit();
    const int forced = p->ov.cluster_split;
    const int forced_ks = p->ov.cluster_ksplit;
    if (p->mode_us[2] >= 0 && forced > 0 && forced_ks == 1) {
        // test override: the k-split variant with this many members per tile
        if (ksplit_fits && ogc_cluster_xcds((desc->m + 31) / 32, forced, p->cluster_spread) >= 0) {
            p->cluster_split = forced;
            p->cluster_ksplit = 1;
            p->mode_us[2] = estimate_cluster_ksplit_us(p, forced);
        }
    } else if (p->mode_us[2] >= 0 && forced < 0) {
        // the model's choice among the cooperative kernel, the cluster kernel (channel blocks split over the waves
        // of all members) and its k-split variant, each with its best split
        const int m_blocks = (desc->m + 31) / 32;
        if (fused_fits && desc->dtype != OGC_F32) {
            for (int split = 2; split <= 16; split *= 2) {
                if (ogc_cluster_xcds(m_blocks, split, p->cluster_spread) < 0) continue;
                // no layer worth an exchange: the members would all run the fused kernel's work
                if (cluster_whole_layers(p, split) == (1u << (L - 1)) - 1u) continue;
                const double e = estimate_cluster_us(p, split);
                if (e < p->mode_us[2]) {
                    p->mode_us[2] = e;
                    p->cluster_split = split;
                    p->cluster_ksplit = 0;
                }
            }
        }
        if (ksplit_fits && forced_ks != 0) {
            for (int split = 2; split <= 32; split *= 2) {
                if (ogc_cluster_xcds(m_blocks, split, p->cluster_spread) < 0) continue;
                const double e = estimate_cluster_ksplit_us(p, split);
                if (e < p->mode_us[2]) {
                    p->mode_us[2] = e;
                    p->cluster_split = split;
                    p->cluster_ksplit = 1;
                }
            }
        }
    } else if (p->mode_us[2] >= 0 && fused_fits) {
        const int m_blocks = (desc->m + 31) / 32;
        if (forced > 0) {
            if (ogc_cluster_xcds(m_blocks, forced, p->cluster_spread) >= 0) {
                p->cluster_split = forced;
                p->mode_us[2] = estimate_cluster_us(p, forced);
            }
        }
    }
    if (mode == OGC_MODE_AUTO) {
        // The mode whose estimate is lowest (section "cost model" of the sources above: each mode has its own fitted
        // model).  The fused kernel is a candidate only where it was timed without its cliff: bf16 / fp32 chains
        // whose weights exceed about 2.5 MB run several times slower per byte in it.
        // A single-launch mode wins ties within 7 %: its model is the tighter one, and it keeps the intermediates
        // on chip.
        int single = -1;
        if (p->mode_us[1] >= 0) single = 1;
        if (p->mode_us[2] >= 0 && (single < 0 || p->mode_us[2] < p->mode_us[1])) single = 2;
        if (single >= 0 && (p->mode_us[0] < 0 || p->mode_us[single] <= 1.07 * p->mode_us[0]))
            mode = single == 1 ? OGC_MODE_FUSED : OGC_MODE_COOP;
        else
            mode = OGC_MODE_PER_LAYER;
    }
    p->mode = mode;
    p->lds_buf_bytes = max_kc * 512;
    p->mp = (int)round_up((size_t)desc->m, 256);
    // Packed blob layout.
    size_t off = 0;
    for (int l = 0; l < L; ++l) {
        LayerPlan& lp = p->layers[l];
        const int rows = lp.nb_out * 32 > lp.d.n ? lp.nb_out * 32 : lp.d.n;
        if (mode == OGC_MODE_PER_LAYER) {
            lp.npw = (int)round_up((size_t)rows, ogc_tile_info(lp.tile).bn);
        } else {
            lp.tile = -1;
            lp.ksplit_log2 = 0;
            lp.est_us = -1.0;
            lp.npw = (int)round_up((size_t)rows, 32);
        }
        lp.w_off = off;
        off += round_up((size_t)lp.npw * lp.kc * 16, 256);
        lp.scale_off = off;
        off += round_up((size_t)lp.npw * 4, 256);
        lp.bias_off = off;
        off += round_up((size_t)lp.npw * 4, 256);
        lp.ncomp_off = off;
        off += round_up((size_t)lp.npw * 4, 256);
    }
    p->sync_off = off;
    if (mode == OGC_MODE_COOP) off += (size_t)OGC_SYNC_WORDS * 8;
    p->packed_bytes = off;
    p->partial_off = p->partial_bytes = 0;
    if (mode != OGC_MODE_COOP) p->cluster_split = p->cluster_ksplit = 0;
    p->cluster_whole_mask = 0;
    p->cluster_tile_stride = 0;
    if (mode == OGC_MODE_COOP && p->cluster_split > 0) {
        assign_cluster_buffers(p);
    } else if (mode == OGC_MODE_COOP) {
        assign_buffers(p);
    } else if (mode == OGC_MODE_PER_LAYER) {
        assign_buffers(p);
        for (int l = 0; l < L; ++l) {
            const LayerPlan& lp = p->layers[l];
            if (lp.ksplit_log2 > 0) {
                const size_t need = ((size_t)p->mp * lp.npw * 4) << lp.ksplit_log2;
                if (need > p->partial_bytes) p->partial_bytes = need;
            }
        }
        if (p->partial_bytes > 0) {
            p->partial_off = round_up(p->workspace_bytes, 256);
            p->workspace_bytes = p->partial_off + p->partial_bytes;
        }
    } else {
        for (int l = 0; l < L; ++l) {
            p->layers[l].out_slot = -1;
            p->layers[l].out_off = 0;
        }
        p->workspace_bytes = 0;
    }
    *out_plan = p;
    return OGC_OK;
}

ogc_status ogc_mlp_packed_bytes(ogc_mlp_plan_t plan, size_t* bytes) {
    if (!plan || !bytes) return OGC_ERR_INVALID_ARG;
    *bytes = plan->packed_bytes;
    return OGC_OK;
}

ogc_status ogc_mlp_blocked_bytes(ogc_mlp_plan_t plan, int32_t which, size_t* bytes) {
    if (!plan || !bytes || (which != 0 && which != 1)) return OGC_ERR_INVALID_ARG;
    const LayerPlan& first = plan->layers.front();
    const LayerPlan& last = plan->layers.back();
    if (which == 0) *bytes = plan->desc.x_layout == OGC_LAYOUT_BLOCKED ? (size_t)plan->mp * first.kc * 16 : 0;
    else *bytes = plan->desc.y_layout == OGC_LAYOUT_BLOCKED ? (size_t)plan->mp * last.kc_out * 16 : 0;
    return OGC_OK;
}

ogc_status ogc_mlp_workspace_bytes(ogc_mlp_plan_t plan, size_t* bytes) {
    if (!plan || !bytes) return OGC_ERR_INVALID_ARG;
    *bytes = plan->workspace_bytes;
    return OGC_OK;
}

ogc_status ogc_mlp_chosen_mode(ogc_mlp_plan_t plan, int32_t* mode) {
    if (!plan || !mode) return OGC_ERR_INVALID_ARG;
    *mode = plan->mode;
    return OGC_OK;
}

ogc_status ogc_mlp_buffer_assignment(ogc_mlp_plan_t plan, int32_t layer, int32_t* slot, size_t* offset) {
    if (!plan || !slot || !offset) return OGC_ERR_INVALID_ARG;
    if (layer < 0 || layer >= (int)plan->layers.size()) return OGC_ERR_INVALID_ARG;
    *slot = plan->layers[layer].out_slot;
    *offset = plan->layers[layer].out_off;
    return OGC_OK;
}

ogc_status ogc_mlp_prepack_weights(ogc_mlp_plan_t plan, const void* const* w, const float* const* bias,
                                   const float* const* w_scale, void* packed, void* stream) {
    if (!plan || !w || !packed) return OGC_ERR_INVALID_ARG;
    if (((uintptr_t)packed & 255) != 0) return OGC_ERR_ALIGNMENT;
    const int L = (int)plan->layers.size();
    const bool i8 = plan->desc.dtype == OGC_I8 || plan->desc.dtype == OGC_F8;  // the quantized scheme: per-channel weight scales
    if (i8 && !w_scale) return OGC_ERR_INVALID_ARG;
    for (int l = 0; l < L; ++l) {
        if (!w[l]) return OGC_ERR_INVALID_ARG;
        if (plan->layers[l].d.has_bias && (!bias || !bias[l])) return OGC_ERR_INVALID_ARG;
        if (i8 && !w_scale[l]) return OGC_ERR_INVALID_ARG;
    }
    uint8_t* blob = (uint8_t*)packed;
    for (int l = 0; l < L; ++l) {
        const LayerPlan& lp = plan->layers[l];
        int rc = ogc_launch_prepack_weights(w[l], blob + lp.w_off, lp.d.k, lp.d.n, lp.kc, lp.npw, plan->esz, stream);
        if (rc != 0) return OGC_ERR_DEVICE;
        rc = ogc_launch_prepack_params(plan->desc.dtype, w[l], i8 ? w_scale[l] : nullptr, lp.d.has_bias ? bias[l] : nullptr,
                                       lp.d.in_scale, lp.d.in_zp, lp.d.k, lp.d.n, lp.npw, (float*)(blob + lp.scale_off),
                                       (float*)(blob + lp.bias_off), (int32_t*)(blob + lp.ncomp_off), stream);
        if (rc != 0) return OGC_ERR_DEVICE;
    }
    if (plan->mode == OGC_MODE_COOP && ogc_launch_zero_sync(blob + plan->sync_off, stream) != 0) return OGC_ERR_DEVICE;
    plan->prepacked.store(1);
    return OGC_OK;
}

// Shared body of ogc_mlp_run / ogc_mlp_run_profiled.  With ev != NULL, event ev[i] is recorded on the stream
// before launch i and ev[n] after the last one.
static ogc_status run_impl(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* workspace, void* stream,
                           hipEvent_t* ev, long long* clocks = nullptr) {
    if (!plan || !x || !y || !packed) return OGC_ERR_INVALID_ARG;
    if (!plan->prepacked.load()) return OGC_ERR_NOT_PREPACKED;
    if (((uintptr_t)packed & 255) != 0) return OGC_ERR_ALIGNMENT;
    const int esz = plan->esz;
    const int L = (int)plan->layers.size();
    const LayerPlan& last = plan->layers[L - 1];
    const int eo = (last.d.out == OGC_OUT_F32) ? 4 : esz;
    const bool x_blocked = plan->desc.x_layout == OGC_LAYOUT_BLOCKED, y_blocked = plan->desc.y_layout == OGC_LAYOUT_BLOCKED;
    if (((uintptr_t)x % (x_blocked ? 256 : esz)) != 0 || ((uintptr_t)y % (y_blocked ? 256 : eo)) != 0) return OGC_ERR_ALIGNMENT;
    if (plan->workspace_bytes > 0) {
        if (!workspace) return OGC_ERR_WORKSPACE;
        if (((uintptr_t)workspace & 255) != 0) return OGC_ERR_ALIGNMENT;
    }
    const uint8_t* blob = (const uint8_t*)packed;
    const long long ldx_b = (long long)plan->desc.ld_x * esz, ldy_b = (long long)plan->desc.ld_y * eo;
    const int x_vec = ((uintptr_t)x % 16 == 0) && (ldx_b % 16 == 0) && (((long long)plan->layers[0].d.k * esz) % 16 == 0);
    const int y_vec = ((uintptr_t)y % 16 == 0) && (ldy_b % 16 == 0);

    auto finish_args = [&](int l, OgcLayerArgs* a) {
        fill_args(plan, l, blob, a);
        if (l == 0) {
            a->x = (const uint8_t*)x;
            a->ldx_bytes = ldx_b;
            a->x_vec_ok = x_vec;
        }
        if (l == L - 1) {
            a->y = (uint8_t*)y;
            a->ldy_bytes = ldy_b;
            a->y_vec_ok = y_vec;
            if (plan->desc.residual) {
                a->res = (const uint8_t*)x;
                a->ldres_bytes = ldx_b;
                a->res_vec_ok = ((uintptr_t)x % 16 == 0) && (ldx_b % 16 == 0);
            }
        }
    };

    if (plan->mode == OGC_MODE_FUSED) {
        OgcChainArgs c;
        std::memset(&c, 0, sizeof(c));
        c.n_layers = L;
        c.lds_buf_bytes = plan->lds_buf_bytes;
        for (int l = 0; l < L; ++l) finish_args(l, &c.layer[l]);
        if (ev && hipEventRecord(ev[0], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
        const int rc = ogc_launch_fused(plan->desc.dtype, &c, (plan->desc.m + 31) / 32, stream);
        if (rc != 0) return OGC_ERR_DEVICE;
        if (ev && hipEventRecord(ev[1], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
        return OGC_OK;
    }
    uint8_t* ws = (uint8_t*)workspace;
    if (plan->mode == OGC_MODE_COOP) {
        OgcChainArgs c;
        std::memset(&c, 0, sizeof(c));
        c.n_layers = L;
        const int m_blocks = (plan->desc.m + 31) / 32;
        long max_blocks = 1;
        for (int l = 0; l < L; ++l) {
            finish_args(l, &c.layer[l]);
            if (l > 0 && plan->layers[l - 1].out_slot >= 0) c.layer[l].x = ws + plan->layers[l - 1].out_off;
            if (l < L - 1 && plan->layers[l].out_slot >= 0) c.layer[l].y = ws + plan->layers[l].out_off;
            const long nb = l < L - 1 ? plan->layers[l].nb_out : (plan->layers[l].d.n + 31) / 32;
            if ((long)m_blocks * nb > max_blocks) max_blocks = (long)m_blocks * nb;
        }
        c.barrier_budget = plan->barrier_budget.load();
        c.barrier_extra = plan->barrier_extra.load();
        int cus = plan->cu_count.load();
        if (cus <= 0) {  // asked once per plan: two runtime calls
            cus = ogc_device_cu_count();
            if (cus <= 0) return OGC_ERR_DEVICE;
            plan->cu_count.store(cus);
        }
        if (plan->cluster_split > 0) {
            c.lds_buf_bytes = plan->lds_buf_bytes;
            c.cluster_whole_mask = plan->cluster_whole_mask;
            c.cluster_tile_stride = (uint32_t)plan->cluster_tile_stride;
            if (ev && hipEventRecord(ev[0], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
            const int rc = ogc_launch_cluster(plan->desc.dtype, plan->cluster_ksplit, &c, m_blocks, plan->cluster_split, plan->cluster_spread,
                                              cus, (void*)(blob + plan->sync_off), stream);
            if (rc != 0) return OGC_ERR_DEVICE;
            if (ev && hipEventRecord(ev[1], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
            return OGC_OK;
        }
        const int grid = (int)(max_blocks < cus ? max_blocks : cus);
        if (ev && hipEventRecord(ev[0], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
        const int rc = ogc_launch_coop(plan->desc.dtype, &c, m_blocks, grid, (void*)(blob + plan->sync_off), stream);
        if (rc != 0) return OGC_ERR_DEVICE;
        if (ev && hipEventRecord(ev[1], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
        return OGC_OK;
    }
    for (int l = 0; l < L; ++l) {
        OgcLayerArgs a;
        finish_args(l, &a);
        if (l > 0) a.x = ws + plan->layers[l - 1].out_off;
        if (l < L - 1) a.y = ws + plan->layers[l].out_off;
        if (plan->layers[l].ksplit_log2 > 0) {
            a.ksplit_log2 = plan->layers[l].ksplit_log2;
            a.partial = ws + plan->partial_off;
            a.pmb = plan->mp / 32;
            a.pnb = plan->layers[l].npw / 32;
        }
        const int t = plan->layers[l].tile;
        if (clocks && (t == OGC_TILE_DMA || t == OGC_TILE_DMA8 || t == OGC_TILE_DMAK2)) a.clocks = clocks + (size_t)l * OGC_CLOCK_WORDS_PER_LAUNCH;
        if (ev && hipEventRecord(ev[l], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
        const int rc = ogc_launch_layer(plan->desc.dtype, plan->layers[l].tile, l == 0 && !x_blocked, l == L - 1 && !y_blocked, &a,
                                        stream);
        if (rc != 0) return OGC_ERR_DEVICE;
    }
    if (ev && hipEventRecord(ev[L], (hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
    return OGC_OK;
}

ogc_status ogc_mlp_run(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* workspace, void* stream) {
    return run_impl(plan, x, y, packed, workspace, stream, nullptr);
}

ogc_status ogc_mlp_run_static(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* stream) {
    if (!plan) return OGC_ERR_INVALID_ARG;
    if (plan->workspace_bytes > (size_t)OGC_STATIC_SCRATCH_BYTES) return OGC_ERR_WORKSPACE;
    void* ws = nullptr;
    if (plan->workspace_bytes > 0 && ogc_static_scratch(&ws) != 0) return OGC_ERR_DEVICE;
    return run_impl(plan, x, y, packed, ws, stream, nullptr);
}

size_t ogc_mlp_static_workspace_limit(void) { return (size_t)OGC_STATIC_SCRATCH_BYTES; }

ogc_status ogc_mlp_run_clocked(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* workspace, void* stream,
                               int64_t* clocks) {
    if (!clocks || ((uintptr_t)clocks & 7) != 0) return clocks ? OGC_ERR_ALIGNMENT : OGC_ERR_INVALID_ARG;
    return run_impl(plan, x, y, packed, workspace, stream, nullptr, (long long*)clocks);
}

size_t ogc_mlp_clock_words_per_launch(void) { return (size_t)OGC_CLOCK_WORDS_PER_LAUNCH; }

ogc_status ogc_quantize_e4m3(const float* x, uint8_t* out, size_t n, float scale, void* stream) {
    if ((n && (!x || !out)) || !(scale > 0.0f) || !std::isfinite(scale)) return OGC_ERR_INVALID_ARG;
    if (((uintptr_t)x & 3) != 0) return OGC_ERR_ALIGNMENT;
    return ogc_launch_quantize_e4m3(x, out, n, 1.0f / scale, stream) == 0 ? OGC_OK : OGC_ERR_DEVICE;
}

ogc_status ogc_dequantize_e4m3(const uint8_t* x, float* out, size_t n, float scale, void* stream) {
    if ((n && (!x || !out)) || !std::isfinite(scale)) return OGC_ERR_INVALID_ARG;
    if (((uintptr_t)out & 3) != 0) return OGC_ERR_ALIGNMENT;
    return ogc_launch_dequantize_e4m3(x, out, n, scale, stream) == 0 ? OGC_OK : OGC_ERR_DEVICE;
}

ogc_status ogc_mlp_num_launches(ogc_mlp_plan_t plan, int32_t* n) {
    if (!plan || !n) return OGC_ERR_INVALID_ARG;
    *n = plan->mode == OGC_MODE_PER_LAYER ? (int32_t)plan->layers.size() : 1;
    return OGC_OK;
}

ogc_status ogc_mlp_run_profiled(ogc_mlp_plan_t plan, const void* x, void* y, const void* packed, void* workspace,
                                void* stream, float* launch_ms) {
    if (!plan || !launch_ms) return OGC_ERR_INVALID_ARG;
    const int n = plan->mode == OGC_MODE_PER_LAYER ? (int)plan->layers.size() : 1;
    hipEvent_t ev[OGC_MAX_LAYERS + 1];
    int made = 0;
    ogc_status st = OGC_OK;
    for (; made <= n; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) {
            st = OGC_ERR_DEVICE;
            break;
        }
    if (st == OGC_OK) st = run_impl(plan, x, y, packed, workspace, stream, ev);
    if (st == OGC_OK && hipEventSynchronize(ev[n]) != hipSuccess) st = OGC_ERR_DEVICE;
    if (st == OGC_OK)
        for (int i = 0; i < n; ++i)
            if (hipEventElapsedTime(&launch_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = OGC_ERR_DEVICE;
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    if (st == OGC_OK) st = ogc_mlp_check(plan, packed, stream);
    return st;
}

ogc_status ogc_mlp_check(ogc_mlp_plan_t plan, const void* packed, void* stream) {
    if (!plan || !packed) return OGC_ERR_INVALID_ARG;
    if (plan->mode != OGC_MODE_COOP) return OGC_OK;  // the other modes have no waits that can give up
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
    uint8_t* word = (uint8_t*)packed + plan->sync_off + (size_t)OGC_SYNC_ERR_WORD * 8;
    unsigned long long v = 0;
    if (hipMemcpy(&v, word, sizeof v, hipMemcpyDeviceToHost) != hipSuccess) return OGC_ERR_DEVICE;
    if (v == 0) return OGC_OK;
    // reported once: the word and the counters start the next run from zero
    if (ogc_launch_zero_sync((uint8_t*)packed + plan->sync_off, stream) != 0) return OGC_ERR_DEVICE;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return OGC_ERR_DEVICE;
    return OGC_ERR_TIMEOUT;
}

ogc_status ogc_mlp_test_barrier(ogc_mlp_plan_t plan, int32_t budget, int32_t extra_target) {
    if (!plan || budget < 1 || extra_target < 0) return OGC_ERR_INVALID_ARG;
    plan->barrier_budget.store(budget);
    plan->barrier_extra.store(extra_target);
    return OGC_OK;
}

ogc_status ogc_mlp_cluster_layout(ogc_mlp_plan_t plan, int32_t* members, int32_t* ksplit, uint32_t* whole_mask, size_t* tile_stride) {
    if (!plan || !members || !ksplit || !whole_mask || !tile_stride) return OGC_ERR_INVALID_ARG;
    *members = plan->mode == OGC_MODE_COOP ? plan->cluster_split : 0;
    *ksplit = plan->cluster_ksplit;
    *whole_mask = plan->cluster_whole_mask;
    *tile_stride = plan->cluster_tile_stride;
    return OGC_OK;
}

void ogc_mlp_destroy(ogc_mlp_plan_t plan) { delete plan; }

const char* ogc_status_string(ogc_status s) {
    switch (s) {
    case OGC_OK: return "ok";
    case OGC_ERR_INVALID_ARG: return "invalid argument";
    case OGC_ERR_UNSUPPORTED: return "unsupported configuration";
    case OGC_ERR_SHAPE: return "bad or inconsistent shape";
    case OGC_ERR_ALIGNMENT: return "misaligned pointer";
    case OGC_ERR_WORKSPACE: return "workspace missing";
    case OGC_ERR_NOT_PREPACKED: return "weights not prepacked";
    case OGC_ERR_DEVICE: return "HIP runtime error";
    case OGC_ERR_TIMEOUT: return "a barrier wait of the cooperative mode gave up: the output of that run is invalid";
    }
    return "unknown status";
}

ogc_status ogc_mlp_estimated_us(ogc_mlp_plan_t plan, int32_t layer, float* us) {
    if (!plan || !us || layer < 0 || layer >= (int)plan->layers.size()) return OGC_ERR_INVALID_ARG;
    *us = (plan->mode == OGC_MODE_PER_LAYER) ? (float)plan->layers[layer].est_us : -1.0f;
    return OGC_OK;
}

ogc_status ogc_mlp_mode_estimates(ogc_mlp_plan_t plan, float us[3]) {
    if (!plan || !us) return OGC_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i) us[i] = (float)plan->mode_us[i];
    return OGC_OK;
}

const char* ogc_mlp_kernel_name(ogc_mlp_plan_t plan, int32_t layer) {
    if (!plan || layer < 0 || layer >= (int)plan->layers.size()) return nullptr;
    if (plan->mode == OGC_MODE_FUSED) return ogc_fused_kernel_name(plan->desc.dtype);
    if (plan->mode == OGC_MODE_COOP)
        return plan->cluster_split > 0 ? ogc_cluster_kernel_name(plan->desc.dtype, plan->cluster_ksplit) : ogc_coop_kernel_name(plan->desc.dtype);
    const int L = (int)plan->layers.size();
    const ogc_layer_desc& d = plan->layers[layer].d;
    return ogc_layer_kernel_name(plan->desc.dtype, plan->layers[layer].tile,
                                 layer == 0 && plan->desc.x_layout == OGC_LAYOUT_PLAIN,
                                 layer == L - 1 && plan->desc.y_layout == OGC_LAYOUT_PLAIN, d.act, d.out == OGC_OUT_F32,
                                 plan->layers[layer].ksplit_log2 > 0);
}

}  // extern "C"
