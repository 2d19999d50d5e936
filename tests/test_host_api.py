"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header declares,
validates descriptions, lays out the packed blob and assigns workspace buffers by life span."""
import ctypes
import os
import re

import pytest

from paper_2301_01333_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _built():
    return os.path.exists(b.LIB_PATH)


pytestmark = pytest.mark.skipif(not _built(), reason="libogc_mlp.so not built (python -m paper_2301_01333_amd.build)")


def layer(k, n, **kw):
    d = dict(k=k, n=n, has_bias=1, act=b.OGC_ACT_RELU, in_scale=0.05, in_zp=128, out_scale=0.1, out_zp=128, out=0)
    d.update(kw)
    return d


def test_library_exports_every_declared_symbol():
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        hdr = open(os.path.join(ROOT, "include", name)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
        declared |= set(re.findall(r"\b(ogc_[a-z_0-9]+)\s*\(", hdr))
    assert {"ogc_mlp_plan", "ogc_mlp_prepack_weights", "ogc_mlp_run", "ogc_mha_run"} <= declared
    lib = ctypes.CDLL(b.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(b.EXPORTS)


def test_status_strings():
    for s in range(0, -8, -1):
        assert b.status_string(s) and b.status_string(s) != "unknown status"
    assert b.status_string(-99) == "unknown status"


@pytest.mark.parametrize("kw,status", [
    (dict(dtype=7), -1),
    (dict(m=0), -3),
    (dict(layers=[]), -3),
    (dict(layers=[layer(8, 8), layer(9, 4)]), -3),                 # k of layer 1 != n of layer 0
    (dict(layers=[layer(0, 8)]), -3),
    (dict(layers=[layer(8, 8, act=9)]), -1),
    (dict(layers=[layer(70000, 8)]), -3),                          # int8 K limit
    (dict(layers=[layer(8, 8, in_scale=0.0)]), -1),
    (dict(layers=[layer(8, 8, in_scale=float("inf"))]), -1),
    (dict(layers=[layer(8, 8, in_zp=256)]), -1),
    (dict(layers=[layer(8, 8, out_scale=-1.0)]), -1),
    (dict(layers=[layer(8, 8, out=1), layer(8, 8)]), -1),          # fp32 output only on the last layer
    (dict(dtype=b.OGC_F32, layers=[layer(8, 8, out=1)]), -1),      # and only for int8
    (dict(ld_x=7), -3),
    (dict(ld_y=7), -3),
    (dict(residual=1), -1),                                        # no residual for int8
    (dict(dtype=b.OGC_BF16, residual=1, layers=[layer(8, 16)], ld_y=16), -3),
    (dict(mode=5), -1),
    (dict(mode=b.OGC_MODE_FUSED, dtype=b.OGC_BF16, layers=[layer(1024, 4096), layer(4096, 1024)], ld_x=1024, ld_y=1024), -2),
])
def test_plan_rejects_bad_descriptions(kw, status):
    args = dict(dtype=b.OGC_I8, m=16, layers=[layer(8, 8)], ld_x=8, ld_y=8, residual=0, mode=0)
    args.update(kw)
    with pytest.raises(b.OgcError) as e:
        b.ogc_mlp_plan(args["dtype"], args["m"], args["layers"], args["ld_x"], args["ld_y"], args["residual"], args["mode"])
    assert e.value.status == status


def test_null_arguments_are_refused():
    lib = b.lib()
    assert lib.ogc_mlp_plan(None, None) == -1
    assert lib.ogc_mlp_packed_bytes(None, None) == -1
    assert lib.ogc_mlp_run(None, None, None, None, None, None) == -1
    assert lib.ogc_mlp_prepack_weights(None, None, None, None, None, None) == -1
    lib.ogc_mlp_destroy(None)
    assert lib.ogc_mlp_kernel_name(None, 0) is None


def test_run_and_prepack_argument_checks_need_no_device():
    p = b.ogc_mlp_plan(b.OGC_I8, 64, [layer(64, 64), layer(64, 64)], 64, 64, 0, b.OGC_MODE_PER_LAYER)
    lib = b.lib()
    fake = 0x7F0000000000  # never dereferenced: every check below fails before any launch
    assert lib.ogc_mlp_run(p, fake, fake, fake, fake, None) == -6              # not prepacked
    arr = (ctypes.c_void_p * 2)(fake, fake)
    assert lib.ogc_mlp_prepack_weights(p, arr, None, arr, fake, None) == -1      # bias missing though has_bias
    assert lib.ogc_mlp_prepack_weights(p, arr, arr, None, fake, None) == -1      # int8 needs w_scale
    assert lib.ogc_mlp_prepack_weights(p, arr, arr, arr, fake + 8, None) == -4   # packed misaligned
    b.ogc_mlp_destroy(p)


def test_mode_choice_and_sizes():
    # config 3 shape: small batch, 2.2 MB of weights -> one launch, a few workgroups per row tile (cluster kernel),
    # intermediates through two workspace slots of 256 rows x 1024 bytes
    dims = [479, 1024, 1024, 512, 256, 1]
    ls = [layer(dims[i], dims[i + 1]) for i in range(5)]
    ls[-1].update(out=1, act=b.OGC_ACT_SIGMOID)
    p = b.ogc_mlp_plan(b.OGC_I8, 256, ls, 479, 1, 0, 0)
    assert b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_COOP
    assert b.ogc_mlp_kernel_name(p, 0) in ("ogc_cluster_chain_kernel<2>", "ogc_cluster_ksplit_chain_kernel<2>")
    assert b.ogc_mlp_workspace_bytes(p) == 2 * 256 * 1024 and b.ogc_mlp_num_launches(p) == 1
    # packed weights: K padded to 64 (479 -> 512), rows padded to 32/64; per-channel params on top
    assert b.ogc_mlp_packed_bytes(p) >= 512 * 1024 + 1024 * 1024 + 1024 * 512 + 512 * 256 + 256 * 32
    assert b.ogc_mlp_packed_bytes(p) < 1.1 * (512 * 1024 + 1024 * 1024 + 1024 * 512 + 512 * 256 + 256 * 64) + 5 * 3 * 4096
    b.ogc_mlp_destroy(p)
    # a narrow chain (config 2's shape): the fused chain kernel, no workspace
    dims2 = [13, 512, 256, 128, 64]
    p = b.ogc_mlp_plan(b.OGC_BF16, 128, [layer(dims2[i], dims2[i + 1]) for i in range(4)], 13, 64, 0, 0)
    assert b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_FUSED
    assert b.ogc_mlp_workspace_bytes(p) == 0 and b.ogc_mlp_num_launches(p) == 1
    b.ogc_mlp_destroy(p)
    # config 5 shape: large batch, wide layers -> per-layer kernels
    p = b.ogc_mlp_plan(b.OGC_I8, 32768, [layer(1024, 1024, has_bias=0)] * 4, 1024, 1024, 0, 0)
    assert b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_PER_LAYER and b.ogc_mlp_num_launches(p) == 4
    assert b.ogc_mlp_kernel_name(p, 0)
    b.ogc_mlp_destroy(p)


def test_cluster_split_override():
    """The cluster_split override picks the cooperative mode's kernel: 0 = blocks dealt to all workgroups, n = n
    workgroups per row tile, where they fit one per CU; unset = the cost model's choice."""
    dims = [479, 1024, 1024, 512, 256]
    ls = [layer(dims[i], dims[i + 1]) for i in range(4)]

    narrow = [layer(256, 512), layer(512, 256)]  # fp32 rows of 1024 values do not fit the two LDS buffers

    ov = {}

    def name(m, dtype=b.OGC_I8):
        p = b.ogc_mlp_plan_with_overrides(dtype, m, narrow if dtype == b.OGC_F32 else ls, 256 if dtype == b.OGC_F32 else 479, 256, 0,
                                          b.OGC_MODE_COOP, overrides=ov)
        n = b.ogc_mlp_kernel_name(p, 0)
        b.ogc_mlp_destroy(p)
        return n

    ov["cluster_split"] = 0
    assert name(256) == "ogc_coop_chain_kernel<2>"
    ov["cluster_split"] = 4
    assert name(256) == "ogc_cluster_chain_kernel<2>"
    assert name(256, b.OGC_F32) == "ogc_cluster_chain_kernel<0>"
    assert name(32 * 65) == "ogc_coop_chain_kernel<2>"      # 65 tiles x 4 members do not fit 256 CUs
    # the variant whose waves split K inside a member
    ov["cluster_ksplit"] = 1
    assert name(256) == "ogc_cluster_ksplit_chain_kernel<2>"
    assert name(256, b.OGC_F32) == "ogc_cluster_ksplit_chain_kernel<0>"
    assert name(32 * 65) == "ogc_coop_chain_kernel<2>"
    # unset: the cost model's choice; cluster_ksplit = 0 keeps the k-split variant out of it
    del ov["cluster_split"]
    ov["cluster_ksplit"] = 0
    assert name(256) == "ogc_cluster_chain_kernel<2>"
    assert name(256, b.OGC_F32) == "ogc_coop_chain_kernel<0>"  # the channel-split kernel is never the model's choice for fp32
    del ov["cluster_ksplit"]
    assert name(256).startswith("ogc_cluster_")
    assert name(256, b.OGC_F32) == "ogc_cluster_ksplit_chain_kernel<0>"
    # a field outside its range is refused; the process environment plays no part in a plan
    with pytest.raises(b.OgcError):
        b.ogc_mlp_plan_with_overrides(b.OGC_I8, 256, ls, 479, 256, 0, b.OGC_MODE_COOP, overrides={"tile": 7})


def test_cooperative_estimate_is_the_lowest_of_its_kernels():
    """ogc_mlp_mode_estimates()[2] is the estimate of the kernel the cooperative mode would launch: never above the
    block-dealing kernel's own estimate (what cluster_split = 0 leaves), equal to it where no cluster kernel fits."""
    def coop_est(dtype, m, dims, ov=None):
        p = b.ogc_mlp_plan_with_overrides(dtype, m, [layer(dims[i], dims[i + 1]) for i in range(len(dims) - 1)], dims[0], dims[-1], 0, 0,
                                          overrides=ov)
        e, name = b.ogc_mlp_mode_estimates(p)[2], b.ogc_mlp_kernel_name(p, 0) if b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_COOP else ""
        b.ogc_mlp_destroy(p)
        return e, name
    cases = [(b.OGC_I8, 256, [479, 1024, 1024, 512, 256]), (b.OGC_F32, 512, [479, 1024, 1024, 512, 256]),
             (b.OGC_BF16, 128, [1024, 1024, 1024]), (b.OGC_I8, 64, [64, 64, 64]), (b.OGC_F32, 32 * 300, [512, 512, 512])]
    for dtype, m, dims in cases:
        base, _ = coop_est(dtype, m, dims, {"cluster_split": 0})
        best, name = coop_est(dtype, m, dims)
        assert 0 < best <= base
        if m > 32 * 128:                      # 300 row tiles: no cluster kernel has a CU for every member
            assert best == base and "cluster" not in name
        if name.startswith("ogc_cluster"):
            assert best < base


def test_cluster_exchange_regions_are_private_per_tile():
    """The members of a row tile are synchronised only among themselves, so two tiles may be layers apart: for every
    pair of exchanged layers that share a workspace slot, the regions of DISTINCT tiles must be disjoint whatever the
    layers' widths, consecutive exchanged layers must sit in different slots, and everything must fit the workspace."""
    def regions(dtype, m, dims, ov):
        ls = [layer(dims[i], dims[i + 1]) for i in range(len(dims) - 1)]
        p = b.ogc_mlp_plan_with_overrides(dtype, m, ls, dims[0], dims[-1], 0, b.OGC_MODE_COOP, overrides=ov)
        members, ksplit, whole, stride = b.ogc_mlp_cluster_layout(p)
        assert members == ov["cluster_split"] and ksplit == ov.get("cluster_ksplit", 0)
        esz = {b.OGC_F32: 4, b.OGC_BF16: 2, b.OGC_I8: 1}[dtype]
        gran = 64 if dtype == b.OGC_I8 else 32
        tiles = (m + 31) // 32
        out = []   # (layer, slot, [(start, end) per tile])
        for l in range(len(ls) - 1):
            slot, off = b.ogc_mlp_buffer_assignment(p, l)
            if (whole >> l) & 1:
                assert slot == -1
                continue
            row_block = 32 * ((dims[l + 1] + gran - 1) // gran * gran) * esz    # one tile's rows of the next layer's input
            assert row_block <= stride
            out.append((l, slot, [(off + t * stride, off + t * stride + row_block) for t in range(tiles)]))
        ws = b.ogc_mlp_workspace_bytes(p)
        b.ogc_mlp_destroy(p)
        return out, ws, whole

    cases = [(b.OGC_I8, 256, [479, 1024, 1024, 512, 256, 1], {"cluster_split": 32, "cluster_ksplit": 1}),   # config 3's launch
             (b.OGC_I8, 256, [479, 1024, 1024, 512, 256, 1], {"cluster_split": 4}),                          # one layer computed whole
             (b.OGC_I8, 256, [479, 1024, 1024, 512, 256, 1], {"cluster_split": 4, "cluster_whole": 0}),
             (b.OGC_BF16, 270, [48, 64, 320, 64, 320, 16], {"cluster_split": 8, "cluster_whole": 0}),
             (b.OGC_F32, 200, [100, 333, 72, 33], {"cluster_split": 16, "cluster_ksplit": 1})]
    saw_whole = False
    for dtype, m, dims, ov in cases:
        regs, ws, whole = regions(dtype, m, dims, ov)
        saw_whole |= whole != 0
        assert regs, "no exchanged layer"
        for i, (l, slot, iv) in enumerate(regs):
            assert slot in (0, 1) and all(e <= ws for _, e in iv)
            if i > 0:
                assert slot != regs[i - 1][1]           # consecutive exchanges alternate (also across whole layers)
            for l2, slot2, iv2 in regs[:i + 1]:
                if slot2 != slot:
                    assert all(e <= iv2[0][0] or s >= iv2[-1][1] for s, e in iv)   # the two slots do not overlap at all
                    continue
                for t, (s, e) in enumerate(iv):
                    for t2, (s2, e2) in enumerate(iv2):
                        if t != t2:
                            assert e <= s2 or e2 <= s, (l, l2, t, t2)
    assert saw_whole


def test_check_without_waits_and_test_hook_arguments():
    """ogc_mlp_check answers OGC_OK at once for plans whose kernels have no bounded waits (no device call, so it runs
    here); the barrier test hook validates its arguments."""
    p = b.ogc_mlp_plan(b.OGC_I8, 64, [layer(64, 64)], 64, 64, 0, b.OGC_MODE_FUSED)
    assert b.ogc_mlp_check(p, 256, 0) == b.OGC_OK
    with pytest.raises(b.OgcError):
        b.ogc_mlp_check(0, 256, 0)
    with pytest.raises(b.OgcError):
        b.ogc_mlp_check(p, 0, 0)
    b.ogc_mlp_test_barrier(p, 100, 1)
    for bad in ((0, 0), (10, -1)):
        with pytest.raises(b.OgcError):
            b.ogc_mlp_test_barrier(p, *bad)
    b.ogc_mlp_destroy(p)
    assert "gave up" in b.status_string(b.OGC_ERR_TIMEOUT)


def test_buffer_reuse_is_ping_pong_for_a_chain():
    """Life-span reuse: layer l's output may take the buffer of layer l-2's output (dead once layer l-1 has
    run), never that of layer l-1's (live as the input).  Peak = two slots of the largest intermediate."""
    m = 1000
    dims = [64, 256, 512, 128, 1024, 64]
    p = b.ogc_mlp_plan(b.OGC_I8, m, [layer(dims[i], dims[i + 1]) for i in range(5)], 64, 64, 0, b.OGC_MODE_PER_LAYER)
    slots = [b.ogc_mlp_buffer_assignment(p, l) for l in range(5)]
    assert [s for s, _ in slots] == [0, 1, 0, 1, -1]
    for l in range(1, 4):
        assert slots[l][0] != slots[l - 1][0]
    mp = (m + 255) // 256 * 256
    sizes = [mp * dims[l + 1] for l in range(4)]
    want = max(sizes[0], sizes[2]) + max(sizes[1], sizes[3])
    assert b.ogc_mlp_workspace_bytes(p) == want
    assert slots[0][1] == 0 and slots[1][1] == max(sizes[0], sizes[2])
    with pytest.raises(b.OgcError):
        b.ogc_mlp_buffer_assignment(p, 5)
    b.ogc_mlp_destroy(p)
    # two layers: one slot; one layer: none
    p = b.ogc_mlp_plan(b.OGC_BF16, 64, [layer(32, 64), layer(64, 32)], 32, 32, 0, b.OGC_MODE_PER_LAYER)
    assert b.ogc_mlp_workspace_bytes(p) == 256 * 64 * 2
    b.ogc_mlp_destroy(p)
    p = b.ogc_mlp_plan(b.OGC_F32, 64, [layer(32, 64)], 32, 64, 0, b.OGC_MODE_PER_LAYER)
    assert b.ogc_mlp_workspace_bytes(p) == 0
    b.ogc_mlp_destroy(p)


def test_split_k_plan_sizes_and_kernel_names():
    """A layer with few 256x256 tiles and a long reduction axis takes k-slicing (Section III): by the model's own
    choice the eight waves of a 128x128 tile split the k-steps between them and add up on chip; a forced split-K
    cuts the axis into ranges computed by different workgroups, and the workspace then carries the partial
    accumulators behind the activation slots.  Either way the layer is one launch step, and kernel names carry
    their template arguments."""
    m, k0, hid = 4096, 1024, 4096
    lay = [layer(k0, hid, act=b.OGC_ACT_GELU_TANH, has_bias=1), layer(hid, k0, act=b.OGC_ACT_NONE, has_bias=1)]
    p = b.ogc_mlp_plan(b.OGC_BF16, m, lay, k0, k0, 1, b.OGC_MODE_AUTO)
    assert b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_PER_LAYER
    assert b.ogc_mlp_num_launches(p) == 2
    hidden_slot = m * hid * 2
    assert b.ogc_mlp_workspace_bytes(p) == hidden_slot
    assert b.ogc_mlp_kernel_name(p, 0) == "ogc_layer_dma_kernel<1, 1, 1, 0, 0>"
    assert b.ogc_mlp_kernel_name(p, 1) == "ogc_layer_dma_kernel<1, 2, 0, 1, 0>"
    # the figures the choice was made by: the estimate of the chosen candidate, in microseconds
    assert 25.0 < b.ogc_mlp_estimated_us(p, 0) < 45.0 and 30.0 < b.ogc_mlp_estimated_us(p, 1) < 50.0
    b.ogc_mlp_destroy(p)
    # forced: two ranges per layer on the four-wave stream shape, fp32 accumulators of both layers' ranges behind the slot
    p = b.ogc_mlp_plan_with_overrides(b.OGC_BF16, m, lay, k0, k0, 1, b.OGC_MODE_AUTO, overrides={"tile": 3, "ksplit_log2": 1})
    assert b.ogc_mlp_workspace_bytes(p) == hidden_slot + 2 * m * hid * 4
    assert b.ogc_mlp_kernel_name(p, 0) == "ogc_layer_dma_kernel<1, 0, 1, 0, 2>"
    assert b.ogc_mlp_kernel_name(p, 1) == "ogc_layer_dma_kernel<1, 0, 0, 0, 2>"
    assert b.ogc_mlp_estimated_us(p, 1) > 45.0
    b.ogc_mlp_destroy(p)
    # the k-sliced shape needs an even number of k-steps: forced where it cannot run, the plan falls back
    p = b.ogc_mlp_plan_with_overrides(b.OGC_I8, 300, [layer(64 * 3, 64)], 192, 64, 0, b.OGC_MODE_PER_LAYER, overrides={"tile": 5})
    assert "dma" not in b.ogc_mlp_kernel_name(p, 0)
    b.ogc_mlp_destroy(p)
    # a forced split that does not divide the k-steps is ignored
    p = b.ogc_mlp_plan_with_overrides(b.OGC_I8, 300, [layer(64 * 4, 64)], 256, 64, 0, b.OGC_MODE_PER_LAYER,
                                      overrides={"tile": 4, "ksplit_log2": 3})   # 4 k-steps
    assert b.ogc_mlp_workspace_bytes(p) == 0
    b.ogc_mlp_destroy(p)
    p = b.ogc_mlp_plan_with_overrides(b.OGC_I8, 300, [layer(64 * 4, 64)], 256, 64, 0, b.OGC_MODE_PER_LAYER,
                                      overrides={"tile": 4, "ksplit_log2": 2})
    assert b.ogc_mlp_workspace_bytes(p) == 4 * 512 * 256 * 4      # ranges x padded rows x padded channels x 4 bytes
    b.ogc_mlp_destroy(p)


def test_blocked_layout_plan():
    """Blocked x / y at the boundary: sizes, the forced per-layer mode, and what is refused."""
    lay = [layer(100, 72), layer(72, 40)]
    p = b.ogc_mlp_plan(b.OGC_I8, 300, lay, 100, 40, 0, b.OGC_MODE_AUTO, b.OGC_LAYOUT_BLOCKED, b.OGC_LAYOUT_BLOCKED)
    assert b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_PER_LAYER      # small enough for the fused kernel, but blocked
    assert b.ogc_mlp_blocked_bytes(p, 0) == 512 * 128            # rows to 256, 100 u8 columns to 128
    assert b.ogc_mlp_blocked_bytes(p, 1) == 512 * 64
    with pytest.raises(b.OgcError):
        b.ogc_mlp_blocked_bytes(p, 2)
    b.ogc_mlp_destroy(p)
    p = b.ogc_mlp_plan(b.OGC_BF16, 10, [layer(33, 17)], 33, 17, 0, b.OGC_MODE_PER_LAYER, 0, b.OGC_LAYOUT_BLOCKED)
    assert b.ogc_mlp_blocked_bytes(p, 0) == 0 and b.ogc_mlp_blocked_bytes(p, 1) == 256 * 32 * 2
    b.ogc_mlp_destroy(p)
    for kw, status in (
            (dict(mode=b.OGC_MODE_FUSED, x_layout=1), -2),
            (dict(mode=b.OGC_MODE_FUSED, y_layout=1), -2),
            (dict(x_layout=2), -1),
            (dict(y_layout=-1), -1)):
        with pytest.raises(b.OgcError) as e:
            b.ogc_mlp_plan(b.OGC_I8, 64, lay, 100, 40, 0, kw.get("mode", 0), kw.get("x_layout", 0), kw.get("y_layout", 0))
        assert e.value.status == status, kw
    with pytest.raises(b.OgcError) as e:      # the residual is read from a plain x
        b.ogc_mlp_plan(b.OGC_BF16, 64, [layer(40, 40)], 40, 40, 1, 0, b.OGC_LAYOUT_BLOCKED, 0)
    assert e.value.status == -2
    with pytest.raises(b.OgcError) as e:      # an fp32 result is a plain tensor
        b.ogc_mlp_plan(b.OGC_I8, 64, [layer(40, 8, out=b.OGC_OUT_F32)], 40, 8, 0, 0, 0, b.OGC_LAYOUT_BLOCKED)
    assert e.value.status == -1
    # strides of a blocked tensor are ignored
    p = b.ogc_mlp_plan(b.OGC_F32, 64, [layer(40, 8)], 0, 0, 0, 0, b.OGC_LAYOUT_BLOCKED, b.OGC_LAYOUT_BLOCKED)
    assert b.ogc_mlp_blocked_bytes(p, 0) == 256 * 64 * 4 and b.ogc_mlp_blocked_bytes(p, 1) == 256 * 32 * 4
    b.ogc_mlp_destroy(p)


def test_auto_mode_choice_follows_the_cost_models():
    """OGC_MODE_AUTO takes the mode whose fitted model gives the lowest estimate for the chain (a single-launch
    mode wins near ties).  Checked on shapes whose fastest mode was measured."""
    def mode(dtype, m, dims, **kw):
        lay = [layer(dims[i], dims[i + 1], **kw) for i in range(len(dims) - 1)]
        p = b.ogc_mlp_plan(dtype, m, lay, dims[0], dims[-1], 0, b.OGC_MODE_AUTO)
        r = b.ogc_mlp_chosen_mode(p)
        est = b.ogc_mlp_mode_estimates(p)
        b.ogc_mlp_destroy(p)
        assert est[r - 1] > 0 and all(e < 0 or e >= est[r - 1] / 1.07 for e in est)
        return r
    mlp1, mlp2 = [13, 512, 256, 128], [479, 1024, 1024, 512, 256, 1]
    assert mode(b.OGC_F32, 32, [13, 64, 32, 16]) == b.OGC_MODE_FUSED                   # config 1
    assert mode(b.OGC_BF16, 128, [13, 512, 256, 128, 64]) == b.OGC_MODE_FUSED          # config 2
    assert mode(b.OGC_I8, 256, mlp2) == b.OGC_MODE_COOP                                # config 3 (cluster kernel)
    assert mode(b.OGC_BF16, 4096, [1024, 4096, 1024]) == b.OGC_MODE_PER_LAYER          # config 4
    assert mode(b.OGC_I8, 32768, [1024] * 5) == b.OGC_MODE_PER_LAYER                   # config 5
    assert mode(b.OGC_F32, 64, mlp1) == b.OGC_MODE_COOP and mode(b.OGC_F32, 8192, mlp1) == b.OGC_MODE_FUSED
    assert mode(b.OGC_F32, 512, mlp2) == b.OGC_MODE_COOP and mode(b.OGC_F32, 8192, mlp2) == b.OGC_MODE_PER_LAYER
    # 2048 rows of MLP-2: four workgroups per row tile (measured 48 us bf16, 29 us int8) beat a launch per layer (63)
    # and the fused kernel (34.5, int8 only)
    assert mode(b.OGC_BF16, 128, mlp2) == b.OGC_MODE_COOP and mode(b.OGC_BF16, 2048, mlp2) == b.OGC_MODE_COOP
    assert mode(b.OGC_I8, 32, mlp2) == b.OGC_MODE_COOP and mode(b.OGC_I8, 2048, mlp2) == b.OGC_MODE_COOP
    assert mode(b.OGC_BF16, 8192, mlp2) == b.OGC_MODE_PER_LAYER
    assert mode(b.OGC_I8, 64, mlp1) == b.OGC_MODE_FUSED
    # wide int8 layers at a small batch: every CU on each layer beats one launch per layer (measured 33 against 51 us)
    assert mode(b.OGC_I8, 128, [2048] * 4) == b.OGC_MODE_COOP and mode(b.OGC_I8, 2048, [2048] * 4) == b.OGC_MODE_PER_LAYER
    # a bf16 chain whose weights exceed what the fused kernel streams well is not offered to it
    p = b.ogc_mlp_plan(b.OGC_BF16, 64, [layer(1024, 1024), layer(1024, 1024)], 1024, 1024, 0, b.OGC_MODE_AUTO)
    assert b.ogc_mlp_mode_estimates(p)[1] == -1.0 and b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_COOP
    b.ogc_mlp_destroy(p)
    # the cooperative kernel is never chosen for blocked tensors, and refuses them when asked for
    p = b.ogc_mlp_plan(b.OGC_F32, 64, [layer(512, 512), layer(512, 512)], 512, 512, 0, b.OGC_MODE_AUTO, 0, b.OGC_LAYOUT_BLOCKED)
    assert b.ogc_mlp_chosen_mode(p) == b.OGC_MODE_PER_LAYER
    b.ogc_mlp_destroy(p)
    with pytest.raises(b.OgcError) as e:
        b.ogc_mlp_plan(b.OGC_F32, 64, [layer(512, 512)], 512, 512, 0, b.OGC_MODE_COOP, b.OGC_LAYOUT_BLOCKED, 0)
    assert e.value.status == -2
    # one launch step, workspace slots as in per-layer mode, the barrier counters behind the packed parameters
    lay = [layer(64, 256), layer(256, 512), layer(512, 64)]
    pc = b.ogc_mlp_plan(b.OGC_I8, 100, lay, 64, 64, 0, b.OGC_MODE_COOP)
    pl = b.ogc_mlp_plan(b.OGC_I8, 100, lay, 64, 64, 0, b.OGC_MODE_FUSED)
    assert b.ogc_mlp_num_launches(pc) == 1 and b.ogc_mlp_kernel_name(pc, 0) in (
        "ogc_coop_chain_kernel<2>", "ogc_cluster_chain_kernel<2>", "ogc_cluster_ksplit_chain_kernel<2>")
    members, _, whole, stride = b.ogc_mlp_cluster_layout(pc)
    if members:   # a cluster kernel: two slots (one if a single layer is exchanged) of a private region per row tile
        exchanged = 2 - bin(whole & 3).count("1")
        assert stride >= 32 * 512 and b.ogc_mlp_workspace_bytes(pc) == min(exchanged, 2) * 4 * stride
    else:
        assert b.ogc_mlp_workspace_bytes(pc) == 256 * 256 + 256 * 512
    assert b.ogc_mlp_packed_bytes(pc) == b.ogc_mlp_packed_bytes(pl) + 2048 * 8
    b.ogc_mlp_destroy(pc)
    b.ogc_mlp_destroy(pl)


# ---- attention subgraph: description checks (host only) ---------------------------------------------------------
@pytest.mark.parametrize("kw,status", [
    (dict(), 0),
    (dict(dtype=b.OGC_BF16, head_dim=96), 0),
    (dict(dtype=7), -1),
    (dict(softmax=2), -1),
    (dict(scale=float("inf")), -1),
    (dict(seq=0), -3),
    (dict(batch=-1), -3),
    (dict(batch=4096, heads=16), -3),
    (dict(seq=65537), -3),
    (dict(dtype=b.OGC_I8), -2),
    (dict(head_dim=80), -2),
    (dict(head_dim=256), -2),
    (dict(q_stride=(1000, 64, 130)), -4),       # 130 fp32 elements: not a multiple of 16 bytes
    (dict(o_stride=(-1024, 64, 128)), -4),
])
def test_mha_validate(kw, status):
    args = dict(dtype=b.OGC_F32, batch=2, heads=2, seq=128, head_dim=64, scale=0.125)
    args.update(kw)
    assert b.ogc_mha_validate(b.mha_desc(**args)) == status


def test_mha_kernel_names_and_null_checks():
    d = b.mha_desc(b.OGC_BF16, 2, 8, 128, 96, 0.1, b.OGC_SOFTMAX_FAST)
    assert b.ogc_mha_kernel_name(d) == "ogc_mha_kernel<1, 3, 1, 0, 1>"
    assert b.ogc_mha_kernel_name(d, has_mask=False) == "ogc_mha_kernel<1, 3, 1, 1, 1>"
    assert b.ogc_mha_kernel_name(b.mha_desc(b.OGC_F32, 2, 8, 128, 64, 0.1)) == "ogc_mha_kernel<0, 2, 0, 0, 1>"
    # the variant without per-key addends needs whole key blocks (bf16: 64 keys) and a positive scale
    assert b.ogc_mha_kernel_name(b.mha_desc(b.OGC_BF16, 2, 8, 96, 64, 0.1), False) == "ogc_mha_kernel<1, 2, 0, 0, 1>"
    assert b.ogc_mha_kernel_name(b.mha_desc(b.OGC_F32, 2, 8, 96, 64, 0.1), False) == "ogc_mha_kernel<0, 2, 0, 1, 1>"
    assert b.ogc_mha_kernel_name(b.mha_desc(b.OGC_F32, 2, 8, 96, 64, -0.1), False) == "ogc_mha_kernel<0, 2, 0, 0, 1>"
    # bf16 with head_dim <= 64 and a sequence of 256 or more: two 32-query groups per wavefront
    assert b.ogc_mha_kernel_name(b.mha_desc(b.OGC_BF16, 2, 8, 512, 64, 0.1)) == "ogc_mha_kernel<1, 2, 0, 0, 2>"
    assert b.ogc_mha_kernel_name(b.mha_desc(b.OGC_BF16, 2, 8, 512, 128, 0.1)) == "ogc_mha_kernel<1, 4, 0, 0, 1>"
    assert b.ogc_mha_kernel_name(b.mha_desc(b.OGC_F32, 2, 8, 128, 70, 0.1)) == ""
    assert b.lib().ogc_mha_validate(None) == -1
    # argument checks come before any device call: NULL tensors and misaligned bases are refused on the host
    with pytest.raises(b.OgcError) as e:
        b.ogc_mha_run(d, 0, 256, 256, 0, 256)
    assert e.value.status == -1
    with pytest.raises(b.OgcError) as e:
        b.ogc_mha_run(d, 256, 256, 264, 0, 256)
    assert e.value.status == -4


def test_cost_model_choices():
    """The plan's cost model (Section III: score candidate template parameters, no tuning run) on shapes whose
    fastest candidate was measured: big batches take the eight-wave stream tile, a short wide layer with a long
    reduction axis is cut along K on the four-wave tile, mid-size layers take the small register-staged tile."""
    def mid_layer(dtype, m, dims, ov=None):
        lay = [layer(dims[i], dims[i + 1], has_bias=0) for i in range(3)]
        p = b.ogc_mlp_plan_with_overrides(dtype, m, lay, dims[0], dims[3], 0, b.OGC_MODE_PER_LAYER, overrides=ov)
        r = b.ogc_mlp_kernel_name(p, 1), b.ogc_mlp_estimated_us(p, 1)
        b.ogc_mlp_destroy(p)
        return r

    assert mid_layer(b.OGC_I8, 32768, [1024] * 4)[0] == "ogc_layer_dma_kernel<2, 1, 0, 0, 1>"
    assert mid_layer(b.OGC_I8, 256, [256, 8192, 256, 8192])[0] == "ogc_layer_dma_kernel<2, 0, 0, 0, 2>"   # K = 8192, split
    assert mid_layer(b.OGC_BF16, 512, [1024, 4096, 1024, 4096])[0] == "ogc_layer_dma_kernel<1, 0, 0, 0, 2>"
    assert mid_layer(b.OGC_I8, 2048, [1024] * 4)[0] == "ogc_layer_kernel<2, 2, 0, 0>"
    # estimates grow with the batch once the chip is full, and a forced worse candidate is estimated slower
    e1, e2 = mid_layer(b.OGC_I8, 16384, [1024] * 4)[1], mid_layer(b.OGC_I8, 32768, [1024] * 4)[1]
    assert 0 < e1 < e2 < 2.5 * e1
    best = mid_layer(b.OGC_I8, 256, [256, 8192, 256, 8192])[1]
    assert mid_layer(b.OGC_I8, 256, [256, 8192, 256, 8192], {"tile": 4, "ksplit_log2": 0})[1] > 2 * best
    # fp32 layers choose among the register-staged tiles: the big one once the batch is large
    assert mid_layer(b.OGC_F32, 128, [512] * 4)[0] == "ogc_layer_kernel<0, 2, 0, 0>"
    assert mid_layer(b.OGC_F32, 16384, [2048] * 4)[0] == "ogc_layer_kernel<0, 0, 0, 0>"
    # a forced stream tile falls back to the mid register-staged tile where the stream kernel cannot run
    assert mid_layer(b.OGC_F32, 4096, [512] * 4, {"tile": 4})[0] == "ogc_layer_kernel<0, 1, 0, 0>"
