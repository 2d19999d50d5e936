"""The entry point that allocates nothing (ogc_mlp_run_static) against ogc_mlp_run, through the C ABI: same kernels,
so every output byte must be identical; two calls in a row on the shared static workspace, the second on a smaller
input, and a plan beyond the static limit is refused."""
import numpy as np
import pytest

from paper_2301_01333_amd import binding, synth

pytestmark = pytest.mark.gpu

RELU, SIGM = synth.ACT_RELU, synth.ACT_SIGMOID


def _pair(wl, mode, overrides=None):
    """Runs the chain through ogc_mlp_run (caller's workspace) and through ogc_mlp_run_static; returns both outputs."""
    import torch

    from paper_2301_01333_amd.harness import DeviceMLP

    d = DeviceMLP(wl, mode, overrides=overrides)
    assert 0 < d.mlp.workspace_bytes <= binding.ogc_mlp_static_workspace_limit()
    d.run()
    want = d.result().copy()
    assert d.mlp.check() == binding.OGC_OK
    d.y.fill_(0xCD)
    d.mlp.workspace.fill_(0xEE)          # the caller's workspace must play no part in the static call
    before = torch.cuda.memory_allocated()
    stream = int(torch.cuda.current_stream().cuda_stream)
    binding.ogc_mlp_run_static(d.mlp.plan, d.x.data_ptr(), d.y.data_ptr(), d.mlp.packed.data_ptr(), stream)
    got = d.result().copy()
    assert d.mlp.check() == binding.OGC_OK
    assert torch.cuda.memory_allocated() == before
    assert (d.mlp.workspace == 0xEE).all().item()
    d.close()
    return got, want


@pytest.mark.parametrize("mode,ov", [(binding.OGC_MODE_PER_LAYER, None), (binding.OGC_MODE_PER_LAYER, {"tile": 3, "ksplit_log2": 1}),
                                     (binding.OGC_MODE_COOP, {"cluster_split": 0}), (binding.OGC_MODE_COOP, {"cluster_split": 4, "cluster_whole": 0})])
def test_static_workspace_matches_the_callers_workspace(oracle_mod, mode, ov):
    dims = [479, 1024, 1024, 512, 256, 1]
    acts = [RELU] * 4 + [SIGM]
    for m in (256, 77):                  # two calls in a row on the shared array, the second on a smaller input
        wl = synth.make_mlp("i8", m, dims, acts, seed=77, last_f32=True, name="static-workspace")
        print("case: static workspace, M=%d mode=%d overrides=%s" % (m, mode, ov), flush=True)
        got, want = _pair(wl, mode, ov)
        assert np.array_equal(got.view(np.uint8), want.view(np.uint8))
        ref = oracle_mod.mlp(wl)
        assert np.abs(got[:, :1].astype(np.float64) - ref).max() <= 1e-5 * (1.0 + np.abs(ref).max())
    for dtype in ("bf16", "f32"):
        for m in (300, 100):
            wl = synth.make_mlp(dtype, m, [100, 333, 72, 33], [RELU, RELU, RELU], seed=601, name="static-workspace")
            got, want = _pair(wl, mode, ov if mode == binding.OGC_MODE_COOP else None)
            assert np.array_equal(got.view(np.uint8), want.view(np.uint8))


def test_static_workspace_refuses_what_does_not_fit():
    import torch

    wl = synth.make_config(5, m=32768)
    lay = [dict(k=l.k, n=l.n, has_bias=int(l.has_bias), act=l.act, in_scale=l.in_scale, in_zp=l.in_zp, out_scale=l.out_scale,
                out_zp=l.out_zp) for l in wl.layers]
    p = binding.ogc_mlp_plan(binding.OGC_I8, wl.m, lay, 1024, 1024, 0, binding.OGC_MODE_PER_LAYER)
    assert binding.ogc_mlp_workspace_bytes(p) > binding.ogc_mlp_static_workspace_limit()
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.OgcError) as e:
        binding.ogc_mlp_run_static(p, buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), 0)
    assert e.value.status == -5
    binding.ogc_mlp_destroy(p)
