"""The entry point that allocates nothing (moesd_moe_forward_static: scratch in a static device array of
the library) against moesd_moe_forward with a caller's workspace, through the C ABI: two calls in a row on
the same GPU, the second with a smaller batch, so the array still holds the first call's contents."""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2505_19645_amd import synth
from paper_2505_19645_amd.synth import LayerShape


def _static_forward(gpu, layer, x_np):
    import torch
    import paper_2505_19645_amd as moesd
    s, T = layer.shape, x_np.shape[0]
    K, E, d = s.top_k, s.E, s.d
    dev = gpu.DEV
    x = gpu.to_dev_bf16(x_np)
    out = torch.full((T, d), 0x7FC0, dtype=torch.int16, device=dev)
    out32 = torch.full((T, d), float("nan"), dtype=torch.float32, device=dev)
    ids = torch.full((T, K), -1, dtype=torch.int32, device=dev)
    w = torch.full((T, K), float("nan"), dtype=torch.float32, device=dev)
    counts = torch.full((E,), -1, dtype=torch.int32, device=dev)
    offsets = torch.full((E + 1,), -1, dtype=torch.int32, device=dev)
    perm = torch.full((T * K,), -1, dtype=torch.int32, device=dev)
    inv = torch.full((T * K,), -1, dtype=torch.int32, device=dev)
    na = torch.full((1,), -1, dtype=torch.int32, device=dev)
    moesd.moesd_moe_forward_static(layer.desc, layer.weights, x, T, out, out_f32=out32, topk_ids=ids, topk_w=w,
                                   counts=counts, offsets=offsets, perm=perm, inv_perm=inv, n_active=na)
    torch.cuda.synchronize()
    return dict(out_bf16=out.cpu().numpy().view(np.uint16), out_f32=out32.cpu().numpy(), ids=ids.cpu().numpy(),
                w=w.cpu().numpy(), counts=counts.cpu().numpy(), offsets=offsets.cpu().numpy(),
                perm=perm.cpu().numpy(), inv=inv.cpu().numpy(), n_active=int(na.item()))


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2505_19645_amd as moesd
    from paper_2505_19645_amd import binding
    from tests import gpu_harness as gpu
    # shared expert with a gate, ragged sizes, softmax routing; 2.5 MB of scratch at T = 64
    shape = LayerShape("static-scratch", d=1032, E=40, top_k=6, inter=520, shared_inter=776, shared_gate=1, seed=91)
    layer = gpu.GpuLayer(shape, synth.make_layer(shape))
    for T, point in ((64, 1), (5, 2)):   # the second, smaller call finds the first one's contents in the array
        print(f"[case] static scratch T={T}", flush=True)
        sys.stdout.flush()
        assert 0 < moesd.moesd_workspace_bytes(layer.desc, T) <= binding.STATIC_SCRATCH_BYTES
        x = synth.make_tokens(shape, T, point=point)
        want = layer.forward(x)
        got = _static_forward(gpu, layer, x)
        for k in ("ids", "counts", "offsets", "perm", "inv"):
            assert np.array_equal(want[k], got[k]), k
        assert want["n_active"] == got["n_active"]
        assert np.array_equal(want["w"], got["w"])
        # the same kernels on the same inputs: the same bits (within the output tolerance would do)
        assert np.array_equal(want["out_f32"], got["out_f32"])
        assert np.array_equal(want["out_bf16"], got["out_bf16"])
        assert not np.isnan(got["out_f32"]).any()
    # more tokens than the array can serve: refused, nothing enqueued
    big = synth.make_tokens(shape, 2000, point=3)
    xb = gpu.to_dev_bf16(big)
    ob = torch.zeros((2000, shape.d), dtype=torch.int16, device=gpu.DEV)
    assert moesd.moesd_workspace_bytes(layer.desc, 2000) > binding.STATIC_SCRATCH_BYTES
    st = moesd.moesd_moe_forward_static(layer.desc, layer.weights, xb, 2000, ob, check=False)
    assert st == binding.WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert int(ob.abs().sum().item()) == 0
