"""GPU test of the entry point that allocates nothing (spec_layer_forward_static): its output equals
spec_layer_forward's bit for bit (same kernels, workspace in the static scratch array), on two calls in
a row, the second with a smaller input; a workspace beyond the array is refused."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def test_static_scratch_layer_equals_workspace_layer():
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev, host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=1, n_q_heads=8, n_kv_heads=2)
    hm = host_model_pinned(shp, seed=3, std=0.05)
    n_new, ctx = 9, 70
    s = P.Session(hm, None, batch_max=7, k_max=n_new - 1, ctx_max=ctx + n_new + 2, page_tokens=32)
    try:
        for B in (7, 3):                                   # the second call is smaller and finds the first one's data
            x, kc, vc = synth.make_layer_inputs(shp, B, n_new, ctx, seed=10 + B)
            P.spec_kv_import(s.ctx, 0, 0, dev(kc), dev(vc), B, ctx)
            xd = dev(x)
            ref = torch.zeros((B * n_new, shp.d_model), dtype=torch.float32, device="cuda")
            got = torch.full((B * n_new, shp.d_model), float("nan"), dtype=torch.float32, device="cuda")
            P.spec_layer_forward(s.ctx, 0, 0, xd, n_new, ref)
            P.spec_layer_forward_static(s.ctx, 0, 0, xd, n_new, got)
            P.spec_sync(s.ctx, 0)
            a, b = ref.cpu().numpy(), got.cpu().numpy()
            assert np.isfinite(a).all() and np.abs(a).max() > 0.1
            assert np.array_equal(a, b), f"B={B}: max diff {np.abs(a - b).max()}"
    finally:
        s.close()


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev, host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=1)
    hm = host_model_pinned(shp, seed=3, std=0.05)
    B, n_new = 2048, 9                                     # 18432 rows x ~6 KB of workspace > 64 MiB
    s = P.Session(hm, None, batch_max=B, k_max=n_new - 1, ctx_max=16)
    try:
        P.spec_kv_import(s.ctx, 0, 0, None, None, B, 0)
        x = torch.zeros((B * n_new, shp.d_model), dtype=torch.bfloat16, device="cuda")
        out = torch.zeros((B * n_new, shp.d_model), dtype=torch.float32, device="cuda")
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_layer_forward_static(s.ctx, 0, 0, x, n_new, out)
        assert e.value.code == P.SPEC_ERR_CAPACITY and "static" in str(e.value)
        P.spec_layer_forward(s.ctx, 0, 0, x, n_new, out)  # the allocating sibling still takes it
        P.spec_sync(s.ctx, 0)
    finally:
        s.close()
