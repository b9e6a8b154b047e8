"""hyperattn_forward_static (the entry point that allocates nothing: its scratch
is an array built into the library) against hyperattn_forward on a caller-owned
workspace: same kernels, so outputs must agree bit for bit.  Two calls in a row,
the second on a smaller problem, so that whatever the first call left in the
shared array is seen by the second."""
import numpy as np
import pytest

import synth_inputs
from ha_testutil import have_gpu, to_device

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not have_gpu(), reason="needs a GPU")]


def _both(ha, cfg):
    import torch
    Q, K, V = (to_device(x, cfg["dtype"]) for x in synth_inputs.make_qkv(cfg))
    kw = dict(causal=bool(cfg["causal"]), n_min=cfg["n_min"], seed=cfg["seed"])
    ref_o, ref_l = ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], **kw)
    out = torch.full_like(Q, float("nan"))
    lse = torch.full(Q.shape[:3], float("nan"), dtype=torch.float32, device=Q.device)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ha.hyperattn_forward_static(Q, K, V, out, lse, cfg["b"], cfg["m"], cfg["r"], **kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out.view(torch.int16) if out.dtype == torch.bfloat16 else out,
                       ref_o.view(torch.int16) if ref_o.dtype == torch.bfloat16 else ref_o)
    assert torch.equal(lse, ref_l)


def test_static_scratch_forward_matches_workspace_forward():
    import paper_2310_05869_amd as ha
    ha.lib()
    big = dict(B=1, H=3, n=8192, d=128, dtype="bf16", law="iid", b=256, m=256, r=7, causal=1, n_min=1024, seed=3)
    small = dict(B=2, H=1, n=1536, d=64, dtype="bf16", law="iid", b=64, m=33, r=5, causal=0, n_min=4096, seed=9)
    f32 = dict(B=1, H=1, n=1024, d=64, dtype="fp32", law="iid", b=64, m=64, r=7, causal=0, n_min=4096, seed=0)
    for cfg in (big, small, f32, big):
        _both(ha, cfg)


def test_static_scratch_limit_is_an_error_not_a_launch():
    import torch
    import paper_2310_05869_amd as ha
    shape = ha.make_shape(1, 32, 131072, 128, ha.HA_BF16)
    params = ha.make_params(256, 256, 7, True, 4096, 0)
    assert ha.ha_workspace_bytes(shape, params) > ha.ha_static_scratch_bytes() == 32 << 20
    # pointers are never dereferenced: the size check comes first
    q = torch.empty(16, dtype=torch.bfloat16, device="cuda")
    l = torch.empty(16, dtype=torch.float32, device="cuda")
    st = ha.lib().hyperattn_forward_static(q.data_ptr(), q.data_ptr(), q.data_ptr(), q.data_ptr(), l.data_ptr(),
                                           shape, params, None)
    assert st == -7 and "hyperattn_forward" in ha.strerror(st)
