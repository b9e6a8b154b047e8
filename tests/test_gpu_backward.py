"""GPU parity of the backward pass: hyperattn_backward / exact_attn_backward
(through the C ABI) against the oracle's fp64 vector-Jacobian product on the
same seeded inputs, hash codes first (sign bits the GPU resolved differently on
a vanishing projection are replayed in the oracle, as in the forward tests).

Tolerance (derived from the arithmetic; the paper states none for gradients):
every term P_ij x or dS_ij x of a gradient element reaches the fp32 accumulator
with a relative error of at most 2^-8 (P or dS rounded to bf16 as matrix-core
operand: 2^-9; delta_i built from the bf16 output: 2^-9), the terms' errors are
independent, and the result is rounded to bf16 once more.  So the error of a
tensor is about 2^-9 .. 2^-8 of its size in the root-mean-square sense and a
few times that at its worst element:
    ||got - ref||_F <= 5e-3 ||ref||_F   and   max|got - ref| <= 1e-2 max|ref|
(measured: 2.3e-3 .. 2.6e-3 and 2e-3 .. 5e-3 when a row has hundreds of keys, up to 3.3e-3 and 7e-3 when it has
five and the operand roundings do not average out; rounding the fp64 result to bf16 alone gives 2.3e-3).
A dropped term, a wrong mask, sign or weight moves both by O(1)."""
import numpy as np
import pytest

import synth_inputs
from oracle import hyperattn_oracle as orc
from ha_testutil import compare_codes, have_gpu, to_device, to_host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not have_gpu(), reason="needs a GPU")]

FRO_TOL = 5e-3
MAX_TOL = 1e-2


@pytest.fixture(scope="module")
def ha():
    import paper_2310_05869_amd as mod
    mod.lib()
    return mod


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


def _assert_grad_close(got, ref, what):
    fro = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    mx = np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)
    print(f"  {what}: relative Frobenius error {fro:.2e}, worst element / max|ref| {mx:.2e}", flush=True)
    assert np.isfinite(got).all(), what
    assert fro <= FRO_TOL, (what, fro)
    assert mx <= MAX_TOL, (what, mx)


def _cotangent(shape, seed):
    g = np.random.default_rng(seed).standard_normal(shape).astype(np.float32)
    return synth_inputs.round_to_bf16(g)


def _run_case(ha, torch, cfg, seed_data=77):
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    Q, K, V = synth_inputs.make_qkv(cfg, seed=seed_data)
    G = _cotangent(Q.shape, seed_data + 1)
    dQ_, dK_, dV_, dG_ = (to_device(x, "bf16") for x in (Q, K, V, G))
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    kw = dict(causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"])
    out, lse = ha.hyperattn_forward(dQ_, dK_, dV_, cfg["b"], cfg["m"], cfg["r"], workspace=ws, **kw)
    gq, gk, gv = ha.hyperattn_backward(dQ_, dK_, dV_, out, lse, dG_, cfg["b"], cfg["m"], cfg["r"], fwd_workspace=ws, **kw)
    torch.cuda.synchronize()
    flips = []
    lay = ha.ha_workspace_layout(shape, params)
    if lay.levels > 0:
        views = ha.workspace_views(ws, shape, params)
        stages = {}
        orc.hyperattn_forward(Q, K, V, b=cfg["b"], m=cfg["m"], r=cfg["r"], causal=bool(cfg["causal"]),
                              n_min=cfg["n_min"], seed=cfg["seed"], stages=stages)
        gpu_codes = np.stack([views["codes_q"].cpu().numpy(), views["codes_k"].cpu().numpy()])
        flips = compare_codes(gpu_codes, stages, cfg["r"])
    rq, rk, rv = orc.hyperattn_backward(Q, K, V, G, b=cfg["b"], m=cfg["m"], r=cfg["r"], causal=bool(cfg["causal"]),
                                        n_min=cfg["n_min"], seed=cfg["seed"], flip=flips or None)
    _assert_grad_close(to_host(gq), rq, "dQ")
    _assert_grad_close(to_host(gk), rk, "dK")
    _assert_grad_close(to_host(gv), rv, "dV")
    return (gq, gk, gv), (dQ_, dK_, dV_, out, lse, dG_, ws)


@pytest.mark.parametrize("d,n,b,m", [(128, 2048, 256, 256), (64, 2048, 256, 512), (128, 1536, 128, 100),
                                     (64, 640, 64, 0), (128, 512, 512, 32), (64, 1024, 32, 16),
                                     (128, 8192, 256, 256)])
def test_backward_unmasked(ha, torch, d, n, b, m):
    print(f"backward unmasked d={d} n={n} b={b} m={m}", flush=True)
    cfg = dict(B=1, H=2, n=n, d=d, dtype="bf16", law="iid", b=b, m=m, r=7, causal=0, n_min=4096, seed=0)
    _run_case(ha, torch, cfg)


@pytest.mark.parametrize("d,n,n_min,b,m", [(128, 2048, 256, 128, 64), (64, 4096, 1024, 256, 256),
                                           (128, 1024, 4096, 256, 256), (128, 1024, 512, 512, 0),
                                           (64, 2048, 64, 32, 16), (128, 8192, 1024, 256, 256),
                                           (64, 8192, 32, 32, 16)])  # eight levels: more than the epilogue unrolls
def test_backward_causal(ha, torch, d, n, n_min, b, m):
    print(f"backward causal d={d} n={n} n_min={n_min} b={b} m={m}", flush=True)
    cfg = dict(B=2, H=1, n=n, d=d, dtype="bf16", law="iid", b=b, m=m, r=7, causal=1, n_min=n_min, seed=3)
    _run_case(ha, torch, cfg)


@pytest.mark.parametrize("d,n,causal", [(128, 300, False), (128, 300, True), (64, 1000, True), (64, 257, False)])
def test_exact_attn_backward(ha, torch, d, n, causal):
    print(f"exact backward d={d} n={n} causal={causal}", flush=True)
    cfg = dict(B=1, H=2, n=n, d=d, dtype="bf16", law="iid")
    Q, K, V = synth_inputs.make_qkv(cfg, seed=5)
    G = _cotangent(Q.shape, 6)
    tq, tk, tv, tg = (to_device(x, "bf16") for x in (Q, K, V, G))
    out, lse = ha.exact_attn_forward(tq, tk, tv, causal=causal)
    gq, gk, gv = ha.exact_attn_backward(tq, tk, tv, out, lse, tg, causal=causal)
    torch.cuda.synchronize()
    if causal:   # the recursion that never splits is exact causal attention
        ref = orc.hyperattn_backward(Q, K, V, G, b=1, m=0, r=1, causal=True, n_min=n)
    else:        # one block and no samples is exact attention
        ref = orc.hyperattn_backward(Q, K, V, G, b=n, m=0, r=1, causal=False)
    for got, r_, name in zip((gq, gk, gv), ref, ("dQ", "dK", "dV")):
        _assert_grad_close(to_host(got), r_, name)


def test_backward_is_deterministic_and_leaves_inputs_alone(ha, torch):
    print("backward determinism", flush=True)
    cfg = dict(B=1, H=2, n=2048, d=128, dtype="bf16", law="iid", b=128, m=128, r=7, causal=1, n_min=512, seed=1)
    (gq, gk, gv), (tq, tk, tv, out, lse, tg, ws) = _run_case(ha, torch, cfg)
    before = [t.clone() for t in (tq, tk, tv, out, lse, tg, ws)]
    kw = dict(causal=1, n_min=512, seed=1)
    gq2, gk2, gv2 = ha.hyperattn_backward(tq, tk, tv, out, lse, tg, 128, 128, 7, fwd_workspace=ws, **kw)
    torch.cuda.synchronize()
    for a_, b_ in zip((gq, gk, gv), (gq2, gk2, gv2)):
        assert torch.equal(a_.view(torch.int16), b_.view(torch.int16))
    for a_, b_ in zip(before, (tq, tk, tv, out, lse, tg, ws)):
        assert torch.equal(a_.view(torch.uint8) if a_.dtype != torch.uint8 else a_,
                           b_.view(torch.uint8) if b_.dtype != torch.uint8 else b_)


def test_backward_error_paths(ha, torch):
    print("backward errors", flush=True)
    q = torch.zeros((1, 1, 256, 64), dtype=torch.float32, device="cuda")
    shape = ha.make_shape(1, 1, 256, 64, ha.HA_FP32)
    params = ha.make_params(64, 16, 7, False, 4096, 0)
    with pytest.raises(ha.HyperAttnError):          # fp32 tensors: no backward path
        ha.ha_backward_workspace_bytes(shape, params)
    qb = q.to(torch.bfloat16)
    shape = ha.make_shape(1, 1, 256, 64, ha.HA_BF16)
    ws = ha.alloc_workspace(shape, params)
    out, lse = ha.hyperattn_forward(qb, qb, qb, 64, 16, 7, workspace=ws)
    small = torch.zeros(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(ha.HyperAttnError):          # backward workspace too small
        ha.hyperattn_backward(qb, qb, qb, out, lse, qb, 64, 16, 7, fwd_workspace=ws, bwd_workspace=small)
    with pytest.raises(ha.HyperAttnError):          # forward workspace too small
        ha.hyperattn_backward(qb, qb, qb, out, lse, qb, 64, 16, 7, fwd_workspace=small)


@pytest.mark.parametrize("name", ["cfg2_n32k", "cfg4_n131k_causal", "sweep_h12_d64_n65536_causal"])
def test_backward_full_size_sampled_head(ha, torch, name):
    """The benchmark configurations at full size: every head runs, head 0 of
    batch 0 (fed from the seeded host generator) is compared with the oracle."""
    cfg = synth_inputs.CONFIGS[name]
    print(f"backward full size {name}", flush=True)
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    host = synth_inputs.make_qkv(cfg, B=1, H=1)
    Gh = _cotangent(host[0].shape, 9)
    dev = []
    for i in range(4):
        t = torch.randn((B, H, n, d), generator=gen, device="cuda", dtype=torch.float32)
        if i < 3:
            t.mul_(d ** -0.25)
        t = t.to(torch.bfloat16)
        t[0, :1] = to_device((host[i] if i < 3 else Gh)[0], "bf16")
        dev.append(t.contiguous())
    Q, K, V, G = dev
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    kw = dict(causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"])
    out, lse = ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], workspace=ws, **kw)
    grads = ha.hyperattn_backward(Q, K, V, out, lse, G, cfg["b"], cfg["m"], cfg["r"], fwd_workspace=ws, **kw)
    torch.cuda.synchronize()
    views = ha.workspace_views(ws, shape, params)
    stages = {}
    okw = dict(b=cfg["b"], m=cfg["m"], r=cfg["r"], causal=bool(cfg["causal"]), n_min=cfg["n_min"], seed=cfg["seed"])
    orc.hyperattn_forward(*host, stages=stages, **okw)
    gpu_codes = np.stack([views["codes_q"][:1].cpu().numpy(), views["codes_k"][:1].cpu().numpy()])
    flips = compare_codes(gpu_codes, stages, cfg["r"])
    ref = orc.hyperattn_backward(*host, Gh, flip=flips or None, **okw)
    for got, r_, what in zip(grads, ref, ("dQ", "dK", "dV")):
        _assert_grad_close(to_host(got[0, :1])[None], r_, what)
        assert torch.isfinite(got.float()).all()


@pytest.mark.parametrize("n,n_min,b,m,causal", [(64, 4096, 1, 4, 0),      # blocks of one key
                                                (128, 8, 8, 20, 1),       # more samples than keys in the deep nodes
                                                (192, 4096, 96, 7, 0),    # block not a multiple of 64, odd m
                                                (96, 4096, 96, 96, 0)])   # a single block
def test_backward_degenerate_shapes(ha, torch, n, n_min, b, m, causal):
    print(f"backward degenerate n={n} n_min={n_min} b={b} m={m} causal={causal}", flush=True)
    cfg = dict(B=1, H=2, n=n, d=64, dtype="bf16", law="iid", b=b, m=m, r=4, causal=causal, n_min=n_min, seed=9)
    _run_case(ha, torch, cfg)


def test_backward_of_nothing(ha, torch):
    """Empty batches and empty sequences are accepted and touch nothing."""
    print("backward empty", flush=True)
    for shp in ((0, 2, 256, 64), (1, 2, 0, 64)):
        q = torch.zeros(shp, dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros(shp[:3], dtype=torch.float32, device="cuda")
        ws = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
        grads = ha.hyperattn_backward(q, q, q, q, lse, q, 64, 16, 7, fwd_workspace=ws, bwd_workspace=ws.clone())
        assert all(g.shape == q.shape for g in grads)
