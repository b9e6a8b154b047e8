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
A dropped term, a wrong mask, sign or weight moves both by O(1).

Peaked rows are the exception.  dS_ij = P_ij (<dO_i, v_j> - delta_i) with delta_i =
<dO_i, O_i> is a difference that cancels when a row's weight sits on few keys, and delta
inherits two errors of the forward: the rounding of the output to bf16 (avoided by
hyperattn_forward_train's fp32 copy, used here) and the rounding of the softmax weights
to bf16 as matrix operands (inherent to the forward; std of delta's error about
2^-9/sqrt(3) * sqrt(sum_j P_ij^2 <dO_i,v_j>^2)).  dQ_i and dK_j pick that error up times
sum_j P_ij k_j resp. q_i, with no small factor in front.  On the 64-centre mixture
(scores up to +-250) dQ is off by 1.2e-2 in the Frobenius sense (2.6e-2 with delta from
the bf16 output) and dK by 4e-3; that law is tested against 3e-2 / 5e-2, and the seeded
random cases avoid the regime (no m in 1..15, whose sample weight s/m puts a row's
weight on a handful of sampled keys).  dV carries no such difference and keeps the
tight bound everywhere."""
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


def _assert_grad_close(got, ref, what, fro_tol=FRO_TOL, max_tol=MAX_TOL):
    fro = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    mx = np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)
    print(f"  {what}: relative Frobenius error {fro:.2e}, worst element / max|ref| {mx:.2e}", flush=True)
    assert np.isfinite(got).all(), what
    assert fro <= fro_tol, (what, fro)
    assert mx <= max_tol, (what, mx)


def _cotangent(shape, seed):
    g = np.random.default_rng(seed).standard_normal(shape).astype(np.float32)
    return synth_inputs.round_to_bf16(g)


# Peaked rows (the mixture law): see the module docstring.
PEAKED_FRO_TOL = 3e-2
PEAKED_MAX_TOL = 5e-2


def _run_case(ha, torch, cfg, seed_data=77, peaked=False):
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    Q, K, V = synth_inputs.make_qkv(cfg, seed=seed_data)
    G = _cotangent(Q.shape, seed_data + 1)
    dQ_, dK_, dV_, dG_ = (to_device(x, "bf16") for x in (Q, K, V, G))
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    kw = dict(causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"])
    out32 = torch.empty(dQ_.shape, dtype=torch.float32, device="cuda")
    out, lse = ha.hyperattn_forward(dQ_, dK_, dV_, cfg["b"], cfg["m"], cfg["r"], workspace=ws, out_f32=out32, **kw)
    assert torch.equal(out32.to(torch.bfloat16).view(torch.int16), out.view(torch.int16))  # the copy rounds to the output
    gq, gk, gv = ha.hyperattn_backward(dQ_, dK_, dV_, out, lse, dG_, cfg["b"], cfg["m"], cfg["r"], fwd_workspace=ws,
                                       out_f32=out32, **kw)
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
    tols = (PEAKED_FRO_TOL, PEAKED_MAX_TOL) if peaked else (FRO_TOL, MAX_TOL)
    _assert_grad_close(to_host(gq), rq, "dQ", *tols)
    _assert_grad_close(to_host(gk), rk, "dK", *tols)
    _assert_grad_close(to_host(gv), rv, "dV")      # dV has no cancelling difference
    return (gq, gk, gv), (dQ_, dK_, dV_, out, lse, dG_, ws, out32)


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
    out32 = torch.empty(tq.shape, dtype=torch.float32, device="cuda")
    out, lse = ha.exact_attn_forward(tq, tk, tv, causal=causal, out_f32=out32)
    gq, gk, gv = ha.exact_attn_backward(tq, tk, tv, out, lse, tg, causal=causal, out_f32=out32)
    torch.cuda.synchronize()
    if causal:   # the recursion that never splits is exact causal attention
        ref = orc.hyperattn_backward(Q, K, V, G, b=1, m=0, r=1, causal=True, n_min=n)
    else:        # one block and no samples is exact attention
        ref = orc.hyperattn_backward(Q, K, V, G, b=n, m=0, r=1, causal=False)
    for got, r_, name in zip((gq, gk, gv), ref, ("dQ", "dK", "dV")):
        _assert_grad_close(to_host(got), r_, name)


def test_backward_on_the_mixture_law(ha, torch):
    """Peaked attention rows (scores up to +-250): dQ and dK against the looser bound the
    cancellation in dP - delta calls for, dV against the tight one."""
    print("backward mixture", flush=True)
    cfg = dict(B=1, H=2, n=4096, d=64, dtype="bf16", law="mixture", b=256, m=512, r=7, causal=0, n_min=4096, seed=0)
    _run_case(ha, torch, cfg, peaked=True)


def test_backward_with_delta_from_the_bf16_output(ha, torch):
    print("backward, delta from bf16 out", flush=True)
    cfg = dict(B=1, H=2, n=2048, d=128, dtype="bf16", law="iid", b=256, m=256, r=7, causal=1, n_min=512, seed=0)
    Q, K, V = synth_inputs.make_qkv(cfg, seed=77)
    G = _cotangent(Q.shape, 78)
    tq, tk, tv, tg = (to_device(x, "bf16") for x in (Q, K, V, G))
    shape = ha.make_shape(1, 2, 2048, 128, ha.HA_BF16)
    ws = ha.alloc_workspace(shape, ha.make_params(256, 256, 7, True, 512, 0))
    kw = dict(causal=True, n_min=512, seed=0)
    out, lse = ha.hyperattn_forward(tq, tk, tv, 256, 256, 7, workspace=ws, **kw)
    grads = ha.hyperattn_backward(tq, tk, tv, out, lse, tg, 256, 256, 7, fwd_workspace=ws, **kw)
    torch.cuda.synchronize()
    ref = orc.hyperattn_backward(Q, K, V, G, b=256, m=256, r=7, causal=True, n_min=512, seed=0)
    for got, r_, what in zip(grads, ref, ("dQ", "dK", "dV")):
        _assert_grad_close(to_host(got), r_, what)


def test_backward_is_deterministic_and_leaves_inputs_alone(ha, torch):
    print("backward determinism", flush=True)
    cfg = dict(B=1, H=2, n=2048, d=128, dtype="bf16", law="iid", b=128, m=128, r=7, causal=1, n_min=512, seed=1)
    (gq, gk, gv), (tq, tk, tv, out, lse, tg, ws, out32) = _run_case(ha, torch, cfg)
    before = [t.clone() for t in (tq, tk, tv, out, lse, tg, ws)]
    kw = dict(causal=1, n_min=512, seed=1)
    gq2, gk2, gv2 = ha.hyperattn_backward(tq, tk, tv, out, lse, tg, 128, 128, 7, fwd_workspace=ws, out_f32=out32, **kw)
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


def _random_cases(count, seed):
    """Seeded random (d, n, n_min, b, m, r, causal) combinations within what the library accepts."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        d = int(rng.choice([64, 128]))
        causal = int(rng.integers(0, 2))
        b = int(rng.choice([8, 16, 24, 32, 48, 64, 96, 128, 256]))
        r = int(rng.integers(1, 9))
        m = int(rng.choice([0, 16, 33, 64, 100, 256]))
        if causal:
            n_min = b * int(rng.integers(1, 5))
            n = n_min * (1 << int(rng.integers(0, 5)))
        else:
            n_min = 4096
            n = b * int(rng.integers(1, 20))
        if n > 3000:
            continue
        cases.append((d, n, n_min, b, m, r, causal))
    return cases


@pytest.mark.parametrize("d,n,n_min,b,m,r,causal", _random_cases(24, 2024))
def test_forward_and_backward_on_random_small_problems(ha, torch, d, n, n_min, b, m, r, causal):
    """Forward (codes, outputs) and backward against the oracle on seeded random parameter combinations."""
    from ha_testutil import assert_close, assert_lse_close, run_oracle
    print(f"random case d={d} n={n} n_min={n_min} b={b} m={m} r={r} causal={causal}", flush=True)
    cfg = dict(B=1, H=2, n=n, d=d, dtype="bf16", law="iid", b=b, m=m, r=r, causal=causal, n_min=n_min, seed=n + m)
    _, (tq, tk, tv, out, lse, tg, ws, _) = _run_case(ha, torch, cfg, seed_data=1000 + n)
    Q, K, V = synth_inputs.make_qkv(cfg, seed=1000 + n)
    flips = []
    shape = ha.make_shape(1, 2, n, d, ha.HA_BF16)
    params = ha.make_params(b, m, r, causal, n_min, cfg["seed"])
    if ha.ha_workspace_layout(shape, params).levels > 0:
        views = ha.workspace_views(ws, shape, params)
        stages = {}
        run_oracle(Q, K, V, cfg, stages=stages)
        flips = compare_codes(np.stack([views["codes_q"].cpu().numpy(), views["codes_k"].cpu().numpy()]), stages, r)
    # rows with few keys average little: the operand-rounding term 2^-8 sum_j p_j |v_j| is passed explicitly
    ref_out, ref_lse, absv = run_oracle(Q, K, V, cfg, flip=flips or None, with_absv=True)
    assert_close(to_host(out), ref_out, "bf16", "out", absv)
    assert_lse_close(to_host(lse), ref_lse, "bf16", "lse")
