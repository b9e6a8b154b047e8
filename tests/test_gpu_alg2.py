"""GPU parity of the Algorithm 2 / Lemma 2 options (hyperattn_forward_alg2) against the
oracle's dense evaluation: the rows of T bit-exact; the rows drawn by squared value norm
(Lemma 2, inverse of the cumulative law in fp64 on both sides) equal except where the
oracle's uniform lies within 1e-9 of a boundary of that law (counted, and replayed in the
oracle like a projection too close to zero); log tau and log d~ within fp32 accuracy, outputs
within the forward's tolerance (bf16: 2e-3 + half an ulp; fp32: 1e-5 + 1e-5 |ref|).  Where
fewer than 16 sampled rows carry a row's whole value product (Lemma 2 with a small m) the
rounding of the weights to bf16 as matrix-core operands does not average out and an element
may also use 2^-8 sum_j w_j |v_j| (the oracle run on |V| with the draws of V); the share of
the elements that need it is printed and must stay below 0.5 %."""
import numpy as np
import pytest

import synth_inputs
from oracle import hyperattn_oracle as orc
from ha_testutil import assert_close, have_gpu, to_device, to_host

pytestmark = [pytest.mark.gpu, pytest.mark.skipif(not have_gpu(), reason="needs a GPU")]


@pytest.fixture(scope="module")
def ha():
    import paper_2310_05869_amd as mod
    mod.lib()
    return mod


@pytest.fixture(scope="module")
def torch():
    import torch as t
    return t


CASES = [  # dtype, d, n, b, m, r, cap_scale, kappa, vnorm
    ("bf16", 64, 512, 64, 48, 5, 0.0, 0.0, False),      # no caps: the Section 4 estimator
    ("bf16", 64, 512, 64, 48, 5, 8.0, 1.2, False),      # both caps bind on part of the rows (12 % / 65 %)
    ("bf16", 128, 768, 96, 100, 6, 1e-4, 2.0, False),   # cap below every entry
    ("bf16", 128, 768, 96, 100, 6, 4.0, 1.1, True),     # Lemma 2's value product, caps binding (27 % / 86 %)
    ("fp32", 64, 384, 32, 20, 4, 25.0, 1.5, True),
    ("fp32", 64, 384, 32, 20, 4, 0.0, 0.0, True),
    ("bf16", 64, 600, 200, 7, 7, 10.0, 0.0, True),      # block not a multiple of the row tile, cap without lower cap
    ("bf16", 128, 2048, 256, 256, 7, 8.0, 1.2, False),  # the benchmark's b and m: two query tiles per block, four key tiles per segment
    ("bf16", 128, 2048, 256, 256, 7, 4.0, 1.1, True),
    ("bf16", 64, 1536, 512, 300, 6, 6.0, 1.3, True),    # four query tiles per block, five ragged sample tiles
    ("bf16", 64, 1000, 8, 130, 3, 5.0, 1.5, False),     # tiny blocks, tau rows over ragged key tiles
]


@pytest.mark.parametrize("dtype,d,n,b,m,r,cap_scale,kappa,vnorm", CASES)
def test_alg2_options_match_the_oracle(ha, torch, dtype, d, n, b, m, r, cap_scale, kappa, vnorm):
    print(f"alg2 {dtype} d={d} n={n} b={b} m={m} r={r} cap={cap_scale} kappa={kappa} vnorm={vnorm}", flush=True)
    cfg = dict(B=1, H=2, n=n, d=d, dtype=dtype, law="iid")
    Q, K, V = synth_inputs.make_qkv(cfg, seed=11 + n)
    rng = np.random.default_rng(n)
    V = V * rng.uniform(0.2, 2.0, size=(1, 2, n, 1)).astype(np.float32)       # unequal value-row norms
    V = synth_inputs.round_to_bf16(V) if dtype == "bf16" else V.astype(np.float32)
    seed = 5
    tq, tk, tv = (to_device(x, dtype) for x in (Q, K, V))
    out, lse, ws = ha.hyperattn_forward_alg2(tq, tk, tv, b, m, r, seed=seed, cap_scale=cap_scale, kappa=kappa,
                                             vnorm_sampling=vnorm)
    torch.cuda.synchronize()
    shape = ha.make_shape(1, 2, n, d, ha.HA_BF16 if dtype == "bf16" else ha.HA_FP32)
    params = ha.make_params(b, m, r, False, 4096, seed)
    views = ha.alg2_workspace_views(ws, shape, params)
    replay = {}
    if vnorm:
        for bh in range(2):
            w = (V[0, bh].astype(np.float64) ** 2).sum(axis=1)
            np.testing.assert_allclose(views["vnorm_w"][bh].cpu().numpy(), w, rtol=1e-13)
            marg = []
            idx, logw = orc.vnorm_samples(V[0, bh], seed, bh, m, margin=marg)
            got = views["vnorm_samples"][bh, 0].cpu().numpy()
            for r_ in np.nonzero(got != idx)[0]:
                assert marg[r_] < 1e-9 and abs(int(got[r_]) - int(idx[r_])) == 1, (bh, r_, got[r_], idx[r_], marg[r_])
                replay.setdefault(bh, {})[int(r_)] = int(got[r_])
            idx, logw = orc.vnorm_samples(V[0, bh], seed, bh, m, replay=replay.get(bh))
            np.testing.assert_allclose(views["vnorm_logw"][bh, 0].cpu().numpy(), logw, rtol=1e-6, atol=1e-6)
        print(f"  Lemma 2 draws within rounding of a boundary (replayed): {sum(len(v) for v in replay.values())}", flush=True)
    ref_out, ref_lse, ref_tau = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, cap_scale=cap_scale,
                                                           kappa=kappa, vnorm_sampling=vnorm, vnorm_replay=replay)
    if cap_scale > 0 or kappa > 0:   # the options must actually act in this instance, or the case tests nothing
        plain = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed)[1]
        changed = np.abs(plain - ref_lse) > 1e-9
        print(f"  caps change log d~ on {changed.mean():.0%} of the rows", flush=True)
        assert changed.any()
    np.testing.assert_array_equal(views["tau_rows"][0].cpu().numpy(), orc.tau_rows(seed, n, m))
    np.testing.assert_allclose(views["log_tau"][:, 0].cpu().numpy(), ref_tau, rtol=2e-5, atol=2e-5)
    np.testing.assert_allclose(to_host(lse), ref_lse, rtol=3e-5, atol=3e-5)
    absv = None
    if dtype == "bf16" and 0 < m < 16:   # squared row norms, hence the draws, are those of V
        absv = orc.hyperattn_forward_alg2(Q, K, np.abs(V), b=b, m=m, r=r, seed=seed, cap_scale=cap_scale, kappa=kappa,
                                          vnorm_sampling=vnorm, vnorm_from=V, vnorm_replay=replay)[0]
    assert_close(to_host(out), ref_out, dtype, "out", absv, 0.005)


CAUSAL_CASES = [  # dtype, d, n, n_min, b, m, r, cap_scale, kappa, vnorm
    ("bf16", 128, 2048, 256, 128, 64, 6, 6.0, 1.3, False),     # three levels, 1 + 2 + 4 nodes
    ("bf16", 128, 2048, 256, 128, 64, 6, 5.0, 1.2, True),
    ("bf16", 64, 1024, 128, 32, 40, 5, 8.0, 1.5, True),        # nodes of 512, 256, 128 rows; ragged sample tiles
    ("fp32", 64, 512, 64, 32, 20, 4, 10.0, 1.5, True),
    ("fp32", 64, 512, 64, 32, 20, 4, 0.0, 0.0, False),         # no caps: the Section 4 causal forward
    ("bf16", 64, 4096, 1024, 256, 256, 7, 8.0, 1.2, False),    # the benchmark's b and m, two levels
]


@pytest.mark.parametrize("dtype,d,n,n_min,b,m,r,cap_scale,kappa,vnorm", CAUSAL_CASES)
def test_alg2_options_on_causal_problems(ha, torch, dtype, d, n, n_min, b, m, r, cap_scale, kappa, vnorm):
    """Algorithm 4 with Algorithm 2 as printed at every off-diagonal node: every node's rows of T bit-exact,
    log tau of every node, Lemma 2's draws per node (replayed where a uniform sits within rounding of a
    boundary), then log D~ and the outputs."""
    print(f"alg2 causal {dtype} d={d} n={n} n_min={n_min} b={b} m={m} r={r} cap={cap_scale} kappa={kappa} vnorm={vnorm}", flush=True)
    H = 2
    cfg = dict(B=1, H=H, n=n, d=d, dtype=dtype, law="iid")
    Q, K, V = synth_inputs.make_qkv(cfg, seed=23 + n)
    rng = np.random.default_rng(n + 1)
    V = V * rng.uniform(0.1, 1.0, size=(1, H, n, 1)).astype(np.float32)          # unequal value-row norms
    V = synth_inputs.round_to_bf16(V) if dtype == "bf16" else V.astype(np.float32)
    seed = 8
    tq, tk, tv = (to_device(x, dtype) for x in (Q, K, V))
    out, lse, ws = ha.hyperattn_forward_alg2(tq, tk, tv, b, m, r, seed=seed, cap_scale=cap_scale, kappa=kappa,
                                             vnorm_sampling=vnorm, causal=True, n_min=n_min)
    torch.cuda.synchronize()
    shape = ha.make_shape(1, H, n, d, ha.HA_BF16 if dtype == "bf16" else ha.HA_FP32)
    params = ha.make_params(b, m, r, True, n_min, seed)
    views = ha.alg2_workspace_views(ws, shape, params)
    levels = int(np.log2(n // n_min))
    replay = {}
    for level in range(levels):
        s_rows = n >> (level + 1)
        for node in range(1 << level):
            heap = (1 << level) - 1 + node
            np.testing.assert_array_equal(views["tau_rows"][heap].cpu().numpy(), orc.tau_rows(seed, s_rows, m, heap))
            if vnorm:
                for bh in range(H):
                    k0 = 2 * node * s_rows
                    marg = []
                    idx, _ = orc.vnorm_samples(V[0, bh, k0:k0 + s_rows], seed, bh, m, margin=marg, heap=heap, n_heads=H)
                    got = views["vnorm_samples"][bh, heap].cpu().numpy()
                    for r_ in np.nonzero(got != idx)[0]:
                        assert marg[r_] < 1e-9 and abs(int(got[r_]) - int(idx[r_])) == 1, (bh, heap, r_, marg[r_])
                        replay.setdefault((bh, heap), {})[int(r_)] = int(got[r_])
                    _, logw = orc.vnorm_samples(V[0, bh, k0:k0 + s_rows], seed, bh, m, replay=replay.get((bh, heap)),
                                                heap=heap, n_heads=H)
                    np.testing.assert_allclose(views["vnorm_logw"][bh, heap].cpu().numpy(), logw, rtol=1e-6, atol=1e-6)
    okw = dict(b=b, m=m, r=r, seed=seed, cap_scale=cap_scale, kappa=kappa, vnorm_sampling=vnorm, causal=True,
               n_min=n_min, vnorm_replay=replay)
    ref_out, ref_lse, ref_tau = orc.hyperattn_forward_alg2(Q, K, V, **okw)
    if cap_scale > 0 or kappa > 0:
        plain = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, causal=True, n_min=n_min)[1]
        changed = np.abs(plain - ref_lse) > 1e-9
        print(f"  caps change log D~ on {changed.mean():.0%} of the rows; replayed draws {sum(len(v) for v in replay.values())}",
              flush=True)
        assert changed.any()
    np.testing.assert_allclose(views["log_tau"].cpu().numpy(), ref_tau, rtol=3e-5, atol=3e-5)
    np.testing.assert_allclose(to_host(lse), ref_lse, rtol=3e-5, atol=5e-5)
    absv = None
    if dtype == "bf16" and 0 < m < 16:
        absv = orc.hyperattn_forward_alg2(Q, K, np.abs(V), vnorm_from=V, **okw)[0]
    assert_close(to_host(out), ref_out, dtype, "out", absv, 0.005)


def test_alg2_rejects_bad_arguments(ha, torch):
    print("alg2 errors", flush=True)
    shape = ha.make_shape(1, 1, 256, 64, ha.HA_BF16)
    with pytest.raises(ha.HyperAttnError):          # causal: n / n_min must be a power of two
        ha.ha_alg2_workspace_layout(shape, ha.make_params(64, 16, 7, True, 96, 0))
    q = torch.zeros((1, 1, 256, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ha.HyperAttnError):
        ha.hyperattn_forward_alg2(q, q, q, 64, 16, 7, workspace=torch.zeros(256, dtype=torch.uint8, device="cuda"))
    # a causal problem at or below n_min is plain exact causal attention
    out, lse, _ = ha.hyperattn_forward_alg2(q, q, q, 64, 16, 7, causal=True, n_min=256, cap_scale=2.0, kappa=1.5)
    ref, _ = ha.exact_attn_forward(q, q, q, causal=True)
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
