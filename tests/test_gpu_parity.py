"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the
same seeded inputs.  Integer stages (bucket codes, permutations, gathers) must
be bit-exact; floating point outputs must be within the stated tolerance
(bf16: 2e-3 + half a bf16 ulp of the result; fp32: 1e-5 + 1e-5 |result|).

Only where a row's weight can sit on a handful of keys, so that the rounding of
the softmax weights to bf16 (matrix-core operands, relative error up to 2^-9)
does not average out, may an element also use the allowance
2^-8 sum_j p_j |v_j| (the oracle run on |V|): the 64-centre mixture law, and
0 < m < 16, where a single sampled key carries the weight s/m.  There the
number of elements that need the allowance is printed and must stay below
0.5 % (measured: at most 0.17 %); everywhere else the plain criterion is the
assertion."""
import ctypes

import numpy as np
import pytest

import synth_inputs
from oracle import hyperattn_oracle as orc
from ha_testutil import (assert_close, assert_lse_close, compare_codes, have_gpu, run_oracle, to_device, to_host)

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


# ------------------------------------------------------------------ a1: lsh_hash
@pytest.mark.parametrize("dtype,d,r,rows", [("bf16", 128, 7, 4099), ("bf16", 64, 7, 777), ("bf16", 128, 8, 64),
                                           ("bf16", 64, 1, 5), ("fp32", 64, 7, 1024), ("fp32", 128, 3, 1001),
                                           ("bf16", 128, 7, 1)])
def test_lsh_hash_bit_exact(ha, torch, dtype, d, r, rows):
    print(f"lsh_hash {dtype} d={d} r={r} rows={rows}", flush=True)
    X = synth_inputs.iid_qkv(1, 1, rows, d, dtype, seed=7)[0].reshape(rows, d)
    R = orc.make_projection(5, d, r)
    p = orc.lsh_project(X, R)
    ref = orc.lsh_codes(p, r)
    got = ha.ha_lsh_hash(to_device(X, dtype), torch.from_numpy(R.astype(np.float32)).cuda())
    got = got.cpu().numpy().astype(np.int64)
    bad = np.nonzero(got != ref)[0]
    for i in bad:
        assert np.abs(p[i]).min() < 1e-6
    print(f"  disagreements (all with |p|<1e-6): {len(bad)}", flush=True)
    assert len(bad) <= 1


def test_lsh_hash_arbitrary_fp32_R_and_zero_rows(ha, torch):
    rng = np.random.default_rng(0)
    d, r, rows = 64, 6, 300
    X = rng.standard_normal((rows, d)).astype(np.float32)
    X[5] = 0.0                      # projections exactly 0 -> all bits 0 -> bucket 0
    R = rng.standard_normal((d, r)).astype(np.float32)
    ref = orc.lsh_codes(orc.lsh_project(X, R), r)
    got = ha.ha_lsh_hash(torch.from_numpy(X).cuda(), torch.from_numpy(R).cuda()).cpu().numpy()
    np.testing.assert_array_equal(got, ref)
    assert got[5] == 0


# ------------------------------------------------------------------ a2: seg_sort
@pytest.mark.parametrize("n_seg,seg_len,nb", [(3, 1, 4), (2, 63, 128), (5, 64, 128), (4, 65, 2), (3, 1000, 128),
                                              (2, 40000, 256), (1, 70000, 1), (6, 4096, 128)])
def test_seg_sort_bit_exact(ha, torch, n_seg, seg_len, nb):
    print(f"seg_sort n_seg={n_seg} seg_len={seg_len} buckets={nb}", flush=True)
    rng = np.random.default_rng(seg_len)
    codes = rng.integers(0, nb, size=(n_seg, seg_len)).astype(np.uint8)
    perm, pos = ha.ha_seg_sort(torch.from_numpy(codes).cuda())
    perm, pos = perm.cpu().numpy(), pos.cpu().numpy()
    for g in range(n_seg):
        rp, rq = orc.sort_lsh(codes[g])
        np.testing.assert_array_equal(perm[g], rp)
        np.testing.assert_array_equal(pos[g], rq)


# ------------------------------------------------------------------ a3: gather
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("fp32", 64)])
def test_gather_rows_exact(ha, torch, dtype, d):
    groups, n = 3, 517
    X = synth_inputs.iid_qkv(1, groups, n, d, dtype, seed=3)[0][0]
    idx = np.stack([np.random.default_rng(g).permutation(n) for g in range(groups)]).astype(np.int32)
    got = to_host(ha.ha_gather_rows(to_device(X, dtype), torch.from_numpy(idx).cuda()))
    for g in range(groups):
        np.testing.assert_array_equal(got[g], X[g][idx[g]])


# ------------------------------------------------------------------ a4-a6: stages
STAGE_CASES = [("bf16", 128, 512, 128, 96), ("bf16", 64, 768, 256, 512), ("fp32", 64, 256, 64, 64),
               ("bf16", 128, 384, 96, 40), ("fp32", 128, 192, 48, 7)]


@pytest.mark.parametrize("dtype,d,n,b,m", STAGE_CASES)
def test_block_sampled_merge_stages(ha, torch, dtype, d, n, b, m):
    """Stage entry points on one node, in the order of the Section 4 pipeline:
    sort -> gather -> block part / sampled part (sorted order) -> merge."""
    print(f"stages {dtype} d={d} n={n} b={b} m={m}", flush=True)
    groups = 2
    Q, K, V = (x[0] for x in synth_inputs.iid_qkv(1, groups, n, d, dtype, seed=21))
    r = 5
    R = orc.make_projection(1, d, r)
    Rd = torch.from_numpy(R.astype(np.float32)).cuda()
    Qd, Kd, Vd = (to_device(x, dtype) for x in (Q, K, V))
    cq = ha.ha_lsh_hash(Qd, Rd)
    ck = ha.ha_lsh_hash(Kd, Rd)
    perm_q, _ = ha.ha_seg_sort(cq)
    perm_k, pos_k = ha.ha_seg_sort(ck)
    Qs = ha.ha_gather_rows(Qd, perm_q)
    Ks = ha.ha_gather_rows(Kd, perm_k)
    Vs = ha.ha_gather_rows(Vd, perm_k)
    samples = orc.make_samples(3, 0, 0, n, m).astype(np.int32)
    o_b, l_b = ha.ha_block_attn(Qs, Ks, Vs, b)
    o_r, l_r = ha.ha_sampled_attn(Qs, Kd, Vd, torch.from_numpy(samples).cuda(), pos_k, b)
    out_dtype = torch.bfloat16 if dtype == "bf16" else torch.float32
    out, lse = ha.ha_merge_unpermute(o_b, l_b, o_r, l_r, perm_q, out_dtype)
    for g in range(groups):
        pq, posq = orc.sort_lsh(orc.lsh_codes(orc.lsh_project(Q[g], R), r))
        pk, posk = orc.sort_lsh(orc.lsh_codes(orc.lsh_project(K[g], R), r))
        np.testing.assert_array_equal(perm_q[g].cpu().numpy(), pq)
        np.testing.assert_array_equal(perm_k[g].cpu().numpy(), pk)
        q64, k64, v64 = (x[g].astype(np.float64) for x in (Q, K, V))
        Ob, Lb = orc.block_part(q64, k64, v64, pq, pk, b)
        Or, Lr = orc.sampled_part(q64, k64, v64, posq, posk, b, samples)
        # stage outputs are in sorted order
        assert_close(to_host(o_b[g]), Ob[pq], "fp32" if dtype == "fp32" else "bf16", "o_b")
        assert_lse_close(to_host(l_b[g]), Lb[pq], dtype, "lse_b")
        assert_close(to_host(o_r[g]), Or[pq], "fp32" if dtype == "fp32" else "bf16", "o_r")
        assert_lse_close(to_host(l_r[g]), Lr[pq], dtype, "lse_r")
        Om, Lm = orc.merge_parts(Ob, Lb, Or, Lr)
        assert_close(to_host(out[g]), Om, dtype, "merged out")
        assert_lse_close(to_host(lse[g]), Lm, dtype, "merged lse")


# ------------------------------------------------------------------ a8: exact attention
@pytest.mark.parametrize("dtype,d,n,causal", [("bf16", 128, 300, False), ("bf16", 128, 300, True),
                                             ("bf16", 64, 1000, True), ("bf16", 64, 129, False),
                                             ("fp32", 64, 200, True), ("fp32", 128, 77, False),
                                             ("bf16", 128, 1, True), ("bf16", 128, 1024, True)])
def test_exact_attn_matches_definition(ha, torch, dtype, d, n, causal):
    print(f"exact {dtype} d={d} n={n} causal={causal}", flush=True)
    Q, K, V = synth_inputs.iid_qkv(1, 2, n, d, dtype, seed=31)
    out, lse = ha.exact_attn_forward(*(to_device(x, dtype) for x in (Q, K, V)), causal=causal)
    for h in range(2):
        ro, rl = orc.exact_attention(Q[0, h], K[0, h], V[0, h], causal)
        assert_close(to_host(out[0, h]), ro, dtype, "exact out")
        assert_lse_close(to_host(lse[0, h]), rl, dtype, "exact lse")


# ------------------------------------------------------------------ whole forward
PLAIN_FRAC = 0.005   # share of the elements that may need the operand-rounding allowance where few keys carry a row
RARE_FRAC = 1e-5     # elsewhere: the plain criterion is met by all but isolated elements (measured on the suite: by all)


def _few_keys_carry_a_row(cfg):
    """Where a handful of keys can hold a row's whole weight, the rounding of the weights to bf16 operands
    (2^-9 each) no longer averages out and the operand-rounding allowance of ha_testutil.assert_close applies,
    for at most PLAIN_FRAC of the elements: the peaked mixture law, m of a few samples weighted s/m, and
    causal problems, where row i of a base block attends to i + 1 keys (a seeded search over 1900 further
    cases met the plain criterion's limit three times, one element each, on such rows)."""
    return cfg["dtype"] == "bf16" and (cfg["law"] == "mixture" or 0 < cfg["m"] < 16 or bool(cfg["causal"]))


def _plain_share(cfg):
    """Share of the elements that may exceed the plain criterion 2e-3 + half an ulp (staying inside the bound with
    the operand-rounding allowance, which the arithmetic guarantees everywhere)."""
    return PLAIN_FRAC if _few_keys_carry_a_row(cfg) else RARE_FRAC


def _forward_and_compare(ha, torch, cfg, Q, K, V, R=None, samples=None, sample_fn=None, plain_frac=None):
    dtype = cfg["dtype"]
    p_rounding_term = dtype == "bf16"
    if plain_frac is None:
        plain_frac = _plain_share(cfg)
    B, H, n, d = Q.shape
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16 if dtype == "bf16" else ha.HA_FP32)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    Rd = None if R is None else torch.from_numpy(R.astype(np.float32)).cuda()
    sd = None if samples is None else torch.from_numpy(samples.astype(np.int32)).cuda()
    out, lse = ha.hyperattn_forward(*(to_device(x, dtype) for x in (Q, K, V)), cfg["b"], cfg["m"], cfg["r"],
                                    causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"], R=Rd, samples=sd,
                                    workspace=ws)
    torch.cuda.synchronize()
    views = ha.workspace_views(ws, shape, params)
    lay = views["layout"]
    # stage 1: codes
    stages = {}
    ref_out, ref_lse, absv = run_oracle(Q, K, V, cfg, R=R, sample_fn=sample_fn, stages=stages, with_absv=True)
    flips = []
    if lay.levels > 0:
        gpu_codes = np.stack([views["codes_q"].cpu().numpy(), views["codes_k"].cpu().numpy()])
        flips = compare_codes(gpu_codes, stages, cfg["r"])
        if flips:
            print(f"  replaying {len(flips)} near-zero sign bits in the oracle", flush=True)
            stages = {}
            ref_out, ref_lse, absv = run_oracle(Q, K, V, cfg, R=R, sample_fn=sample_fn, flip=flips, stages=stages,
                                                with_absv=True)
        # stage 2: permutations of every node
        pq, pk, posk = (views[k].cpu().numpy() for k in ("perm_q", "perm_k", "pos_k"))
        # (and the sorted block of every sampled key, which Algorithm 2's factor 1 - M_{i,l_j} is read from)
        smp = views["samples"].cpu().numpy() if "samples" in views else None
        sblk = views["samp_blk"].cpu().numpy() if "samp_blk" in views else None
        for bh in range(B * H):
            for level in range(lay.levels):
                nodes = (1 << level) if cfg["causal"] else 1
                s = (n >> (level + 1)) if cfg["causal"] else n
                for node in range(nodes):
                    q0 = (2 * node + 1) * s if cfg["causal"] else 0
                    k0 = (2 * node) * s if cfg["causal"] else 0
                    rq, _ = orc.sort_lsh(stages["codes"][0, bh, q0:q0 + s])
                    rk, rposk = orc.sort_lsh(stages["codes"][1, bh, k0:k0 + s])
                    np.testing.assert_array_equal(pq[level, bh, node * s:(node + 1) * s], rq + q0)
                    np.testing.assert_array_equal(pk[level, bh, node * s:(node + 1) * s], rk + k0)
                    np.testing.assert_array_equal(posk[level, bh, node * s:(node + 1) * s], rposk)
                    if sblk is not None and samples is None:
                        heap = (1 << level) - 1 + node
                        np.testing.assert_array_equal(sblk[bh, heap], rposk[smp[heap]] // cfg["b"])
    # stage 3: outputs
    got = to_host(out)
    err = assert_close(got, ref_out, dtype, "out", absv if p_rounding_term else None, plain_frac)
    assert_lse_close(to_host(lse), ref_lse, dtype, "lse")
    over = int((np.abs(got - ref_out) > 2e-3).sum())
    print(f"  max abs err {err:.3e}; elements over 2e-3: {over} of {got.size}; sign flips {len(flips)}", flush=True)
    return out, lse, ref_out, ref_lse


def test_forward_cfg1_fp32(ha, torch):
    cfg = synth_inputs.CONFIGS["cfg1_n1k_fp32"]
    print("forward cfg1", flush=True)
    Q, K, V = synth_inputs.make_qkv(cfg)
    _forward_and_compare(ha, torch, cfg, Q, K, V)


@pytest.mark.parametrize("d,n,b,m,law", [(128, 2048, 256, 256, "iid"), (64, 4096, 256, 512, "mixture"),
                                         (128, 1536, 128, 100, "iid"), (64, 640, 64, 0, "iid"),
                                         (128, 512, 512, 32, "iid")])
def test_forward_unmasked_bf16(ha, torch, d, n, b, m, law):
    print(f"forward bf16 d={d} n={n} b={b} m={m} {law}", flush=True)
    cfg = dict(B=1, H=2, n=n, d=d, dtype="bf16", law=law, b=b, m=m, r=7, causal=0, n_min=4096, seed=0)
    Q, K, V = synth_inputs.make_qkv(cfg)
    _forward_and_compare(ha, torch, cfg, Q, K, V)


@pytest.mark.parametrize("dtype,d,n,n_min,b,m", [("bf16", 128, 2048, 256, 128, 64), ("bf16", 64, 4096, 1024, 256, 256),
                                                 ("fp32", 64, 512, 64, 32, 16), ("bf16", 128, 1024, 4096, 256, 256),
                                                 ("bf16", 128, 1024, 512, 512, 0),
                                                 # nine levels of recursion (more than the epilogue folds row-major)
                                                 ("bf16", 64, 8192, 16, 16, 8),
                                                 # eight levels, base blocks smaller than a query tile
                                                 ("bf16", 128, 8192, 32, 32, 16)])
def test_forward_causal(ha, torch, dtype, d, n, n_min, b, m):
    print(f"forward causal {dtype} d={d} n={n} n_min={n_min} b={b} m={m}", flush=True)
    cfg = dict(B=2, H=1, n=n, d=d, dtype=dtype, law="iid", b=b, m=m, r=7, causal=1, n_min=n_min, seed=3)
    Q, K, V = synth_inputs.make_qkv(cfg)
    _forward_and_compare(ha, torch, cfg, Q, K, V)


@pytest.mark.parametrize("causal", [0, 1])
def test_identity_sampling_equals_exact_attention(ha, torch, causal):
    """Every key sampled exactly once: block part + estimate must be the full
    row sum, i.e. exact attention, whatever the LSH did."""
    print(f"identity sampling causal={causal}", flush=True)
    n, d, b, n_min = 1024, 128, 128, 256
    cfg = dict(B=1, H=2, n=n, d=d, dtype="bf16", law="iid", b=b, m=n // 2 if causal else n, r=6, causal=causal,
               n_min=n_min, seed=9)
    Q, K, V = synth_inputs.make_qkv(cfg)
    if causal:
        # every node's index set has the same length m: use the largest node's size
        # for all (smaller nodes clamp duplicates away is not wanted) -> give each
        # node exactly its own identity by choosing m = s of the top node only
        cfg["n_min"] = n // 2          # one split: a single node of s = n/2 = m
        samples = np.arange(n // 2)[None, :]
    else:
        samples = np.arange(n)[None, :]
    shape = ha.make_shape(1, 2, n, d, ha.HA_BF16)
    params = ha.make_params(b, cfg["m"], cfg["r"], causal, cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    out, lse = ha.hyperattn_forward(*(to_device(x, "bf16") for x in (Q, K, V)), b, cfg["m"], cfg["r"],
                                    causal=causal, n_min=cfg["n_min"], seed=cfg["seed"],
                                    samples=torch.from_numpy(samples.astype(np.int32)).cuda(), workspace=ws)
    for h in range(2):
        ro, rl = orc.exact_attention(Q[0, h], K[0, h], V[0, h], bool(causal))
        assert_close(to_host(out[0, h]), ro, "bf16", "identity-sampled out")
        assert_lse_close(to_host(lse[0, h]), rl, "bf16", "identity-sampled lse")


def test_deterministic_and_inputs_untouched(ha, torch):
    cfg = dict(B=1, H=2, n=1024, d=128, dtype="bf16", law="iid", b=128, m=64, r=7, causal=1, n_min=256, seed=1)
    Q, K, V = (to_device(x, "bf16") for x in synth_inputs.make_qkv(cfg))
    keep = [x.clone() for x in (Q, K, V)]
    o1, l1 = ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], causal=True, n_min=cfg["n_min"], seed=1)
    o2, l2 = ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], causal=True, n_min=cfg["n_min"], seed=1)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(l1, l2)
    for a, b_ in zip(keep, (Q, K, V)):
        assert torch.equal(a.view(torch.int16), b_.view(torch.int16))
    o3, _ = ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], causal=True, n_min=cfg["n_min"], seed=2)
    assert not torch.equal(o1.view(torch.int16), o3.view(torch.int16))


def test_rows_are_normalised_on_gpu(ha, torch):
    """V = 1 must give out = 1: the block part and the estimate share one normaliser."""
    cfg = dict(B=1, H=1, n=2048, d=64, dtype="bf16", law="iid", b=256, m=128, r=7, causal=0, n_min=4096, seed=0)
    Q, K, _ = synth_inputs.make_qkv(cfg)
    V = torch.ones((1, 1, 2048, 64), dtype=torch.bfloat16, device="cuda")
    out, _ = ha.hyperattn_forward(to_device(Q, "bf16"), to_device(K, "bf16"), V, 256, 128, 7)
    assert (out.float() - 1).abs().max().item() <= 2 ** -8


def test_empty_and_error_paths(ha, torch):
    z = torch.empty((0, 2, 64, 64), dtype=torch.bfloat16, device="cuda")
    out, lse = ha.hyperattn_forward(z, z, z, 64, 8, 4)
    assert out.numel() == 0
    q = torch.zeros((1, 1, 100, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ha.HyperAttnError) as e:
        ha.hyperattn_forward(q, q, q, 64, 8, 4)            # n % b != 0
    assert e.value.status == -3
    q = torch.zeros((1, 1, 128, 64), dtype=torch.bfloat16, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(ha.HyperAttnError) as e:
        ha.hyperattn_forward(q, q, q, 64, 8, 4, workspace=small)
    assert e.value.status == -4
    # the binding takes every size from Q: tensors that do not match are refused before the call
    with pytest.raises(ValueError):
        ha.hyperattn_forward(q, q[:, :, :64], q, 64, 8, 4)
    with pytest.raises(TypeError):
        ha.hyperattn_forward(q, q, q.float(), 64, 8, 4)
    with pytest.raises(TypeError):
        ha.hyperattn_forward(q, q, q, 64, 8, 4, lse=torch.zeros((1, 1, 128), dtype=torch.float64, device="cuda"))
    with pytest.raises(ValueError):
        ha.exact_attn_forward(q, q, q, out=torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device="cuda"))
    # caller-supplied sample indices outside their node
    bad = torch.full((1, 8), 128, dtype=torch.int32, device="cuda")
    with pytest.raises(ha.HyperAttnError) as e:
        ha.hyperattn_forward(q, q, q, 64, 8, 4, samples=bad)
    assert e.value.status == -3
    ok = torch.full((1, 8), 127, dtype=torch.int32, device="cuda")
    ha.hyperattn_forward(q, q, q, 64, 8, 4, samples=ok)
    qc = torch.zeros((1, 1, 256, 64), dtype=torch.bfloat16, device="cuda")   # causal: nodes of 128, 64, 64 rows
    with pytest.raises(ha.HyperAttnError):
        ha.hyperattn_forward(qc, qc, qc, 64, 2, 4, causal=True, n_min=64,
                             samples=torch.tensor([[127, 0], [64, 0], [0, 0]], dtype=torch.int32, device="cuda"))
    ha.hyperattn_forward(qc, qc, qc, 64, 2, 4, causal=True, n_min=64,
                         samples=torch.tensor([[127, 0], [63, 0], [0, 63]], dtype=torch.int32, device="cuda"))


# ------------------------------------------------------------------ hash: the uncertified-sign path
def test_lsh_hash_bf16_rows_with_vanishing_projections(ha, torch):
    """bf16 rows hashed on the matrix cores: rows whose projection is exactly
    zero (or all zero) cannot be certified there and must come out of the fp64
    redo with the oracle's bit (0 for p == 0)."""
    d, r, rows = 128, 7, 200
    R = orc.make_projection(11, d, r)                       # bf16-representable
    X = synth_inputs.iid_qkv(1, 1, rows, d, "bf16", seed=5)[0].reshape(rows, d).copy()
    X[3] = 0.0
    for i, (a, b_) in enumerate([(0, 1), (5, 90), (17, 127)]):
        x = np.zeros(d, dtype=np.float32)
        x[a], x[b_] = R[b_, 0], -R[a, 0]                    # <x, R[:,0]> == 0 exactly
        X[10 + i] = x
    p = orc.lsh_project(X, R)
    assert p[10, 0] == 0.0 and p[11, 0] == 0.0
    ref = orc.lsh_codes(p, r)
    got = ha.ha_lsh_hash(to_device(X, "bf16"), torch.from_numpy(R.astype(np.float32)).cuda()).cpu().numpy()
    np.testing.assert_array_equal(got, ref)


def test_lsh_hash_bf16_rows_with_unrepresentable_R(ha, torch):
    """Caller-supplied hyperplanes that are not bf16 values: every row takes the fp64 path."""
    rng = np.random.default_rng(2)
    d, r, rows = 64, 8, 333
    X = synth_inputs.iid_qkv(1, 1, rows, d, "bf16", seed=6)[0].reshape(rows, d)
    R = rng.standard_normal((d, r)).astype(np.float32)
    ref = orc.lsh_codes(orc.lsh_project(X, R), r)
    got = ha.ha_lsh_hash(to_device(X, "bf16"), torch.from_numpy(R).cuda()).cpu().numpy()
    np.testing.assert_array_equal(got, ref)


# ------------------------------------------------------------------ full benchmark sizes, sampled heads
def _full_size_inputs(torch, cfg, checked):
    """All heads drawn on the device from the configuration's law; the checked
    (batch, head) pairs come from the seeded host generator, one host head each."""
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    host = synth_inputs.make_qkv(cfg, B=1, H=len(checked))
    dev = synth_inputs.device_qkv(cfg, torch, g)
    for i in range(3):
        for j, (bi, hi) in enumerate(checked):
            dev[i][bi, hi] = to_device(host[i][0, j], "bf16")
    return dev, host


@pytest.mark.parametrize("name,checked", [
    ("cfg2_n32k", [(0, 0), (0, 11), (0, 21), (0, 31)]),
    ("cfg3_n32k_causal", [(0, 0), (0, 7), (0, 19), (0, 31)]),
    ("cfg4_n131k_causal", [(0, 0), (0, 13), (0, 22), (0, 31)]),
    ("cfg5_n65k_mixture", [(0, 0), (1, 17)]),             # one head of each batch
    # the 12-head, d = 64 sweep shape: shortest, a middle and the longest length
    ("sweep_h12_d64_n4096", [(0, 0), (0, 11)]), ("sweep_h12_d64_n4096_causal", [(0, 0), (0, 11)]),
    ("sweep_h12_d64_n16384_causal", [(0, 0), (0, 5)]), ("sweep_h12_d64_n131072", [(0, 3)]),
    ("sweep_h12_d64_n131072_causal", [(0, 8)])])
def test_full_size_configuration_sampled_heads(ha, torch, name, checked):
    """The benchmark configurations at full size, in the launch configuration
    bench.py times; the (batch, head) pairs fed from the host generator are compared with the
    oracle element by element (codes first, then outputs)."""
    cfg = synth_inputs.CONFIGS[name]
    print(f"full size {name}: checking (batch, head) {checked} against the oracle", flush=True)
    (Q, K, V), host = _full_size_inputs(torch, cfg, checked)
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    out, lse = ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], causal=cfg["causal"], n_min=cfg["n_min"],
                                    seed=cfg["seed"], workspace=ws)
    torch.cuda.synchronize()
    views = ha.workspace_views(ws, shape, params)
    rows = [bi * H + hi for bi, hi in checked]
    stages = {}
    ref_out, ref_lse, absv = run_oracle(*host, cfg, stages=stages, with_absv=True)
    flips = []
    if ha.ha_workspace_layout(shape, params).levels > 0:  # else the call is one exact causal block: nothing is hashed
        gpu_codes = np.stack([views["codes_q"][rows].cpu().numpy(), views["codes_k"][rows].cpu().numpy()])
        flips = compare_codes(gpu_codes, stages, cfg["r"])
    if flips:
        print(f"  replaying {len(flips)} near-zero sign bits in the oracle", flush=True)
        ref_out, ref_lse, absv = run_oracle(*host, cfg, flip=flips, with_absv=True)
    got = np.stack([to_host(out[bi, hi]) for bi, hi in checked])[None]
    got_lse = np.stack([to_host(lse[bi, hi]) for bi, hi in checked])[None]
    err = assert_close(got, ref_out, "bf16", "out", absv, _plain_share(cfg))
    assert_lse_close(got_lse, ref_lse, "bf16", "lse")
    over = int((np.abs(got - ref_out) > 2e-3).sum())
    print(f"  max abs err {err:.3e}; elements over 2e-3: {over} of {got.size}; sign flips {len(flips)}", flush=True)
    # the unchecked heads: rows are normalised and finite
    assert torch.isfinite(out).all() and torch.isfinite(lse).all()


def test_forward_and_backward_replay_in_a_hip_graph(ha, torch):
    """The library only enqueues kernels on the caller's stream (no allocation, no memset, no host wait), so a
    forward + backward call can be captured in a HIP graph.  The graph is replayed three times on new inputs, with
    eager calls and synchronisations in between, and every replay must equal the eager result bit for bit."""
    print("graph replay", flush=True)
    B, H, n, d, b, m, r = 1, 2, 2048, 128, 128, 64, 7
    kw = dict(causal=True, n_min=512, seed=4)
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(b, m, r, True, 512, 4)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)

    def draw():
        return [(torch.randn((B, H, n, d), generator=gen, device="cuda") * (d ** -0.25 if i < 3 else 1.0)).to(torch.bfloat16)
                for i in range(4)]

    def buffers():
        return dict(ws=ha.alloc_workspace(shape, params), bws=ha.alloc_backward_workspace(shape, params),
                    out=torch.empty((B, H, n, d), dtype=torch.bfloat16, device="cuda"),
                    lse=torch.empty((B, H, n), dtype=torch.float32, device="cuda"),
                    grads=tuple(torch.empty((B, H, n, d), dtype=torch.bfloat16, device="cuda") for _ in range(3)))

    def run(Q, K, V, G, bufs):
        out, lse = ha.hyperattn_forward(Q, K, V, b, m, r, workspace=bufs["ws"], out=bufs["out"], lse=bufs["lse"], **kw)
        ha.hyperattn_backward(Q, K, V, out, lse, G, b, m, r, fwd_workspace=bufs["ws"], bwd_workspace=bufs["bws"],
                              grads=bufs["grads"], **kw)

    static_in = draw()
    g_bufs, e_bufs = buffers(), buffers()
    run(*static_in, g_bufs)                      # eager first: per-kernel attributes are set outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(*static_in, g_bufs)
    for rep in range(3):
        fresh = draw()
        for dst, src in zip(static_in, fresh):
            dst.copy_(src)
        run(*fresh, e_bufs)                      # eager, on its own buffers
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        same = [torch.equal(g_bufs["out"].view(torch.int16), e_bufs["out"].view(torch.int16)),
                torch.equal(g_bufs["lse"], e_bufs["lse"])]
        same += [torch.equal(a.view(torch.int16), c.view(torch.int16)) for a, c in zip(g_bufs["grads"], e_bufs["grads"])]
        assert all(same), (rep, same)
        assert torch.isfinite(g_bufs["out"].float()).all()


def test_stamped_forward_equals_the_forward_and_its_stamps_are_ordered(ha, torch):
    """The instrumented instantiation of the attention kernel computes what the product one does, bit for bit,
    and every workgroup's record is consistent: clock readings in phase order, the tile counts of the causal
    base case (query tile i of a block sees 2 (i + 1) key tiles) and of the nodes (block keys plus kept samples)."""
    print("stamped forward", flush=True)
    B, H, n, d, b, m, r, n_min = 1, 3, 4096, 128, 256, 128, 5, 1024
    kw = dict(causal=True, n_min=n_min, seed=9)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(21)
    Q, K, V = [(torch.randn((B, H, n, d), generator=gen, device="cuda") * d ** -0.25).to(torch.bfloat16) for _ in range(3)]
    out, lse = ha.hyperattn_forward(Q, K, V, b, m, r, **kw)
    out2, lse2, node_st, base_st = ha.hyperattn_forward_stamped(Q, K, V, b, m, r, **kw)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16)) and torch.equal(lse, lse2)
    levels = 2                                        # 4096 -> 2048 -> 1024 = n_min
    assert node_st.shape == (levels * B * H * (n // 2) // 128, ha.STAMP_WORDS)
    assert base_st.shape == (B * H * n // 128, ha.STAMP_WORDS)
    for st in (node_st.cpu().numpy(), base_st.cpu().numpy()):
        c = st[:, :5]
        assert (np.diff(c, axis=1) >= 0).all() and (c[:, 0] > 0).all()
        assert (st[:, 6] >= st[:, 5]).all()
        assert ((c[:, 4] - c[:, 0]) < 50_000_000).all()       # a workgroup lives microseconds, not seconds
    tiles = np.sort(ha.stamp_place(base_st[:, 7].cpu().numpy())[0])
    per_block = n_min // 128
    want = np.sort(np.tile(2 * (np.arange(per_block) + 1), B * H * n // n_min))
    assert np.array_equal(tiles, want)
    nt, xcd, se, cu = ha.stamp_place(node_st[:, 7].cpu().numpy())
    assert (xcd < 8).all() and len(set(zip(xcd.tolist(), se.tolist(), cu.tolist()))) <= 256
    assert (nt >= b // 64).all() and (nt <= (b + m) // 64).all() and (nt > b // 64).any()
    # fp32 tensors have no instrumented kernel; a short record buffer is refused
    with pytest.raises(ha.HyperAttnError):
        ha.hyperattn_forward_stamped(Q.float(), K.float(), V.float(), b, m, r, **kw)
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(b, m, r, True, n_min, 9)
    assert ha.ha_forward_workgroups(shape, params) == (node_st.shape[0], base_st.shape[0])
    ws = ha.alloc_workspace(shape, params)
    rc = ha.lib().hyperattn_forward_stamped(Q.data_ptr(), K.data_ptr(), V.data_ptr(), out2.data_ptr(), lse2.data_ptr(),
                                            ctypes.byref(shape), ctypes.byref(params), ws.data_ptr(), ws.numel(), None, node_st.data_ptr(),
                                            node_st.numel() * 8 - 8, base_st.data_ptr(), base_st.numel() * 8)
    assert rc != 0
    torch.cuda.synchronize()


def test_measurement_aids(ha, torch):
    """The rate probes return plausible figures and reject bad buffers."""
    print("measurement aids", flush=True)
    buf = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
    tf = ha.ha_measure_mfma_rate(buf, iters=500)
    rd, cp = ha.ha_measure_hbm_rate(buf)
    print(f"  MFMA {tf:.0f} TFLOP/s, read {rd:.0f} GB/s, copy {cp:.0f} GB/s", flush=True)
    assert 200.0 < tf < 2600.0          # below the 2.5 PFLOP/s peak, far above the vector rate
    assert 500.0 < rd < 8200.0 and 500.0 < cp < 8200.0
    probes = ha.ha_measure_issue_rates(buf)
    print("  issue probes: " + ", ".join(f"{k} {max(v):.0f}" for k, v in probes.items()), flush=True)
    assert set(probes) == set(ha.binding.ISSUE_PROBES)
    assert 400 < max(probes["mfma_x16"]) < 2000                     # 16 MFMAs of 32 cycles, two waves per SIMD
    assert all(20 < max(v) < 20000 for v in probes.values())
    small = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(ha.HyperAttnError):
        ha.ha_measure_issue_rates(small)
    with pytest.raises(ha.HyperAttnError):
        ha.ha_measure_mfma_rate(small)
    with pytest.raises(ha.HyperAttnError):
        ha.ha_measure_hbm_rate(small)


@pytest.mark.parametrize("causal", [0, 1])
def test_diagnostics_against_the_oracle(ha, torch, causal):
    """The epsilon of Eq. (1), alpha and kappa (Lemma 1) as diagnostics.py obtains them from the
    library's entry points, against the oracle's dense fp64 definitions at a small size.  The
    library's figures come from bf16 tensors: about two significant digits."""
    import diagnostics
    print(f"diagnostics causal={causal}", flush=True)
    cfg = dict(B=1, H=2, n=768, d=64, dtype="bf16", law="iid", b=64, m=32, r=5, causal=causal, n_min=192, seed=0)
    Q, K, V = synth_inputs.make_qkv(cfg, seed=21)
    tq, tk, tv = (to_device(x, "bf16") for x in (Q, K, V))
    kw = dict(causal=bool(causal), n_min=cfg["n_min"], seed=cfg["seed"])
    out_h, _ = ha.hyperattn_forward(tq, tk, tv, cfg["b"], cfg["m"], cfg["r"], **kw)
    out_e, lse_e = ha.exact_attn_forward(tq, tk, tv, causal=bool(causal))
    eps, err_op, p_op, v_op = (x.cpu().numpy() for x in
                               diagnostics.spectral_error_of(torch, ha, tq, tk, tv, out_h, out_e, lse_e, bool(causal), 25))
    ref_out, _ = run_oracle(Q, K, V, cfg)
    stages = {}
    if not causal:
        alpha = diagnostics.alpha_of(torch, ha, tq, tk, lse_e).cpu().numpy()
        _, lse_b = ha.hyperattn_forward(tq, tk, tv, cfg["b"], 0, cfg["r"], **kw)
        kappa, _ = diagnostics.kappa_of(torch, lse_e, lse_b)
        orc.hyperattn_forward(Q, K, V, b=cfg["b"], m=0, r=cfg["r"], causal=False, stages=stages)
    for hd in range(2):
        e_ref = orc.spectral_error(ref_out[0, hd], Q[0, hd], K[0, hd], V[0, hd], bool(causal))
        s_ref = np.linalg.svd(orc.attention_matrix(Q[0, hd], K[0, hd], bool(causal)), compute_uv=False)[0]
        print(f"  head {hd}: epsilon {eps[hd]:.4f} vs {e_ref:.4f}; ||D^-1 A|| {p_op[hd]:.4f} vs {s_ref:.4f}", flush=True)
        assert abs(p_op[hd] - s_ref) <= 0.02 * s_ref
        assert abs(eps[hd] - e_ref) <= 0.05 * e_ref            # both outputs carry bf16 rounding (2e-3 of 0.1 .. 1)
        if not causal:
            a_ref = orc.alpha(Q[0, hd], K[0, hd])
            k_ref = orc.kappa(Q[0, hd], K[0, hd], stages["codes"][0, hd], stages["codes"][1, hd], cfg["b"])
            print(f"          alpha {alpha[hd]:.3f} vs {a_ref:.3f}; kappa {float(kappa[hd]):.3f} vs {k_ref:.3f}", flush=True)
            assert abs(alpha[hd] - a_ref) <= 0.03 * a_ref      # bf16 weights squared: about 1 %
            assert abs(float(kappa[hd]) - k_ref) <= 0.05 * k_ref


def test_forward_on_a_side_stream_and_under_graph_capture(ha, torch):
    """The library only enqueues on the caller's stream and allocates nothing, so a
    forward call can run on any stream and be captured into a HIP graph.  Replays
    (with eager work and synchronisations between them) must reproduce the eager
    result bit for bit."""
    print("side stream / graph capture", flush=True)
    cfg = dict(B=1, H=2, n=2048, d=128, dtype="bf16", law="iid", b=128, m=64, r=7, causal=1, n_min=512, seed=4)
    Q, K, V = (to_device(x, "bf16") for x in synth_inputs.make_qkv(cfg, seed=31))
    shape = ha.make_shape(1, 2, 2048, 128, ha.HA_BF16)
    params = ha.make_params(128, 64, 7, True, 512, 4)
    ws = ha.alloc_workspace(shape, params)
    kw = dict(causal=True, n_min=512, seed=4, workspace=ws)
    ref_out, ref_lse = ha.hyperattn_forward(Q, K, V, 128, 64, 7, **kw)
    torch.cuda.synchronize()
    ref_out, ref_lse = ref_out.clone(), ref_lse.clone()

    side = torch.cuda.Stream()
    out = torch.zeros_like(Q)
    lse = torch.zeros_like(ref_lse)
    with torch.cuda.stream(side):
        ha.hyperattn_forward(Q, K, V, 128, 64, 7, out=out, lse=lse, **kw)
    side.synchronize()
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16)) and torch.equal(lse, ref_lse)

    graph = torch.cuda.CUDAGraph()
    out.zero_()
    lse.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        ha.hyperattn_forward(Q, K, V, 128, 64, 7, out=out, lse=lse, **kw)
    for rep in range(3):
        out.zero_()
        lse.zero_()
        ws.zero_()                       # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16)), f"replay {rep}"
        assert torch.equal(lse, ref_lse), f"replay {rep}"


def test_exact_attention_wide_workgroups_sampled_rows(ha, torch):
    """Exact attention at n = 8192, causal or not, takes the 8-wave form of the kernel at d = 128; rows
    sampled across the sequence are checked against the definition."""
    print("exact attention, 8-wave workgroups", flush=True)
    for d, causal in ((128, False), (128, True), (64, False)):
        cfg = dict(B=1, H=2, n=8192, d=d, dtype="bf16", law="iid")
        Q, K, V = synth_inputs.make_qkv(cfg, seed=17)
        out, lse = ha.exact_attn_forward(*(to_device(x, "bf16") for x in (Q, K, V)), causal=causal)
        torch.cuda.synchronize()
        rows = np.array([0, 1, 31, 32, 127, 128, 255, 256, 4095, 4096, 8000, 8191])
        for hd in range(2):
            if causal:
                ref = [orc.exact_attention(Q[0, hd][i:i + 1], K[0, hd][:i + 1], V[0, hd][:i + 1]) for i in rows]
                ref_o = np.concatenate([r[0] for r in ref])
                ref_l = np.concatenate([r[1] for r in ref])
            else:
                ref_o, ref_l = orc.exact_attention(Q[0, hd][rows], K[0, hd], V[0, hd])
            assert_close(to_host(out[0, hd])[rows], ref_o, "bf16", f"out d={d} causal={causal} head {hd}")
            assert_lse_close(to_host(lse[0, hd])[rows], ref_l, "bf16", f"lse d={d} causal={causal} head {hd}")


@pytest.mark.parametrize("H,n,n_min,b,m,r,causal", [
    (3, 9999, 4096, 3, 40, 7, 0),       # three chunks, the last ragged; odd head offsets (no 16-byte key loads)
    (2, 12288, 4096, 256, 256, 8, 0),   # exactly three chunks, all 256 buckets in use
    (2, 8200, 4096, 8, 16, 1, 0),       # two buckets; 8 keys in the last chunk
    (2, 32768, 1024, 128, 64, 7, 1),    # causal: segments of 16384 ... 1024 keys = 4, 2, 1, 1, 1 chunks
    (1, 20480, 4096, 256, 300, 5, 0),   # five chunks, more samples than a block holds
])
def test_forward_with_segments_longer_than_a_sort_chunk(ha, torch, H, n, n_min, b, m, r, causal):
    """The forward sorts segments above 4096 keys in chunks, in two passes; codes, permutations,
    positions, the sampled keys' blocks and the outputs are compared with the oracle as everywhere."""
    print(f"chunked sort H={H} n={n} n_min={n_min} b={b} m={m} r={r} causal={causal}", flush=True)
    cfg = dict(B=1, H=H, n=n, d=64, dtype="bf16", law="iid", b=b, m=m, r=r, causal=causal, n_min=n_min, seed=n + r)
    Q, K, V = synth_inputs.make_qkv(cfg, seed=900 + n)
    _forward_and_compare(ha, torch, cfg, Q, K, V)


def _random_forward_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        dtype = str(rng.choice(["bf16", "bf16", "fp32"]))
        d = int(rng.choice([64, 128]))
        causal = int(rng.integers(0, 2))
        b = int(rng.choice([1, 3, 8, 16, 24, 32, 48, 64, 96, 128, 200, 256]))
        r = int(rng.integers(1, 9))
        m = int(rng.choice([0, 1, 2, 5, 16, 33, 64, 100, 256, 300]))
        if causal:
            n_min = b * int(rng.integers(1, 6))
            n = n_min * (1 << int(rng.integers(0, 6)))
        else:
            n_min = 4096
            n = b * int(rng.integers(1, 24))
        if n > 2500 or n < 2:
            continue
        cases.append((dtype, d, n, n_min, b, m, r, causal))
    return cases


@pytest.mark.parametrize("dtype,d,n,n_min,b,m,r,causal", _random_forward_cases(36, 7))
def test_forward_on_random_small_problems(ha, torch, dtype, d, n, n_min, b, m, r, causal):
    """Codes, permutations and outputs against the oracle on seeded random parameter combinations
    (both dtypes, block sizes that divide nothing in the kernels' tiling, tiny and oversized m)."""
    print(f"random forward {dtype} d={d} n={n} n_min={n_min} b={b} m={m} r={r} causal={causal}", flush=True)
    cfg = dict(B=1, H=2, n=n, d=d, dtype=dtype, law="iid", b=b, m=m, r=r, causal=causal, n_min=n_min, seed=3 * n + m)
    Q, K, V = synth_inputs.make_qkv(cfg, seed=500 + n + b)
    _forward_and_compare(ha, torch, cfg, Q, K, V)
