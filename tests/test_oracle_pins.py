"""Pins for the CPU oracle: it is checked here against what the paper and the
mathematics fix, never against itself or the HIP path.

  * Section 1.1 definition, re-derived by explicit loops on tiny inputs
  * degenerate cases in which HyperAttention must equal exact attention:
    one block and no samples; every key sampled exactly once (any b, r, seed);
    causal base case; causal recursion with identity sampling at every node
  * Definition 1: collision probability (1-theta/pi)^r and adjacent-bucket
    probability 2 theta/pi (1-theta/pi)^(r-1), cyclic in 2^r
  * Algorithm 1: M^H has exactly b ones per row and column; sort invariants
  * Algorithm 2: the estimator is unbiased for the unmasked row sum
  * Algorithm 4: lower-half row sums are D_21 + D_C22
"""
import math

import numpy as np
import pytest

from oracle import hyperattn_oracle as orc


def _rand_qkv(n, d, seed, scale=None):
    rng = np.random.default_rng(seed)
    scale = d ** -0.25 if scale is None else scale
    return tuple(rng.standard_normal((n, d)) * scale for _ in range(3))


def _loops_attention(Q, K, V, causal):
    """Section 1.1 / 3.1 with scalar loops: out_i = sum_j A_ij v_j / sum_j A_ij."""
    n, d = Q.shape
    dv = V.shape[1]
    out = np.zeros((n, dv))
    lse = np.zeros(n)
    for i in range(n):
        num = [0.0] * dv
        den = 0.0
        for j in range(K.shape[0]):
            if causal and j > i:
                continue
            a = math.exp(sum(Q[i, c] * K[j, c] for c in range(d)))
            den += a
            for c in range(dv):
                num[c] += a * V[j, c]
        out[i] = [x / den for x in num]
        lse[i] = math.log(den)
    return out, lse


@pytest.mark.parametrize("causal", [False, True])
def test_exact_attention_matches_scalar_loops(causal):
    Q, K, V = _rand_qkv(7, 3, seed=11, scale=0.8)
    out, lse = orc.exact_attention(Q, K, V, causal)
    ref_o, ref_l = _loops_attention(Q, K, V, causal)
    np.testing.assert_allclose(out, ref_o, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, ref_l, rtol=1e-12, atol=1e-14)


def test_exact_attention_is_not_transposed():
    # n_q != n_k makes a transposed operand fail on shape; values pin the rest.
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((4, 3)); K = rng.standard_normal((6, 3)); V = rng.standard_normal((6, 2))
    out, lse = orc.exact_attention(Q, K, V)
    ref_o, ref_l = _loops_attention(Q, K, V, False)
    np.testing.assert_allclose(out, ref_o, rtol=1e-12)
    np.testing.assert_allclose(lse, ref_l, rtol=1e-12)


# ---------------------------------------------------------------- generator
def test_splitmix_known_vector():
    # First output of SplitMix64 seeded with 0 (published reference value).
    assert orc._mix64(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF


def test_projection_is_standard_normal_and_bf16_representable():
    R = np.concatenate([orc.make_projection(s, 128, 8).ravel() for s in range(6)])
    assert R.shape[0] == 6 * 1024
    assert abs(R.mean()) < 4 / math.sqrt(R.size)
    assert abs(R.var() - 1.0) < 0.06
    # kurtosis of a normal is 3
    assert abs((R ** 4).mean() - 3.0) < 0.5
    bits = R.astype(np.float32).view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0)
    assert np.all(R.astype(np.float32).astype(np.float64) == R)
    # entry (c,k) does not depend on r or d
    np.testing.assert_array_equal(orc.make_projection(3, 64, 5), orc.make_projection(3, 128, 8)[:64, :5])


def test_samples_are_uniform_in_range():
    s = orc.make_samples(0, 0, 0, 1000, 20000)
    assert s.min() >= 0 and s.max() < 1000
    counts = np.bincount(s, minlength=1000)
    chi2 = ((counts - 20.0) ** 2 / 20.0).sum()
    assert 800 < chi2 < 1200        # 999 dof, +-4.5 sigma
    # different nodes draw different sets; the set does not depend on batch/head
    assert not np.array_equal(orc.make_samples(0, 1, 0, 1000, 64), orc.make_samples(0, 1, 1, 1000, 64))
    assert not np.array_equal(orc.make_samples(0, 1, 0, 1000, 64), orc.make_samples(1, 1, 0, 1000, 64))


# ---------------------------------------------------------------- Definition 1
def test_gray_rank_inverts_reflected_gray_code():
    for r in range(1, 9):
        rank = orc.gray_rank_table(r)
        assert sorted(rank.tolist()) == list(range(1 << r))
        for s in range(1 << r):
            i = int(rank[s])
            assert i ^ (i >> 1) == s
        # consecutive buckets (cyclically) differ in exactly one hyperplane
        inv = np.argsort(rank)
        for i in range(1 << r):
            diff = int(inv[i]) ^ int(inv[(i + 1) % (1 << r)])
            assert bin(diff).count("1") == 1


def test_negated_vector_gets_complement_word():
    r = 7
    R = orc.make_projection(2, 16, r)
    x = np.random.default_rng(0).standard_normal((50, 16))
    inv = np.argsort(orc.gray_rank_table(r))       # bucket -> word
    w_pos = inv[orc.lsh_codes(orc.lsh_project(x, R), r)]
    w_neg = inv[orc.lsh_codes(orc.lsh_project(-x, R), r)]
    np.testing.assert_array_equal(w_pos ^ w_neg, (1 << r) - 1)


@pytest.mark.parametrize("theta_frac,r", [(0.15, 7), (0.35, 4), (0.08, 7)])
def test_lsh_collision_and_adjacency_probabilities(theta_frac, r):
    """Monte-Carlo over hyperplane draws for a pair at angle theta."""
    theta = theta_frac * math.pi
    x = np.array([[1.0, 0.0, 0.0]])
    y = np.array([[math.cos(theta), math.sin(theta), 0.0]])
    trials = 6000
    same = adj = 0
    nb = 1 << r
    for seed in range(trials):
        R = orc.make_projection(1000 + seed, 3, r)
        cx = int(orc.lsh_codes(orc.lsh_project(x, R), r)[0])
        cy = int(orc.lsh_codes(orc.lsh_project(y, R), r)[0])
        same += cx == cy
        adj += ((cx - cy) % nb) in (1, nb - 1)
    p_same = (1 - theta / math.pi) ** r
    p_adj = 2 * theta / math.pi * (1 - theta / math.pi) ** (r - 1)
    for got, p in ((same, p_same), (adj, p_adj)):
        sigma = math.sqrt(p * (1 - p) / trials)
        assert abs(got / trials - p) < 4.5 * sigma, (got / trials, p)


# ---------------------------------------------------------------- Algorithm 1
def test_sort_invariants_and_mask_counts():
    rng = np.random.default_rng(3)
    n, b = 96, 16
    cq = rng.integers(0, 8, n); ck = rng.integers(0, 8, n)
    for codes in (cq, ck):
        perm, pos = orc.sort_lsh(codes)
        assert sorted(perm.tolist()) == list(range(n))
        np.testing.assert_array_equal(pos[perm], np.arange(n))
        sc = codes[perm]
        assert np.all(np.diff(sc) >= 0)
        ties = np.diff(sc) == 0
        assert np.all(np.diff(perm)[ties] > 0)      # equal codes keep row order
    _, pos_q = orc.sort_lsh(cq)
    _, pos_k = orc.sort_lsh(ck)
    M = (pos_q[:, None] // b) == (pos_k[None, :] // b)
    assert np.all(M.sum(axis=0) == b) and np.all(M.sum(axis=1) == b)


def test_block_part_equals_masked_attention():
    """block_part must be D_M^-1 (M^H . A) V with the mask of Algorithm 1."""
    n, d, b, r = 64, 8, 16, 4
    Q, K, V = _rand_qkv(n, d, seed=4)
    R = orc.make_projection(9, d, r)
    cq = orc.lsh_codes(orc.lsh_project(Q, R), r)
    ck = orc.lsh_codes(orc.lsh_project(K, R), r)
    perm_q, pos_q = orc.sort_lsh(cq)
    perm_k, pos_k = orc.sort_lsh(ck)
    O_b, L_b = orc.block_part(Q, K, V, perm_q, perm_k, b)
    M = (pos_q[:, None] // b) == (pos_k[None, :] // b)
    A = np.exp(Q @ K.T) * M
    np.testing.assert_allclose(O_b, (A @ V) / A.sum(1, keepdims=True), rtol=1e-11)
    np.testing.assert_allclose(L_b, np.log(A.sum(1)), rtol=1e-11)


# ---------------------------------------------------------------- degenerate = exact
def _as4(x):
    return x[None, None]


def test_one_block_no_samples_is_exact():
    n, d = 48, 8
    Q, K, V = _rand_qkv(n, d, seed=1)
    out, lse = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=n, m=0, r=5, seed=3)
    ref_o, ref_l = orc.exact_attention(Q, K, V)
    np.testing.assert_allclose(out[0, 0], ref_o, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(lse[0, 0], ref_l, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("b,r,seed", [(8, 3, 0), (16, 6, 5), (32, 1, 7)])
def test_identity_sampling_is_exact(b, r, seed):
    """m = n and l = (0..n-1): each unmasked key counted once with weight 1, so
    masked part + estimate is the full row sum whatever the LSH produced."""
    n, d = 64, 8
    Q, K, V = _rand_qkv(n, d, seed=seed + 20)
    ident = lambda level, node, n_keys: np.arange(n_keys)
    out, lse = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=b, m=n, r=r, seed=seed,
                                     sample_fn=ident)
    ref_o, ref_l = orc.exact_attention(Q, K, V)
    np.testing.assert_allclose(out[0, 0], ref_o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse[0, 0], ref_l, rtol=1e-10, atol=1e-12)


def test_duplicated_samples_count_with_multiplicity():
    """l = every key twice, m = 2n: weight n/m = 1/2 per hit, still exact."""
    n, d, b = 32, 4, 8
    Q, K, V = _rand_qkv(n, d, seed=2)
    twice = lambda level, node, n_keys: np.repeat(np.arange(n_keys), 2)
    out, lse = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=b, m=2 * n, r=4, seed=1,
                                     sample_fn=twice)
    ref_o, ref_l = orc.exact_attention(Q, K, V)
    np.testing.assert_allclose(out[0, 0], ref_o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse[0, 0], ref_l, rtol=1e-10, atol=1e-12)


def test_rows_are_normalised():
    n, d = 128, 8
    Q, K, _ = _rand_qkv(n, d, seed=9)
    V = np.ones((n, d))
    out, _ = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=16, m=24, r=5, seed=4)
    np.testing.assert_allclose(out, 1.0, rtol=1e-12)
    out, _ = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=16, m=24, r=5, seed=4,
                                   causal=True, n_min=32)
    np.testing.assert_allclose(out, 1.0, rtol=1e-12)


def test_estimator_is_unbiased_for_unmasked_row_sum():
    """E[(s/m) sum_j (1-M_{i,l_j}) exp<q_i,k_{l_j}>] = sum_j (1-M_ij) A_ij."""
    n, d, b, r, m = 64, 8, 16, 4, 16
    Q, K, V = _rand_qkv(n, d, seed=6, scale=0.45)
    R = orc.make_projection(0, d, r)
    _, pos_q = orc.sort_lsh(orc.lsh_codes(orc.lsh_project(Q, R), r))
    _, pos_k = orc.sort_lsh(orc.lsh_codes(orc.lsh_project(K, R), r))
    A = np.exp(Q @ K.T)
    unmasked = (pos_q[:, None] // b) != (pos_k[None, :] // b)
    target_den = (A * unmasked).sum(1)
    target_num = (A * unmasked) @ V
    trials = 1500
    dens = np.zeros((trials, n)); nums = np.zeros((trials, n, d))
    for t in range(trials):
        smp = orc.make_samples(t, 0, 0, n, m)
        O_r, L_r = orc.sampled_part(Q, K, V, pos_q, pos_k, b, smp)
        dens[t] = np.exp(L_r)
        nums[t] = np.exp(L_r)[:, None] * O_r
    se = dens.std(0, ddof=1) / math.sqrt(trials)
    assert np.all(np.abs(dens.mean(0) - target_den) < 5 * se)
    se_n = nums.std(0, ddof=1) / math.sqrt(trials)
    assert np.all(np.abs(nums.mean(0) - target_num) < 5.5 * se_n + 1e-12)


def test_all_samples_masked_gives_empty_residual():
    n, d, b = 16, 4, 16          # one block: every sample falls in the row's own block
    Q, K, V = _rand_qkv(n, d, seed=8)
    pos = np.arange(n)
    O_r, L_r = orc.sampled_part(Q, K, V, pos, pos, b, np.array([1, 5, 5]))
    assert np.all(L_r == -np.inf) and np.all(O_r == 0)
    O_b, L_b = orc.block_part(Q, K, V, pos, pos, b)
    O, L = orc.merge_parts(O_b, L_b, O_r, L_r)
    np.testing.assert_array_equal(O, O_b); np.testing.assert_array_equal(L, L_b)


# ---------------------------------------------------------------- Algorithm 4
def test_causal_base_case_is_exact():
    n, d = 40, 8
    Q, K, V = _rand_qkv(n, d, seed=12)
    out, lse = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=8, m=8, r=4, causal=True, n_min=64)
    ref_o, ref_l = orc.exact_attention(Q, K, V, causal=True)
    np.testing.assert_allclose(out[0, 0], ref_o, rtol=1e-12); np.testing.assert_allclose(lse[0, 0], ref_l, rtol=1e-12)


def test_causal_one_split_full_block_is_exact():
    n, d = 64, 8
    Q, K, V = _rand_qkv(n, d, seed=13)
    out, lse = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=32, m=0, r=4, causal=True, n_min=32)
    ref_o, ref_l = orc.exact_attention(Q, K, V, causal=True)
    np.testing.assert_allclose(out[0, 0], ref_o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse[0, 0], ref_l, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("n,n_min,b", [(128, 16, 8), (64, 32, 16)])
def test_causal_identity_sampling_is_exact_at_any_depth(n, n_min, b):
    d = 8
    Q, K, V = _rand_qkv(n, d, seed=14)
    ident = lambda level, node, n_keys: np.arange(n_keys)
    out, lse = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=b, m=0, r=5, causal=True,
                                     n_min=n_min, sample_fn=ident)
    ref_o, ref_l = orc.exact_attention(Q, K, V, causal=True)
    np.testing.assert_allclose(out[0, 0], ref_o, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(lse[0, 0], ref_l, rtol=1e-10, atol=1e-12)


def test_causal_row_sums_add_and_nodes_use_their_own_samples():
    """exp(lse) of the lower half = D_21 + D_C22, with D_21 from an unmasked
    node on (Q_2, K_1) drawing the (level 0, node 0) index set."""
    n, d, b, m, r, n_min, seed = 64, 8, 8, 8, 4, 32, 5
    Q, K, V = _rand_qkv(n, d, seed=15)
    out, lse = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=b, m=m, r=r, causal=True,
                                     n_min=n_min, seed=seed)
    h = n // 2
    R = orc.make_projection(seed, d, r)
    cq = orc.lsh_codes(orc.lsh_project(Q, R), r); ck = orc.lsh_codes(orc.lsh_project(K, R), r)
    O21, L21 = orc.node_forward(Q[h:], K[:h], V[:h], cq[h:], ck[:h], b,
                                orc.make_samples(seed, 0, 0, h, m))
    O22, L22 = orc.exact_attention(Q[h:], K[h:], V[h:], causal=True)
    np.testing.assert_allclose(np.exp(lse[0, 0, h:]), np.exp(L21) + np.exp(L22), rtol=1e-11)
    w = np.exp(L21) / (np.exp(L21) + np.exp(L22))
    np.testing.assert_allclose(out[0, 0, h:], w[:, None] * O21 + (1 - w)[:, None] * O22, rtol=1e-10, atol=1e-13)
    O1, L1 = orc.exact_attention(Q[:h], K[:h], V[:h], causal=True)
    np.testing.assert_allclose(out[0, 0, :h], O1, rtol=1e-12); np.testing.assert_allclose(lse[0, 0, :h], L1, rtol=1e-12)


def test_approximation_error_shrinks_with_more_samples():
    """Sanity on the method itself: more sampled columns, closer to exact."""
    n, d = 512, 16
    Q, K, V = _rand_qkv(n, d, seed=16)
    ref, _ = orc.exact_attention(Q, K, V)
    errs = []
    for m in (8, 128):
        e = 0.0
        for seed in range(4):
            out, _ = orc.hyperattn_forward(_as4(Q), _as4(K), _as4(V), b=32, m=m, r=4, seed=seed)
            e += np.linalg.norm(out[0, 0] - ref) / np.linalg.norm(ref)
        errs.append(e / 4)
    assert errs[1] < 0.6 * errs[0]


# --------------------------------------------------------------------------
# Backward pass of the oracle: pinned to central finite differences of the
# forward oracle (a different code path: no derivative formula is involved), to
# the dense textbook gradient of softmax attention where the method is exact,
# and to what row-stochasticity fixes.
# --------------------------------------------------------------------------
def _central_difference(f, X, idx, eps=1e-6):
    Xp, Xm = X.copy(), X.copy()
    Xp[idx] += eps
    Xm[idx] -= eps
    return (f(Xp) - f(Xm)) / (2 * eps)


@pytest.mark.parametrize("causal,n,n_min", [(False, 64, 16), (True, 64, 16), (True, 96, 24)])
def test_backward_matches_finite_differences_of_forward(causal, n, n_min):
    rng = np.random.default_rng(11 + n)
    d, b, m = 8, 8, 6
    Q, K, V, G = (rng.standard_normal((1, 2, n, d)) * 0.7 for _ in range(4))
    kw = dict(b=b, m=m, r=3, causal=causal, n_min=n_min, seed=5)
    dQ, dK, dV = orc.hyperattn_backward(Q, K, V, G, **kw)
    loss = lambda q, k, v: float((orc.hyperattn_forward(q, k, v, **kw)[0] * G).sum())
    for name, X, dX in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(16):
            idx = tuple(int(rng.integers(0, s)) for s in X.shape)
            f = {"Q": lambda x: loss(x, K, V), "K": lambda x: loss(Q, x, V), "V": lambda x: loss(Q, K, x)}[name]
            num = _central_difference(f, X, idx)
            assert abs(num - dX[idx]) <= 1e-6 * (1.0 + abs(num)), (name, idx, num, dX[idx])


def _dense_attention_gradients(Q, K, V, G, causal):
    """Softmax-attention gradients from the dense matrices (textbook form)."""
    S = Q @ K.T
    if causal:
        S = np.where(np.tril(np.ones_like(S, dtype=bool)), S, -np.inf)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    dP = G @ V.T
    dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
    return dS @ K, dS.T @ Q, P.T @ G


@pytest.mark.parametrize("causal", [False, True])
def test_backward_with_identity_sampling_is_exact_attention_gradient(causal):
    """Every key of every node sampled exactly once and one block per node... the
    forward is then exact attention, so its gradient must be the dense one."""
    rng = np.random.default_rng(3)
    n, d = 64, 8
    Q, K, V, G = (rng.standard_normal((1, 1, n, d)) * 0.6 for _ in range(4))
    ident = lambda level, node, n_keys: np.arange(n_keys)
    if causal:
        got = orc.hyperattn_backward(Q, K, V, G, b=8, m=0, r=3, causal=True, n_min=16, sample_fn=ident)
    else:
        got = orc.hyperattn_backward(Q, K, V, G, b=8, m=n, r=3, causal=False, sample_fn=ident)
    ref = _dense_attention_gradients(Q[0, 0], K[0, 0], V[0, 0], G[0, 0], causal)
    for g, r_ in zip(got, ref):
        np.testing.assert_allclose(g[0, 0], r_, rtol=1e-9, atol=1e-11)


def test_backward_invariants_from_row_stochasticity():
    rng = np.random.default_rng(8)
    n, d = 128, 8
    Q, K, V, G = (rng.standard_normal((1, 2, n, d)) for _ in range(4))
    kw = dict(b=16, m=12, r=4, causal=True, n_min=32, seed=2)
    dQ, dK, dV = orc.hyperattn_backward(Q, K, V, G, **kw)
    # the weights of every output row sum to one: the columns of dV add up to those of dO
    np.testing.assert_allclose(dV.sum(axis=2), G.sum(axis=2), rtol=1e-10, atol=1e-10)
    # identical value rows make the output constant in Q and K
    Vc = np.broadcast_to(V[:, :, :1], V.shape).copy()
    dQc, dKc, _ = orc.hyperattn_backward(Q, K, Vc, G, **kw)
    assert np.abs(dQc).max() < 1e-12 and np.abs(dKc).max() < 1e-12
    # linear in the cotangent
    dQ2, dK2, dV2 = orc.hyperattn_backward(Q, K, V, -2.0 * G, **kw)
    np.testing.assert_allclose(dQ2, -2.0 * dQ, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dK2, -2.0 * dK, rtol=1e-12, atol=1e-12)


def test_backward_absolute_bound_is_what_its_definition_says():
    """absolute=True: the dense closed form where the method is exact attention; a bound on
    |gradient| everywhere; blind to the signs of V and dO; homogeneous in dO; and large enough
    that perturbing every softmax weight by a relative eps moves no element by more than eps * bound."""
    rng = np.random.default_rng(5)
    n, d = 48, 6
    Q, K, V, G = (rng.standard_normal((1, 1, n, d)) * 0.8 for _ in range(4))
    q, k, v, g = Q[0, 0], K[0, 0], V[0, 0], G[0, 0]
    bq, bk, bv = (x[0, 0] for x in orc.hyperattn_backward(Q, K, V, G, b=n, m=0, r=2, absolute=True))
    S = q @ k.T
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    absO = P @ np.abs(v)
    dS = P * (np.abs(g) @ np.abs(v).T + (np.abs(g) * absO).sum(axis=1, keepdims=True))
    np.testing.assert_allclose(bq, dS @ np.abs(k), rtol=1e-12)
    np.testing.assert_allclose(bk, dS.T @ np.abs(q), rtol=1e-12)
    np.testing.assert_allclose(bv, P.T @ np.abs(g), rtol=1e-12)
    for kw in (dict(b=8, m=10, r=3, causal=False, seed=4), dict(b=4, m=5, r=3, causal=True, n_min=12, seed=4)):
        grads = orc.hyperattn_backward(Q, K, V, G, **kw)
        bounds = orc.hyperattn_backward(Q, K, V, G, absolute=True, **kw)
        for gr, bd in zip(grads, bounds):
            assert (bd >= 0).all() and (np.abs(gr) <= bd * (1 + 1e-12) + 1e-300).all()
        flipped = orc.hyperattn_backward(Q, K, -V, G * rng.choice([-1.0, 1.0], size=G.shape), absolute=True, **kw)
        scaled = orc.hyperattn_backward(Q, K, V, -3.0 * G, absolute=True, **kw)
        for bd, fl, sc in zip(bounds, flipped, scaled):
            np.testing.assert_allclose(fl, bd, rtol=1e-12)
            np.testing.assert_allclose(sc, 3.0 * bd, rtol=1e-12)
    # weights perturbed by a relative eps (what rounding them to fewer bits does), dense exact attention
    eps = 1e-3
    Pp = P * (1.0 + eps * rng.uniform(-1, 1, size=P.shape))
    dP = g @ v.T
    dSp = Pp * (dP - ((Pp @ v) * g).sum(axis=1, keepdims=True))
    exact = orc.hyperattn_backward(Q, K, V, G, b=n, m=0, r=2)
    for got, ref, bd in zip((dSp @ k, dSp.T @ q, Pp.T @ g), exact, (bq, bk, bv)):
        assert (np.abs(got - ref[0, 0]) <= 2.0 * eps * bd).all()


# --------------------------------------------------------------------------
# alpha, kappa and the epsilon of Eq. (1): closed forms
# --------------------------------------------------------------------------
def test_alpha_kappa_and_spectral_error_closed_forms():
    rng = np.random.default_rng(12)
    n, d, b = 64, 8, 8
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    Z = np.zeros((n, d))
    codes = rng.integers(0, 16, size=n)
    # Q = 0: uniform attention, every entry of D^-1 A is 1/n, so alpha = n * n * (1/n)^2 = 1, the matrix
    # is the rank-one projector (1/n) 1 1^T with norm 1, and every unmasked row sum is n - b: kappa = 1
    np.testing.assert_allclose(orc.attention_matrix(Z, K), 1.0 / n, rtol=1e-14)
    assert abs(orc.alpha(Z, K) - 1.0) < 1e-12
    assert abs(orc.kappa(Z, K, codes, codes[::-1].copy(), b) - 1.0) < 1e-12
    # one-hot attention (row i attends to key pi(i) only): D^-1 A is a permutation matrix, alpha = n
    pi = rng.permutation(n)
    E = np.eye(n)
    assert abs(orc.alpha(50.0 * E[pi], E) - n) < 1e-6
    # two keys share all the weight of every row equally: column norms^2 = n / 4 each, alpha = n * n / 4
    Kt = np.zeros((n, 2))
    Kt[3, 0] = Kt[9, 0] = 40.0
    Qt = np.zeros((n, 2))
    Qt[:, 0] = 1.0
    assert abs(orc.alpha(Qt, Kt) - n * n / 4.0) < 1e-6 * n * n
    # kappa on an instance with known row sums: scores 0 except one unmasked entry per row of size log(c_i)
    Kk = np.zeros((n, 1))
    Kk[0, 0] = 1.0
    cq = np.arange(n) // b                      # sorted already: row i in block i // b, key 0 in block 0
    c = rng.uniform(1.0, 9.0, size=n)
    Qk = np.log(c)[:, None]                     # A_i0 = c_i, all other entries 1
    sums = np.where(np.arange(n) < b, n - b, n - b - 1 + c)       # rows of block 0 have key 0 masked
    assert abs(orc.kappa(Qk, Kk, cq, cq, b) - sums.max() / sums.min()) < 1e-12
    # Eq. (1): zero for the exact product; for uniform attention (norm 1), orthonormal V (norm 1) and a
    # rank-one perturbation c u w^T with unit u, w the achieved epsilon is c
    Q = rng.standard_normal((n, d)) * 0.5
    att = orc.exact_attention(Q, K, V)[0]
    assert orc.spectral_error(att, Q, K, V) < 1e-14
    Vo = np.linalg.qr(rng.standard_normal((n, d)))[0]
    u = rng.standard_normal(n)
    w = rng.standard_normal(d)
    pert = 0.37 * np.outer(u / np.linalg.norm(u), w / np.linalg.norm(w))
    exact_u = orc.exact_attention(Z, K, Vo)[0]
    assert abs(orc.spectral_error(exact_u + pert, Z, K, Vo) - 0.37) < 1e-12
    # causal form: D_C^-1 (M^C . A) is lower triangular with unit row sums
    Pc = orc.attention_matrix(Q, K, causal=True)
    assert np.allclose(np.triu(Pc, 1), 0.0) and np.allclose(Pc.sum(axis=1), 1.0)
    assert orc.spectral_error(orc.exact_attention(Q, K, V, causal=True)[0], Q, K, V, causal=True) < 1e-14
    # identity sampling makes the method exact: epsilon = 0 (up to rounding)
    out, _ = orc.hyperattn_forward(Q[None, None], K[None, None], V[None, None], b=b, m=n, r=3,
                                   sample_fn=lambda level, node, s: np.arange(s))
    assert orc.spectral_error(out[0, 0], Q, K, V) < 1e-13


# --------------------------------------------------------------------------
# Frozen record of the oracle on tiny problems (tests/golden/, written by
# tests/golden/make_golden.py from the oracle alone): guards against an
# unnoticed change of its arithmetic; not an independent pin.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("case", ["unmasked_n32_d4", "causal_n32_d4"])
def test_oracle_matches_its_frozen_record(case):
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mg = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mg)
    with open(os.path.join(here, f"oracle_{case}.json")) as f:
        stored = json.load(f)
    now = mg.compute(case)
    for key, val in stored.items():
        np.testing.assert_allclose(np.asarray(now[key], dtype=np.float64), np.asarray(val, dtype=np.float64),
                                   rtol=1e-12, atol=1e-14, err_msg=f"{case}: {key}")


# --------------------------------------------------------------------------
# Algorithm 2 as printed (caps) and Lemma 2's value sampling
# --------------------------------------------------------------------------
def _alg2_inputs(n=96, d=8, seed=0, scale=0.8):
    rng = np.random.default_rng(seed)
    return tuple(rng.standard_normal((1, 1, n, d)) * scale for _ in range(3))


def test_alg2_without_caps_is_the_section4_forward():
    """Two independently written evaluations (dense here, part by part there) of the same estimator."""
    Q, K, V = _alg2_inputs()
    a = orc.hyperattn_forward(Q, K, V, b=16, m=20, r=4, seed=5)
    b_ = orc.hyperattn_forward_alg2(Q, K, V, b=16, m=20, r=4, seed=5)
    np.testing.assert_allclose(b_[0], a[0], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(b_[1], a[1], rtol=1e-12, atol=1e-13)


def test_alg2_tau_cap_and_lower_cap_follow_their_definitions():
    n, b, m, r, seed = 96, 16, 24, 4, 2
    Q, K, V = _alg2_inputs(n=n, seed=1)
    q, k = Q[0, 0], K[0, 0]
    R = orc.make_projection(seed, q.shape[1], r)
    _, pos_q = orc.sort_lsh(orc.lsh_codes(orc.lsh_project(q, R), r))
    _, pos_k = orc.sort_lsh(orc.lsh_codes(orc.lsh_project(k, R), r))
    A = np.exp(q @ k.T)
    Mh = (pos_q[:, None] // b) == (pos_k[None, :] // b)
    masked = (A * Mh).sum(axis=1)
    unmasked = (A * ~Mh).sum(axis=1)
    T = orc.tau_rows(seed, n, m)
    assert T.min() >= 0 and T.max() < n and len(T) == m
    tau = unmasked[T].max()
    samples = orc.make_samples(seed, 0, 0, n, m)
    kept = (~Mh[:, samples]).sum(axis=1)
    # a cap far below every entry: every kept sample contributes exactly C_i
    cap_scale, kappa = 1e-6, 2.5
    out, log_dt, log_tau = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, cap_scale=cap_scale, kappa=kappa)
    np.testing.assert_allclose(np.exp(log_tau[0]), tau, rtol=1e-12)
    C = cap_scale * m / (n * math.log(n)) * (masked + tau / kappa)
    d_i = (n / m) * kept * C
    np.testing.assert_allclose(np.exp(log_dt[0, 0]), masked + np.maximum(d_i, tau / kappa), rtol=1e-11)
    # a cap above every entry changes nothing; the lower cap alone acts as max(d_i, tau / kappa)
    big = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, cap_scale=1e12, kappa=kappa)
    d_plain = (n / m) * (A[:, samples] * ~Mh[:, samples]).sum(axis=1)
    np.testing.assert_allclose(np.exp(big[1][0, 0]), masked + np.maximum(d_plain, tau / kappa), rtol=1e-11)
    assert (np.maximum(d_plain, tau / kappa) > d_plain).any()      # the lower cap binds somewhere in this instance


def test_causal_alg2_is_algorithm4_over_algorithm2():
    """Causal problems: with the caps off the result is the Section 4 causal forward (dense per-node
    evaluation here, part by part there); at n <= n_min it is exact causal attention; the row sum of a
    lower-half row is the node's D~ (a direct call of the node with that node's draws) plus the
    diagonal block's; every node has its own T."""
    n, d, b, m, r, n_min, seed = 128, 8, 8, 12, 4, 32, 6
    Q, K, V = _alg2_inputs(n=n, d=d, seed=3)
    plain = orc.hyperattn_forward(Q, K, V, b=b, m=m, r=r, causal=True, n_min=n_min, seed=seed)
    got = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, causal=True, n_min=n_min)
    np.testing.assert_allclose(got[0], plain[0], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(got[1], plain[1], rtol=1e-11, atol=1e-12)
    assert got[2].shape == (1, 3) and np.isfinite(got[2]).all()          # two levels: nodes 0, 1, 2 in heap order
    ex = orc.exact_attention(Q[0, 0], K[0, 0], V[0, 0], causal=True)
    small = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, causal=True, n_min=n, cap_scale=3.0, kappa=1.5)
    np.testing.assert_allclose(small[0][0, 0], ex[0], rtol=1e-12)
    assert small[2].shape == (1, 0)
    # with caps: top split.  Lower half = node (Q_2, K_1, V_1) with the draws of (level 0, node 0), merged with
    # the causal result of the lower-right block, itself the recursion on (Q_2, K_2, V_2) as nodes (1, 1), ...
    cap_scale, kappa = 6.0, 1.3
    out, lse, taus = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, causal=True, n_min=n_min,
                                                cap_scale=cap_scale, kappa=kappa, vnorm_sampling=True)
    h = n // 2
    q, k, v = Q[0, 0], K[0, 0], V[0, 0]
    R = orc.make_projection(seed, d, r)
    cq, ck = orc.lsh_codes(orc.lsh_project(q, R), r), orc.lsh_codes(orc.lsh_project(k, R), r)
    vs = orc.vnorm_samples(v[:h], seed, 0, m, heap=0, n_heads=1)
    O21, L21, t21 = orc.alg2_head_forward(q[h:], k[:h], v[:h], cq[h:], ck[:h], b, orc.make_samples(seed, 0, 0, h, m),
                                          orc.tau_rows(seed, h, m, heap=0), cap_scale, kappa, vs)
    assert abs(taus[0, 0] - t21) < 1e-12
    # lower-right block on its own is a causal problem whose root is heap node 2 of the full problem: rebuild it
    # from the full result by subtraction of row sums
    L22 = np.log(np.exp(lse[0, 0, h:]) - np.exp(L21))
    w21 = np.exp(L21 - lse[0, 0, h:])
    O22 = (out[0, 0, h:] - w21[:, None] * O21) / (1.0 - w21)[:, None]
    # its first quarter (rows h .. h + n_min) is an exact causal base block
    ex22 = orc.exact_attention(q[h:h + n_min], k[h:h + n_min], v[h:h + n_min], causal=True)
    np.testing.assert_allclose(L22[:n_min], ex22[1], rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(O22[:n_min], ex22[0], rtol=1e-7, atol=1e-9)
    # the caps act in this instance, and the nodes' subsets T differ
    plain_v = orc.hyperattn_forward_alg2(Q, K, V, b=b, m=m, r=r, seed=seed, causal=True, n_min=n_min)
    assert np.abs(plain_v[1] - lse).max() > 1e-3
    assert not np.array_equal(orc.tau_rows(seed, 32, m, heap=1), orc.tau_rows(seed, 32, m, heap=2))
    assert np.array_equal(orc.tau_rows(seed, 64, m, heap=0), orc.tau_rows(seed, 64, m))


def test_tau_rows_are_uniform_and_independent_of_the_samples():
    """T of Algorithm 2: m uniform rows.  A chi-square test over many seeds pins the law (a biased or
    truncated draw fails it); T must also not repeat the estimator's own index set."""
    n, m, seeds = 64, 256, 40
    counts = np.zeros(n)
    for s in range(seeds):
        T = orc.tau_rows(s, n, m)
        assert T.shape == (m,) and T.min() >= 0 and T.max() < n
        counts += np.bincount(T, minlength=n)
    expected = seeds * m / n
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 63 + 5 * math.sqrt(2 * 63), chi2            # mean n-1, sd sqrt(2(n-1))
    assert chi2 > 63 - 5 * math.sqrt(2 * 63), chi2            # nor suspiciously regular (a stride would be)
    # both ends of the range occur, also for n that is no power of two
    T = np.concatenate([orc.tau_rows(s, 1000, 300) for s in range(30)])
    assert T.min() < 5 and T.max() > 994
    # serial independence: consecutive draws are uncorrelated
    T = orc.tau_rows(7, 1 << 20, 4000).astype(np.float64)
    assert abs(np.corrcoef(T[:-1], T[1:])[0, 1]) < 5 / math.sqrt(4000)
    assert not np.array_equal(orc.tau_rows(3, 4096, 64), orc.make_samples(3, 0, 0, 4096, 64))


def test_vnorm_sampling_weights_distribution_and_unbiasedness():
    n, d, m = 48, 6, 16
    rng = np.random.default_rng(4)
    Q, K = (rng.standard_normal((1, 1, n, d)) * 0.7 for _ in range(2))
    V = rng.standard_normal((1, 1, n, d)) * rng.uniform(0.1, 3.0, size=(1, 1, n, 1))      # very unequal row norms
    p = orc.vnorm_probabilities(V[0, 0])
    # Lemma 2's law, retyped with a scalar loop
    w = np.array([sum(x * x for x in row) for row in V[0, 0]])
    np.testing.assert_allclose(p, w / w.sum(), rtol=1e-13)
    np.testing.assert_allclose(orc.vnorm_probabilities(np.zeros((5, 3))), 0.2)
    # a zero row is never drawn; a single non-zero row is always drawn, with rescaling 1/m
    Vz = np.zeros((7, 3))
    Vz[4] = [1.0, -2.0, 0.5]
    idx, logw = orc.vnorm_samples(Vz, 1, 0, 9)
    assert (idx == 4).all()
    np.testing.assert_allclose(logw, -math.log(9))
    # the margin of every draw is its uniform's distance to the nearest boundary of the cumulative law
    marg = []
    idx, _ = orc.vnorm_samples(V[0, 0], 5, 0, m, margin=marg)
    cdf = np.concatenate([[0.0], np.cumsum(p)])
    u = orc.vnorm_uniforms(5, 0, m)
    for r_ in range(m):
        assert cdf[idx[r_]] <= u[r_] < cdf[idx[r_] + 1]
        assert abs(marg[r_] - min(u[r_] - cdf[idx[r_]], cdf[idx[r_] + 1] - u[r_])) < 1e-15
    assert orc.vnorm_samples(V[0, 0], 5, 0, m, replay={3: 11})[0][3] == 11
    # draws follow p_l, and E[A S^T S V] = A V (Lemma 2's sampling matrix is unbiased)
    A = np.exp(Q[0, 0] @ K[0, 0].T)
    exact = A @ V[0, 0]
    acc = np.zeros_like(exact)
    counts = np.zeros(n)
    trials = 3000
    for s in range(trials):
        idx, logw = orc.vnorm_samples(V[0, 0], s, 0, m)
        acc += (A[:, idx] * np.exp(logw)[None, :]) @ V[0, 0][idx]
        counts += np.bincount(idx, minlength=n)
    assert np.abs(counts / (trials * m) - p).max() < 5 * np.sqrt(p.max() / (trials * m))
    rel = np.linalg.norm(acc / trials - exact) / np.linalg.norm(exact)
    assert rel < 0.05, rel
    # the sampled value product with D~ of the same call reproduces out
    out, log_dt, _ = orc.hyperattn_forward_alg2(Q, K, V, b=8, m=m, r=3, seed=9, vnorm_sampling=True)
    idx, logw = orc.vnorm_samples(V[0, 0], 9, 0, m)
    np.testing.assert_allclose(out[0, 0], ((A[:, idx] * np.exp(logw)[None, :]) @ V[0, 0][idx]) / np.exp(log_dt[0, 0])[:, None],
                               rtol=1e-11)
