"""CPU oracle for the HyperAttention forward pass (arXiv 2310.05869).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 NumPy implementation
written from the paper, used by the tests, by the smoke check and by the
benchmark's CPU-baseline leg to judge the HIP path.  It shares no code with the
HIP library and must never be imported by the product package.

HyperAttention is an approximation, so apart from `exact_attention` (which is
the definition of Section 1.1 written out) every function here follows the
algorithm's steps in the paper's order and notation:

  exact_attention      Section 1.1: Att = D^-1 A V, A = exp(Q K^T); Section 3.1
                       for the causal form D_C^-1 (M^C . A) V
  make_projection      Definition 1 read as r random hyperplanes (sign of a
                       Gaussian projection), the family whose collision
                       probability is exactly (1 - theta/pi)^r
  lsh_project/lsh_codes  Definition 1 + Algorithm 1 step "hash rows of Q, K";
                       buckets numbered by their position in the reflected
                       binary Gray code, so buckets i and i+-1 (mod 2^r) differ
                       in exactly one hyperplane
  sort_lsh             Algorithm 1: permutations P_Q, P_K ordering rows by hash
  block_part           Algorithm 1 mask M^H (equal floor(P/b)) evaluated as in
                       the Implementation Detail paragraph of Section 4: the
                       i-th group of sorted queries against the i-th group of
                       sorted keys
  sampled_part         Algorithm 2, the estimator d_i = (n/m) sum_j (1-M_{i,l_j})
                       exp<q_i, k_{l_j}> with one index set shared by all rows
                       and reused for the value product (Section 4,
                       Implementation Detail), without the cap C_i and the
                       lower cap, which that paragraph leaves out
  merge_parts          Algorithm 2, last step: row sum = masked part + estimate
  causal_forward       Algorithm 4 with the outputs combined by the same
                       row-sum weights (D_21 + D_C22)
  hyperattn_forward    Algorithm 3 in its Section 4 form over [B, H, n, d]
  hyperattn_forward_alg2  Algorithm 2 as printed (cap C_i, tau from a row subset,
                       lower cap tau / kappa) and Lemma 2 / Algorithm 3's value
                       product D~^-1 A S^T S V with rows drawn by squared norm,
                       evaluated densely (small n); the unspecified constants
                       are caller's numbers
  hyperattn_backward   the forward's vector-Jacobian product (Section 4.2 times
                       forward + backward), random draws held fixed, written
                       out part by part in the forward's structure
  attention_matrix, alpha, kappa, spectral_error
                       the quantities the guarantees are stated in, from the dense
                       matrices: D^-1 A; Lemma 1's alpha = n max_j |D^-1 A e_j|^2
                       and kappa = max / min unmasked row sum; the epsilon of
                       Eq. (1), |Att~ - Att|_op / (|D^-1 A|_op |V|_op)

Pins (tests/test_oracle_pins.py): brute-force equivalence in the degenerate
cases (one block and no samples; causal base case; every key sampled exactly
once), the closed-form collision and adjacent-bucket probabilities of
Definition 1, unbiasedness of the estimator, row-stochasticity (V = 1 gives
out = 1), permutation/stability invariants of the sort, and additivity of the
causal row sums; for the backward pass central finite differences of the
forward, the dense softmax-attention gradient where the method is exact, and
the identities row-stochasticity implies.  At the full benchmark configurations the randomised output
itself has no independent pin beyond these (no worked example is printed in
the paper): there the oracle is trusted as the same code that passed them.
"""
from __future__ import annotations

import math

import numpy as np

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15

STREAM_PROJECTION = 1      # counter stream of the hyperplane matrix R
STREAM_SAMPLES = 2         # + heap index of the node: counter stream of its samples


# --------------------------------------------------------------------------
# Counter-based random numbers (the method's random draws).  The HIP library
# implements the same generator independently; a test compares the two.
# --------------------------------------------------------------------------
def _mix64(z: int) -> int:
    """SplitMix64 output function (Steele, Lea, Flood 2014)."""
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def rand_u64(seed: int, stream: int, ctr: int) -> int:
    key = _mix64(seed + _GOLDEN * (stream + 1))
    return _mix64(key + _GOLDEN * (ctr + 1))


def _unit_open(u: int) -> float:
    """Top 53 bits of u mapped to the open interval (0, 1)."""
    return ((u >> 11) + 0.5) * (2.0 ** -53)


def _round_fp32_to_bf16(x: np.ndarray) -> np.ndarray:
    bits = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    bits = bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))
    return (bits & np.uint64(0xFFFF0000)).astype(np.uint32).view(np.float32)


def make_projection(seed: int, d: int, r: int) -> np.ndarray:
    """R in R^{d x r}: i.i.d. N(0,1) hyperplane normals (Definition 1).

    Entry (c, k) is a Box-Muller normal from counters 2*(8c+k), 2*(8c+k)+1 of
    the projection stream, rounded to fp32 and then to the nearest bf16 value,
    so that products with bf16 inputs are exact in fp32.  Returned as fp64.
    """
    R = np.empty((d, r), dtype=np.float64)
    for c in range(d):
        for k in range(r):
            ctr = 2 * (8 * c + k)
            u1 = _unit_open(rand_u64(seed, STREAM_PROJECTION, ctr))
            u2 = _unit_open(rand_u64(seed, STREAM_PROJECTION, ctr + 1))
            R[c, k] = math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2)
    return _round_fp32_to_bf16(R.astype(np.float32)).astype(np.float64).reshape(d, r)


def make_samples(seed: int, level: int, node: int, n_keys: int, m: int) -> np.ndarray:
    """l_1..l_m i.i.d. uniform on [0, n_keys), with replacement (Algorithm 2).

    One index set per node of the causal recursion (level 0, node 0 for the
    unmasked problem), shared by every batch, head and query row.
    """
    stream = STREAM_SAMPLES + (1 << level) + node
    out = np.empty(m, dtype=np.int64)
    for j in range(m):
        hi = rand_u64(seed, stream, j) >> 32
        out[j] = (hi * n_keys) >> 32
    return out


# --------------------------------------------------------------------------
# Section 1.1 / 3.1: the definition (brute force; small n only)
# --------------------------------------------------------------------------
def exact_attention(Q, K, V, causal=False):
    """Att = D^-1 A V with A = exp(Q K^T) (no 1/sqrt(d)); returns (Att, log D)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    S = Q @ K.T
    if causal:
        i = np.arange(S.shape[0])[:, None]
        j = np.arange(S.shape[1])[None, :]
        S = np.where(i >= j, S, -np.inf)          # M^C_{ij} = 1{i >= j}
    mx = S.max(axis=1, keepdims=True)
    A = np.exp(S - mx)
    D = A.sum(axis=1, keepdims=True)
    return (A @ V) / D, (mx + np.log(D))[:, 0]


# --------------------------------------------------------------------------
# Definition 1 + Algorithm 1: sortLSH
# --------------------------------------------------------------------------
def lsh_project(X, R):
    """p[i, k] = <x_i, R[:, k]> in fp64."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(R, dtype=np.float64)


def gray_rank_table(r: int) -> np.ndarray:
    """rank[s] = position of the r-bit word s in the reflected Gray sequence."""
    rank = np.empty(1 << r, dtype=np.int64)
    for i in range(1 << r):
        rank[i ^ (i >> 1)] = i
    return rank


def lsh_bits(p) -> np.ndarray:
    """Sign bits: bit k of a row is 1 iff its projection on hyperplane k is > 0."""
    return np.asarray(p) > 0


def codes_from_bits(bits, r: int) -> np.ndarray:
    """Bucket index: hyperplane k contributes bit k of the word; the bucket is
    the word's position in the reflected Gray sequence."""
    word = np.zeros(bits.shape[0], dtype=np.int64)
    for k in range(r):
        word |= bits[:, k].astype(np.int64) << k
    return gray_rank_table(r)[word]


def lsh_codes(p, r: int) -> np.ndarray:
    """Bucket index of each row from its r projections."""
    return codes_from_bits(lsh_bits(p), r)


def sort_lsh(codes):
    """Algorithm 1: perm[pos] = row, rows ordered by bucket; ties keep the
    original row order (any order satisfies the algorithm; this one is unique).
    Returns (perm, pos) with pos[perm[p]] == p."""
    perm = np.argsort(np.asarray(codes), kind="stable")
    pos = np.empty_like(perm)
    pos[perm] = np.arange(perm.shape[0])
    return perm, pos


# --------------------------------------------------------------------------
# One unmasked node: s queries against s keys (Algorithms 1-3, Section 4 form)
# --------------------------------------------------------------------------
def block_part(Qn, Kn, Vn, perm_q, perm_k, b):
    """Entries selected by M^H: sorted query group t against sorted key group t.

    Returns (O_b, LSE_b) in the node's original row order: the normalised
    output of the masked entries and the log of their row sum."""
    s = Qn.shape[0]
    O = np.zeros((s, Vn.shape[1]), dtype=np.float64)
    L = np.full(s, -np.inf, dtype=np.float64)
    for t in range(s // b):
        I = perm_q[t * b:(t + 1) * b]
        J = perm_k[t * b:(t + 1) * b]
        S = Qn[I] @ Kn[J].T
        mx = S.max(axis=1, keepdims=True)
        A = np.exp(S - mx)
        den = A.sum(axis=1, keepdims=True)
        O[I] = (A @ Vn[J]) / den
        L[I] = (mx + np.log(den))[:, 0]
    return O, L


def sampled_part(Qn, Kn, Vn, pos_q, pos_k, b, samples):
    """Algorithm 2's estimator of the unmasked row sum and, with the same
    indices, of the unmasked part of A V.

    den_i = (s/m) sum_j (1 - M_{i,l_j}) exp<q_i, k_{l_j}>, and the numerator
    carries v_{l_j} along.  Returns (O_r, LSE_r) with LSE_r = log den (-inf and
    a zero row when every sample of a row is masked, or m = 0)."""
    s = Qn.shape[0]
    m = len(samples)
    O = np.zeros((s, Vn.shape[1]), dtype=np.float64)
    L = np.full(s, -np.inf, dtype=np.float64)
    if m == 0:
        return O, L
    samples = np.asarray(samples, dtype=np.int64)
    S = Qn @ Kn[samples].T                                         # s x m
    keep = (pos_q[:, None] // b) != (pos_k[samples][None, :] // b)  # 1 - M
    S = np.where(keep, S, -np.inf)
    mx = S.max(axis=1, keepdims=True)
    live = np.isfinite(mx[:, 0])
    mx = np.where(np.isfinite(mx), mx, 0.0)
    A = np.exp(S - mx)
    den = A.sum(axis=1)
    num = A @ Vn[samples]
    O[live] = num[live] / den[live][:, None]
    L[live] = mx[live, 0] + np.log(den[live]) + math.log(s / m)
    return O, L


def merge_parts(O1, L1, O2, L2):
    """Row sums add (d~_i = masked part + estimate); outputs are combined with
    the corresponding weights.  L = log(exp L1 + exp L2)."""
    L = np.logaddexp(L1, L2)
    with np.errstate(invalid="ignore"):
        w1 = np.where(np.isfinite(L1), np.exp(L1 - L), 0.0)
        w2 = np.where(np.isfinite(L2), np.exp(L2 - L), 0.0)
    return w1[:, None] * O1 + w2[:, None] * O2, L


def node_forward(Qn, Kn, Vn, codes_q, codes_k, b, samples, parts=None):
    """Unmasked HyperAttention on one node: sortLSH, masked part, estimate."""
    perm_q, pos_q = sort_lsh(codes_q)
    perm_k, pos_k = sort_lsh(codes_k)
    O_b, L_b = block_part(Qn, Kn, Vn, perm_q, perm_k, b)
    O_r, L_r = sampled_part(Qn, Kn, Vn, pos_q, pos_k, b, samples)
    if parts is not None:
        parts.update(perm_q=perm_q, perm_k=perm_k, pos_q=pos_q, pos_k=pos_k,
                     O_b=O_b, L_b=L_b, O_r=O_r, L_r=L_r)
    return merge_parts(O_b, L_b, O_r, L_r)


# --------------------------------------------------------------------------
# Algorithm 4: causal masking by recursive halving
# --------------------------------------------------------------------------
def causal_forward(Q, K, V, codes_q, codes_k, b, n_min, sample_fn, level=0, node=0):
    """Returns (out, lse) for causal attention on n rows.

    n <= n_min: the definition (exact causal attention).  Otherwise the two
    diagonal halves recurse and the off-diagonal block A_21 = (Q_2, K_1, V_1)
    is an unmasked node; the lower half's row sum is D_21 + D_C22."""
    n = Q.shape[0]
    if n <= n_min:
        return exact_attention(Q, K, V, causal=True)
    h = n // 2
    O1, L1 = causal_forward(Q[:h], K[:h], V[:h], codes_q[:h], codes_k[:h], b, n_min,
                            sample_fn, level + 1, 2 * node)
    O22, L22 = causal_forward(Q[h:], K[h:], V[h:], codes_q[h:], codes_k[h:], b, n_min,
                              sample_fn, level + 1, 2 * node + 1)
    O21, L21 = node_forward(Q[h:], K[:h], V[:h], codes_q[h:], codes_k[:h], b,
                            sample_fn(level, node, h))
    O2, L2 = merge_parts(O21, L21, O22, L22)
    return np.concatenate([O1, O2]), np.concatenate([L1, L2])


# --------------------------------------------------------------------------
# Whole forward pass over [B, H, n, d]
# --------------------------------------------------------------------------
def hyperattn_forward(Q, K, V, b, m, r, causal=False, n_min=4096, seed=0,
                      R=None, sample_fn=None, flip=None, stages=None):
    """HyperAttention forward.  Q, K, V: [B, H, n, d] (already rounded to the
    storage dtype).  R / sample_fn override the seed-derived hyperplanes and
    per-node index sets.  `flip`, if given, is a list of (tensor, bh, row, k)
    sign bits to invert before bucketing (tensor 0 = Q, 1 = K): used to follow
    the HIP path through projections too close to zero to call.  `stages`, if
    a dict, receives codes and (unmasked case) the per-head intermediate
    parts.  Returns (out [B,H,n,d], lse [B,H,n]) in fp64."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, n, d = Q.shape
    if R is None:
        R = make_projection(seed, d, r)
    if sample_fn is None:
        def sample_fn(level, node, n_keys):
            return make_samples(seed, level, node, n_keys, m)
    dv = V.shape[-1]                      # V may be wider or narrower than Q, K
    out = np.empty((B, H, n, dv), dtype=np.float64)
    lse = np.empty((B, H, n), dtype=np.float64)
    all_codes = np.empty((2, B * H, n), dtype=np.int64)
    all_proj = np.empty((2, B * H, n, r), dtype=np.float64)
    for bh in range(B * H):
        q, k = (x.reshape(B * H, n, d)[bh] for x in (Q, K))
        v = V.reshape(B * H, n, dv)[bh]
        pq, pk = lsh_project(q, R), lsh_project(k, R)
        all_proj[0, bh], all_proj[1, bh] = pq, pk
        bits = [lsh_bits(pq), lsh_bits(pk)]
        if flip:
            for (t, fbh, row, kk) in flip:
                if fbh == bh:
                    bits[t][row, kk] = ~bits[t][row, kk]
        codes = [codes_from_bits(bits[t], r) for t in range(2)]
        cq, ck = codes
        all_codes[0, bh], all_codes[1, bh] = cq, ck
        if causal:
            o, l = causal_forward(q, k, v, cq, ck, b, n_min, sample_fn)
        else:
            parts = {} if stages is not None else None
            o, l = node_forward(q, k, v, cq, ck, b, sample_fn(0, 0, n), parts)
            if stages is not None:
                stages.setdefault("parts", []).append(parts)
        out.reshape(B * H, n, dv)[bh] = o
        lse.reshape(B * H, n)[bh] = l
    if stages is not None:
        stages["codes"] = all_codes
        stages["proj"] = all_proj
    return out, lse


# --------------------------------------------------------------------------
# Backward pass: the vector-Jacobian product of the forward map above, with the
# random draws (hyperplanes, index sets) and hence the permutations held fixed
# (they are piecewise constant in Q and K).  The paper times forward + backward
# (Section 4.2) and obtains the backward by differentiating its forward; this is
# that derivative written out part by part, in the forward's own structure.
# Every part is "O = A V / den, L = log den" for some non-negative A = w . exp(S);
# with cotangents (dO, dL):  P = A / den,  dV = P^T dO,
#   dS = P . (dO V^T - <dO, O>) + P dL,  dQ = dS K,  dK = dS^T Q.
# --------------------------------------------------------------------------
def _softmax_part_backward(Qs, Ks, Vs, S_mask, O, L, dO, dL, absolute=False):
    """Cotangents of one part.  Qs [a,d], Ks, Vs [c,*]; S_mask [a,c] boolean
    (True = entry present); O, L the part's outputs (L without additive
    constants matters only through P, which is recomputed here); returns
    (dQs, dKs, dVs).  absolute: the bound described at hyperattn_backward; Vs and
    dO are then non-negative and dL carries, per row, this part's share of
    <|dO_i|, sum_j P_ij |v_j|> of the whole row."""
    S = Qs @ Ks.T
    S = np.where(S_mask, S, -np.inf)
    mx = S.max(axis=1, keepdims=True)
    live = np.isfinite(mx[:, 0])
    mx = np.where(np.isfinite(mx), mx, 0.0)
    A = np.exp(S - mx)
    den = A.sum(axis=1, keepdims=True)
    P = np.where(live[:, None], A / np.where(den > 0, den, 1.0), 0.0)
    dP = dO @ Vs.T
    delta = (dO * O).sum(axis=1, keepdims=True)
    dLc = np.where(live, dL, 0.0)[:, None]
    if absolute:
        dS = P * (dP + dLc)
        return dS @ np.abs(Ks), dS.T @ np.abs(Qs), P.T @ dO
    dS = P * (dP - delta + dLc)
    return dS @ Ks, dS.T @ Qs, P.T @ dO


def _merge_backward(O1, L1, O2, L2, O, L, dO, dL, absolute=False):
    """Cotangents of merge_parts: returns (dO1, dL1, dO2, dL2)."""
    with np.errstate(invalid="ignore"):
        w1 = np.where(np.isfinite(L1), np.exp(L1 - L), 0.0)
        w2 = np.where(np.isfinite(L2), np.exp(L2 - L), 0.0)
    if absolute:   # a part's weights are w times the row's final ones: everything scales by w
        return w1[:, None] * dO, w1 * dL, w2[:, None] * dO, w2 * dL
    g = (dO * O).sum(axis=1)
    dL1 = w1 * (dL + (dO * O1).sum(axis=1) - g)
    dL2 = w2 * (dL + (dO * O2).sum(axis=1) - g)
    return w1[:, None] * dO, dL1, w2[:, None] * dO, dL2


def node_backward(Qn, Kn, Vn, codes_q, codes_k, b, samples, dO, dL, absolute=False):
    """Backward of node_forward; returns (dQn, dKn, dVn)."""
    s = Qn.shape[0]
    parts = {}
    O, L = node_forward(Qn, Kn, Vn, codes_q, codes_k, b, samples, parts)
    dO_b, dL_b, dO_r, dL_r = _merge_backward(parts["O_b"], parts["L_b"], parts["O_r"], parts["L_r"], O, L, dO, dL,
                                             absolute)
    dQ = np.zeros_like(Qn)
    dK = np.zeros_like(Kn)
    dV = np.zeros_like(Vn)
    perm_q, perm_k, pos_q, pos_k = parts["perm_q"], parts["perm_k"], parts["pos_q"], parts["pos_k"]
    for t in range(s // b):                       # masked part, block by block
        I = perm_q[t * b:(t + 1) * b]
        J = perm_k[t * b:(t + 1) * b]
        full = np.ones((len(I), len(J)), dtype=bool)
        gq, gk, gv = _softmax_part_backward(Qn[I], Kn[J], Vn[J], full, parts["O_b"][I], parts["L_b"][I], dO_b[I],
                                            dL_b[I], absolute)
        dQ[I] += gq
        dK[J] += gk
        dV[J] += gv
    samples = np.asarray(samples, dtype=np.int64)
    if len(samples) > 0:                          # estimate: the same index set for every row
        keep = (pos_q[:, None] // b) != (pos_k[samples][None, :] // b)
        gq, gk, gv = _softmax_part_backward(Qn, Kn[samples], Vn[samples], keep, parts["O_r"], parts["L_r"], dO_r, dL_r,
                                            absolute)
        dQ += gq
        np.add.at(dK, samples, gk)                # an index may be drawn more than once
        np.add.at(dV, samples, gv)
    return dQ, dK, dV


def causal_backward(Q, K, V, codes_q, codes_k, b, n_min, sample_fn, dO, dL, level=0, node=0, absolute=False):
    """Backward of causal_forward; returns (dQ, dK, dV)."""
    n = Q.shape[0]
    if n <= n_min:
        O, L = exact_attention(Q, K, V, causal=True)
        i = np.arange(n)[:, None]
        j = np.arange(n)[None, :]
        return _softmax_part_backward(Q, K, V, i >= j, O, L, dO, dL, absolute)
    h = n // 2
    O22, L22 = causal_forward(Q[h:], K[h:], V[h:], codes_q[h:], codes_k[h:], b, n_min, sample_fn, level + 1, 2 * node + 1)
    samples = sample_fn(level, node, h)
    O21, L21 = node_forward(Q[h:], K[:h], V[:h], codes_q[h:], codes_k[:h], b, samples)
    O2, L2 = merge_parts(O21, L21, O22, L22)
    dO21, dL21, dO22, dL22 = _merge_backward(O21, L21, O22, L22, O2, L2, dO[h:], dL[h:], absolute)
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    g = causal_backward(Q[:h], K[:h], V[:h], codes_q[:h], codes_k[:h], b, n_min, sample_fn, dO[:h], dL[:h], level + 1,
                        2 * node, absolute)
    dQ[:h] += g[0]
    dK[:h] += g[1]
    dV[:h] += g[2]
    g = causal_backward(Q[h:], K[h:], V[h:], codes_q[h:], codes_k[h:], b, n_min, sample_fn, dO22, dL22, level + 1,
                        2 * node + 1, absolute)
    dQ[h:] += g[0]
    dK[h:] += g[1]
    dV[h:] += g[2]
    g = node_backward(Q[h:], K[:h], V[:h], codes_q[h:], codes_k[:h], b, samples, dO21, dL21, absolute)
    dQ[h:] += g[0]
    dK[:h] += g[1]
    dV[:h] += g[2]
    return dQ, dK, dV


def hyperattn_backward(Q, K, V, dO, b, m, r, causal=False, n_min=4096, seed=0, R=None, sample_fn=None, flip=None,
                       absolute=False):
    """Gradients (dQ, dK, dV) of sum(out * dO) for out = hyperattn_forward(Q, K, V, ...)[0],
    all [B, H, n, d] in fp64; arguments as in hyperattn_forward.

    absolute=True returns instead, element by element, the sum of the magnitudes of the terms
    a gradient element consists of.  With P_ij the final weight of key j in row i (all parts
    under their shared normaliser) every pair contributes dV_j += P_ij dO_i,
    dS_ij = P_ij (<dO_i, v_j> - <dO_i, O_i>), dQ_i += dS_ij k_j, dK_j += dS_ij q_i; the bound is
    the same with |dO|, |v|, |k|, |q|, with sum_j P_ij |v_j| for O_i and a sum for the
    difference.  An evaluation whose operands carry a relative rounding error eps is off by at
    most eps times this bound; the tests scale their tolerance for the gradients by it."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    if absolute:
        V, dO = np.abs(V), np.abs(dO)
    B, H, n, d = Q.shape
    if R is None:
        R = make_projection(seed, d, r)
    if sample_fn is None:
        def sample_fn(level, node, n_keys):
            return make_samples(seed, level, node, n_keys, m)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    for bh in range(B * H):
        q, k, v, g = (x.reshape(B * H, n, -1)[bh] for x in (Q, K, V, dO))
        bits = [lsh_bits(lsh_project(q, R)), lsh_bits(lsh_project(k, R))]
        if flip:
            for (t, fbh, row, kk) in flip:
                if fbh == bh:
                    bits[t][row, kk] = ~bits[t][row, kk]
        cq, ck = (codes_from_bits(bits[t], r) for t in range(2))
        zero = np.zeros(n)
        if absolute:   # v = |V|, g = |dO|: the forward on |V| gives sum_j P_ij |v_j|
            if causal:
                o_abs, _ = causal_forward(q, k, v, cq, ck, b, n_min, sample_fn)
            else:
                o_abs, _ = node_forward(q, k, v, cq, ck, b, sample_fn(0, 0, n))
            zero = (g * o_abs).sum(axis=1)
        if causal:
            gq, gk, gv = causal_backward(q, k, v, cq, ck, b, n_min, sample_fn, g, zero, absolute=absolute)
        else:
            gq, gk, gv = node_backward(q, k, v, cq, ck, b, sample_fn(0, 0, n), g, zero, absolute)
        dQ.reshape(B * H, n, -1)[bh] = gq
        dK.reshape(B * H, n, -1)[bh] = gk
        dV.reshape(B * H, n, -1)[bh] = gv
    return dQ, dK, dV


# --------------------------------------------------------------------------
# Algorithm 2 as printed (caps) and Lemma 2 / Algorithm 3 (value sampling by
# squared row norms): the estimator variants that Section 4's implementation
# paragraph leaves out.  Causal problems run them at every off-diagonal node, as
# Algorithm 4 does ("run the unmasked algorithm on Q_2, K_1"), each node with its
# own subset T, index set and value rows (counters offset by the node's heap
# index 2^level - 1 + node, so the unmasked problem is node 0).
#
# Readings: the constant in C_i = Theta(eps^2 m / (n log n) * (masked row sum +
# tau / kappa)) is a caller's number `cap_scale` (natural log; cap_scale <= 0: no
# cap); kappa is a caller's number (<= 0: no lower cap); the subset T is m rows
# drawn uniformly WITH replacement (Lemma 1's proof bounds the chance that T
# misses the t heaviest rows by (1 - t/n)^m, the bound for independent draws)
# from counter stream 0.  Lemma 2's rows are drawn with p_l = |V_l|^2 / |V|_F^2
# by inverting the cumulative distribution: draw r of head bh takes the uniform
# u in (0, 1) given by the top 53 bits of counter bh * m + r of stream 2 and is
# the first l with p_0 + ... + p_l > u; its rescaling is 1 / (m p_l).
# --------------------------------------------------------------------------
STREAM_TAU_ROWS = 0
STREAM_VNORM = 2


def tau_rows(seed: int, n: int, m: int, heap: int = 0) -> np.ndarray:
    """The rows of Algorithm 2's subset T for a node of n rows (node-local indices)."""
    return np.array([((rand_u64(seed, STREAM_TAU_ROWS, heap * m + j) >> 32) * n) >> 32 for j in range(m)],
                    dtype=np.int64)


def vnorm_probabilities(Vh) -> np.ndarray:
    """Lemma 2: p_l = |V_l|^2 / |V|_F^2 (uniform if V = 0, where every choice gives the same product)."""
    Vh = np.asarray(Vh, dtype=np.float64)
    w = np.sum(Vh ** 2, axis=1)
    total = w.sum()
    if not total > 0.0:
        return np.full(Vh.shape[0], 1.0 / Vh.shape[0])
    return w / total


def vnorm_uniforms(seed: int, bh: int, m: int, heap: int = 0, n_heads: int = 1) -> np.ndarray:
    return np.array([_unit_open(rand_u64(seed, STREAM_VNORM, (heap * n_heads + bh) * m + r_)) for r_ in range(m)])


def vnorm_samples(Vh, seed: int, bh: int, m: int, replay=None, margin=None, heap: int = 0, n_heads: int = 1):
    """(indices l'_1..l'_m, log of their rescaling factors 1 / (m p_l)) for head bh (Lemma 2).

    `replay` {r: l} fixes individual draws (used to follow another evaluation
    through a uniform that falls within rounding of a boundary of the
    cumulative distribution); `margin`, if a list, receives for every draw the
    distance of its uniform to the nearest such boundary."""
    p = vnorm_probabilities(Vh)
    cdf = np.cumsum(p)
    u = vnorm_uniforms(seed, bh, m, heap, n_heads)
    idx = np.minimum(np.searchsorted(cdf, u, side="right"), len(p) - 1).astype(np.int64)
    if margin is not None:
        lower = np.where(idx > 0, cdf[np.maximum(idx - 1, 0)], 0.0)
        margin.extend(np.minimum(u - lower, cdf[idx] - u).tolist())
    if replay:
        for r_, l in replay.items():
            idx[r_] = l
    logw = -np.log(float(m) * p[idx])
    return idx, logw


def alg2_head_forward(Qh, Kh, Vh, codes_q, codes_k, b, samples, t_rows, cap_scale, kappa, vsamp=None):
    """One head.  Returns (out, log d~, log tau).  vsamp = (indices, log weights) selects
    Algorithm 3's value product D~^-1 A S^T S V; None keeps Section 4's numerator (masked
    part exactly + the uniform samples, uncapped)."""
    n = Qh.shape[0]
    m = len(samples)
    perm_q, pos_q = sort_lsh(codes_q)
    perm_k, pos_k = sort_lsh(codes_k)
    blk_q = pos_q // b
    blk_k = pos_k // b
    S = Qh @ Kh.T                                                    # dense: small n only
    Mh = blk_q[:, None] == blk_k[None, :]                            # M^H
    with np.errstate(divide="ignore"):
        log_masked = np.log(np.where(Mh, np.exp(S - S.max()), 0.0).sum(axis=1)) + S.max()
        log_unmasked = np.log(np.where(Mh, 0.0, np.exp(S - S.max())).sum(axis=1)) + S.max()
    log_tau = log_unmasked[t_rows].max() if len(t_rows) else -np.inf            # line "tau <- max_{j in T}"
    floor_term = log_tau - math.log(kappa) if kappa > 0 else -np.inf            # tau / kappa
    samples = np.asarray(samples, dtype=np.int64)
    keep = ~Mh[:, samples] if m else np.zeros((n, 0), dtype=bool)               # 1 - M_{i, l_j}
    Ss = S[:, samples] if m else np.zeros((n, 0))
    if cap_scale > 0 and m > 0:
        log_cap = math.log(cap_scale * m / (n * math.log(n))) + np.logaddexp(log_masked, floor_term)   # C_i
        Sc = np.minimum(Ss, log_cap[:, None])
    else:
        Sc = Ss
    with np.errstate(divide="ignore"):
        ref = max(float(S.max()), 0.0)
        d_i = np.where(keep, np.exp(Sc - ref), 0.0).sum(axis=1) * (n / m if m else 0.0)
        log_d = np.log(d_i) + ref                                                # line "d_i <- (n/m) sum ..."
    log_dt = np.logaddexp(log_masked, np.maximum(log_d, floor_term))             # line "d~_i <- ... + max(d_i, tau/kappa)"
    if vsamp is not None:
        vi, vlogw = vsamp
        num = np.exp(S[:, vi] + vlogw[None, :] - log_dt[:, None]) @ Vh[vi]      # D~^-1 A S^T S V
    else:
        P_masked = np.where(Mh, np.exp(S - log_dt[:, None]), 0.0)
        num = P_masked @ Vh
        if m:
            num = num + (n / m) * (np.where(keep, np.exp(Ss - log_dt[:, None]), 0.0) @ Vh[samples])
    return num, log_dt, log_tau


def causal_forward_alg2(Q, K, V, codes_q, codes_k, b, n_min, node_draws, cap_scale, kappa, taus, level=0, node=0):
    """Algorithm 4 with Algorithm 2 as printed at every off-diagonal node.  node_draws(level, node, s, V1)
    returns (samples, rows of T, value draws or None) of the node; taus[heap] receives its log tau.
    Returns (out, log D~) like causal_forward."""
    n = Q.shape[0]
    if n <= n_min:
        return exact_attention(Q, K, V, causal=True)
    h = n // 2
    O1, L1 = causal_forward_alg2(Q[:h], K[:h], V[:h], codes_q[:h], codes_k[:h], b, n_min, node_draws, cap_scale, kappa,
                                 taus, level + 1, 2 * node)
    O22, L22 = causal_forward_alg2(Q[h:], K[h:], V[h:], codes_q[h:], codes_k[h:], b, n_min, node_draws, cap_scale,
                                   kappa, taus, level + 1, 2 * node + 1)
    samples, t_rows, vsamp = node_draws(level, node, h, V[:h])
    O21, L21, log_tau = alg2_head_forward(Q[h:], K[:h], V[:h], codes_q[h:], codes_k[:h], b, samples, t_rows, cap_scale,
                                          kappa, vsamp)
    taus[(1 << level) - 1 + node] = log_tau
    O2, L2 = merge_parts(O21, L21, O22, L22)                       # D~_21 + D~_C22
    return np.concatenate([O1, O2]), np.concatenate([L1, L2])


def hyperattn_forward_alg2(Q, K, V, b, m, r, seed=0, cap_scale=0.0, kappa=0.0, vnorm_sampling=False, R=None,
                           vnorm_from=None, vnorm_replay=None, causal=False, n_min=4096):
    """HyperAttention with Algorithm 2's estimator as printed.  Returns (out, log d~, log tau); log tau is
    [B*H] for the unmasked problem and [B*H, nodes] (heap order) for the causal one, where every
    off-diagonal node of Algorithm 4 runs Algorithm 2 with its own draws.
    vnorm_from: the value tensor whose row norms define Lemma 2's draws (default V itself; the tests
    pass V when they evaluate the same draws on |V|); vnorm_replay: {(bh, heap): {r: l}} fixed draws
    ({bh: {r: l}} is accepted for the unmasked problem)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, n, d = Q.shape
    if R is None:
        R = make_projection(seed, d, r)
    replay = vnorm_replay or {}
    out = np.empty_like(V)
    lse = np.empty((B, H, n))
    levels = 0
    if causal:
        while (n >> levels) > n_min:
            levels += 1
    taus = np.full((B * H, (1 << levels) - 1), -np.inf) if causal else np.empty(B * H)
    Vsrc = V if vnorm_from is None else np.asarray(vnorm_from, dtype=np.float64)
    for bh in range(B * H):
        q, k, v = (x.reshape(B * H, n, -1)[bh] for x in (Q, K, V))
        vsrc = Vsrc.reshape(B * H, n, -1)[bh]
        cq, ck = lsh_codes(lsh_project(q, R), r), lsh_codes(lsh_project(k, R), r)
        if not causal:
            vs = None
            if vnorm_sampling:
                vs = vnorm_samples(vsrc, seed, bh, m, replay=replay.get((bh, 0), replay.get(bh)))
            o, l, t = alg2_head_forward(q, k, v, cq, ck, b, make_samples(seed, 0, 0, n, m), tau_rows(seed, n, m),
                                        cap_scale, kappa, vs)
            taus[bh] = t
        else:
            def node_draws(level, node, s, V1, bh=bh, vsrc=vsrc):
                heap = (1 << level) - 1 + node
                vs = None
                if vnorm_sampling:
                    k0 = 2 * node * s                              # the node's keys are rows [2 node s, (2 node + 1) s)
                    vs = vnorm_samples(vsrc[k0:k0 + s], seed, bh, m, replay=replay.get((bh, heap)), heap=heap,
                                       n_heads=B * H)
                return make_samples(seed, level, node, s, m), tau_rows(seed, s, m, heap), vs
            node_taus = {}
            o, l = causal_forward_alg2(q, k, v, cq, ck, b, n_min, node_draws, cap_scale, kappa, node_taus)
            for heap, t in node_taus.items():
                taus[bh, heap] = t
        out.reshape(B * H, n, -1)[bh] = o
        lse.reshape(B * H, n)[bh] = l
    return out, lse, taus


# --------------------------------------------------------------------------
# The quantities the paper's guarantees are stated in (Section 1.1 Eq. (1),
# Lemma 1, Section 4.3), from the dense matrices (small n only).
# --------------------------------------------------------------------------
def attention_matrix(Q, K, causal=False) -> np.ndarray:
    """D^-1 A (causal: D_C^-1 (M^C . A)) as a dense n x n matrix."""
    n = np.asarray(Q).shape[0]
    return exact_attention(Q, K, np.eye(n), causal)[0]


def alpha(Q, K) -> float:
    """Lemma 1: alpha = n * max_j |D^-1 A e_j|_2^2, the largest squared column norm of the softmax matrix times n."""
    P = attention_matrix(Q, K)
    return float(P.shape[0] * (P ** 2).sum(axis=0).max())


def kappa(Q, K, codes_q, codes_k, b) -> float:
    """Lemma 1: ratio of the largest to the smallest unmasked row sum <1 - M^H_i, A_i>, with M^H of Algorithm 1."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    _, pos_q = sort_lsh(codes_q)
    _, pos_k = sort_lsh(codes_k)
    S = Q @ K.T
    ref = S.max()
    outside = (pos_q[:, None] // b) != (pos_k[None, :] // b)          # 1 - M^H
    unmasked = np.where(outside, np.exp(S - ref), 0.0).sum(axis=1)
    return float(unmasked.max() / unmasked.min())


def spectral_error(att_approx, Q, K, V, causal=False) -> float:
    """The epsilon Eq. (1) is satisfied with: |Att~ - Att|_op / (|D^-1 A|_op |V|_op), operator norms
    being largest singular values."""
    V = np.asarray(V, dtype=np.float64)
    P = attention_matrix(Q, K, causal)
    err = np.asarray(att_approx, dtype=np.float64) - P @ V
    top = lambda M: float(np.linalg.svd(M, compute_uv=False)[0])
    return top(err) / (top(P) * top(V))
