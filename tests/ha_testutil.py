"""Helpers shared by the GPU parity tests: moving seeded inputs to the device,
the tolerances, and the staged comparison (codes, then permutations, then
outputs) between the HIP library and the CPU oracle."""
import numpy as np

import synth_inputs
from oracle import hyperattn_oracle as orc


def have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def to_device(x_fp32: np.ndarray, dtype: str):
    """fp32 host array (already rounded to `dtype`) -> device tensor of that dtype."""
    import torch
    if dtype == "bf16":
        bits = synth_inputs.bf16_bits(x_fp32).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x_fp32, dtype=np.float32)).cuda()


def to_host(t) -> np.ndarray:
    import torch
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def half_ulp_bf16(x: np.ndarray) -> np.ndarray:
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 8)


def out_tolerance(ref: np.ndarray, dtype: str, absv=None) -> np.ndarray:
    """bf16: 2e-3 absolute plus the half-ulp of rounding the result to bf16.
    The bf16 path feeds the softmax weights to the matrix cores as bf16 (relative
    rounding error at most 2^-8 each), which moves an output by at most
    2^-8 * sum_j p_j |v_j|; where the caller passes that sum (`absv`: the oracle
    run on |V|) it is added, otherwise it must fit in the 2e-3 (it does when
    |V| is small, as for the iid workloads).
    The half-ulp is that of the value that gets rounded, which may lie in the binade
    above the reference's when the reference sits just under a power of two: it is
    taken at |ref| plus the rest of the tolerance.
    fp32: 1e-5 absolute plus 1e-5 relative."""
    if dtype == "bf16":
        tol = np.full_like(ref, 2e-3, dtype=np.float64)
        if absv is not None:
            tol = tol + 2.0 ** -8 * absv
        return tol + half_ulp_bf16(np.abs(ref) + tol)
    return 1e-5 + 1e-5 * np.abs(ref)


LSE_TOL = {"bf16": 1e-3, "fp32": 2e-5}


def assert_close(got, ref, dtype, what, absv=None, max_plain_frac=0.0):
    """Element-wise comparison.  Without `absv` the criterion is the plain one of out_tolerance().
    With `absv` (bf16 only) an element may also use the operand-rounding allowance
    2^-8 sum_j p_j |v_j|, the bound the arithmetic guarantees; the number of elements that fail
    the plain criterion is printed and must not exceed max_plain_frac of all elements (one
    element is always allowed: the caller chooses the share by how many keys carry a row)."""
    err = np.abs(got - ref)
    plain = err > out_tolerance(ref, dtype)
    if absv is None:
        bad = plain
    else:
        bad = err > out_tolerance(ref, dtype, absv)
        frac = plain.mean() if plain.size else 0.0
        print(f"  {what}: {int(plain.sum())} of {plain.size} elements ({frac:.3%}) exceed the plain criterion "
              f"(allowed {max_plain_frac:.3%}); worst excess {float((err - out_tolerance(ref, dtype)).max()):.2e}", flush=True)
        assert plain.sum() <= max(1, int(max_plain_frac * plain.size)), \
            f"{what}: {frac:.3%} of the elements need the operand-rounding allowance"
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; "
                           f"max abs err {err.max():.3e} (|ref| there {np.abs(ref).ravel()[err.argmax()]:.3e})")
    return float(err.max())


def assert_lse_close(got, ref, dtype, what):
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin), f"{what}: -inf pattern differs"
    if fin.any():
        err = np.abs(got[fin] - ref[fin])
        tol = LSE_TOL[dtype] * np.maximum(1.0, np.abs(ref[fin]))
        assert (err <= tol).all(), f"{what}: lse max abs err {err.max():.3e}"


def compare_codes(gpu_codes, stages, r):
    """Bucket codes must be bit-exact, except where the oracle's projection is
    closer to zero than 1e-6.  Returns the list of (tensor, bh, row, k) sign bits
    on which the HIP path differs (to be replayed by the oracle) and asserts that
    each of them has |projection| < 1e-6."""
    inv = np.argsort(orc.gray_rank_table(r))  # bucket -> word
    flips = []
    for t in range(2):
        g = gpu_codes[t].astype(np.int64)
        o = stages["codes"][t]
        for (bh, row) in zip(*np.nonzero(g != o)):
            diff = int(inv[g[bh, row]]) ^ int(inv[o[bh, row]])
            for k in range(r):
                if (diff >> k) & 1:
                    p = stages["proj"][t, bh, row, k]
                    assert abs(p) < 1e-6, f"sign differs at |projection| = {abs(p):.3e}"
                    flips.append((t, int(bh), int(row), k))
    return flips


def run_oracle(Q, K, V, cfg, R=None, sample_fn=None, flip=None, stages=None, with_absv=False):
    """The oracle's (out, lse); with_absv also returns sum_j p_j |v_j| (the
    oracle is linear in V, so [V, |V|] side by side gives both in one run)."""
    if with_absv:
        d = V.shape[-1]
        both, lse = run_oracle(Q, K, np.concatenate([V, np.abs(V)], axis=-1), cfg, R, sample_fn, flip, stages)
        return both[..., :d], lse, both[..., d:]
    return orc.hyperattn_forward(Q, K, V, b=cfg["b"], m=cfg["m"], r=cfg["r"], causal=bool(cfg["causal"]),
                                 n_min=cfg["n_min"], seed=cfg["seed"], R=R, sample_fn=sample_fn, flip=flip,
                                 stages=stages)
