#!/usr/bin/env python3
"""Quality diagnostics of the HyperAttention approximation on a synthetic workload,
in the quantities the paper's guarantees are stated in (Section 1.1 Eq. (1),
Lemma 1, Theorem 1, Section 4.3):

  spectral_error  ||Att~ - Att||_op / (||D^-1 A||_op ||V||_op)      (Eq. (1): the epsilon achieved)
  alpha           n * max_j ||D^-1 A e_j||_2^2                       (Lemma 1)
  kappa           max_i / min_i of the unmasked row sums <1 - M^H_i, A_i>   (Lemma 1)

    python diagnostics.py [--workload cfg2_n32k] [--heads 2] [--iters 12]

Everything heavy runs in the library's own kernels, through the same entry
points as the benchmark:
  * Att~ and Att: hyperattn_forward and exact_attn_forward;
  * ||D^-1 A||_op: block power iteration with P X = exact_attn_forward(V := X) and
    P^T Y = the dV of exact_attn_backward(dO := Y);
  * alpha: the column sums of P o P are the dV of exact attention on (2Q, K) with log row
    sums 2L and dO = 1, because P_ij^2 = exp(2<q_i,k_j> - 2L_i);
  * kappa: unmasked row sum = exact row sum - block row sum, the latter from
    hyperattn_forward with m = 0 (Algorithm 1's mask alone).
torch is used for d x d Gram matrices, their eigenvalues, QR and max / min reductions.
Tensors are bf16, so the figures carry about two to three significant digits.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs  # noqa: E402


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def op_norm_tall(torch, X):
    """Largest singular value of each [n, d] matrix in X [..., n, d] (via the d x d Gram matrix, fp64)."""
    Xd = X.double()
    gram = Xd.transpose(-1, -2) @ Xd
    return torch.linalg.eigvalsh(gram)[..., -1].clamp_min(0).sqrt()


def softmax_op_norm(torch, ha, Q, K, lse, causal, iters):
    """||P||_op per head of batch 0, P = D^-1 A (causal: D_C^-1 (M^C o A)): block power iteration on P^T P."""
    _, H, n, d = Q.shape
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    X = torch.randn((1, H, n, d), generator=g, device="cuda", dtype=torch.float32)
    p_op = torch.zeros(H, dtype=torch.float64, device="cuda")
    for _ in range(iters):
        Xq, _ = torch.linalg.qr(X[0].double())                 # orthonormal columns per head
        Xb = Xq.float().to(torch.bfloat16)[None].contiguous()
        Y, _ = ha.exact_attn_forward(Q, K, Xb, causal=causal)  # P X
        p_op = op_norm_tall(torch, Y[0].float())               # ||P X||_op, X orthonormal: a lower bound that converges
        _, _, Z = ha.exact_attn_backward(Q, K, Xb, Y, lse, Y, causal=causal)  # its dV is P^T Y
        X = Z.float()
    return p_op


def alpha_of(torch, ha, Q, K, lse):
    """n * max_j sum_i P_ij^2 per head of batch 0 (unmasked attention)."""
    n = Q.shape[2]
    ones = torch.ones_like(Q)
    Q2 = (Q.float() * 2).to(torch.bfloat16)                    # exact in bf16
    _, _, colsq = ha.exact_attn_backward(Q2, K, ones, ones, (2.0 * lse).contiguous(), ones, causal=False)
    return n * colsq[0, :, :, 0].float().max(dim=1).values


def kappa_of(torch, lse_exact, lse_block):
    """max / min over rows of the unmasked row sum exp(L) - exp(L_block), per head of batch 0,
    and the mean share of the row sum that the block part holds."""
    gap = (lse_block.double() - lse_exact.double()).clamp_max(-1e-7)   # log(block share) < 0
    log_unmasked = lse_exact.double() + torch.log1p(-torch.exp(gap))
    kappa = torch.exp(log_unmasked[0].max(dim=1).values - log_unmasked[0].min(dim=1).values)
    return kappa, torch.exp(gap[0]).mean(dim=1)


def spectral_error_of(torch, ha, Q, K, V, out_approx, out_exact, lse_exact, causal, iters):
    """The epsilon of Eq. (1) per head of batch 0: ||Att~ - Att||_op / (||D^-1 A||_op ||V||_op).
    Returns (epsilon, ||Att~ - Att||_op, ||D^-1 A||_op, ||V||_op)."""
    err = out_approx.float() - out_exact.float()
    err_op = op_norm_tall(torch, err[0])
    v_op = op_norm_tall(torch, V[0].float())
    p_op = softmax_op_norm(torch, ha, Q, K, lse_exact, causal, iters)
    return err_op / (p_op * v_op), err_op, p_op, v_op


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg2_n32k", choices=sorted(synth_inputs.CONFIGS))
    ap.add_argument("--heads", type=int, default=2, help="heads of batch 0 to analyse")
    ap.add_argument("--iters", type=int, default=12, help="power iterations for ||D^-1 A||_op")
    args = ap.parse_args()

    import torch
    import paper_2310_05869_amd as ha
    ha.lib()
    if not torch.cuda.is_available():
        sys.exit("diagnostics.py: no GPU visible")
    cfg = dict(synth_inputs.CONFIGS[args.workload])
    if cfg["dtype"] != "bf16":
        sys.exit("diagnostics.py: bf16 workloads only (the exact backward used for P^T is bf16)")
    H = min(args.heads, cfg["H"])
    n, d, causal = cfg["n"], cfg["d"], bool(cfg["causal"])
    host = synth_inputs.make_qkv(cfg, B=1, H=H)
    Q, K, V = (torch.from_numpy(x).cuda().to(torch.bfloat16).contiguous() for x in host)
    kw = dict(causal=causal, n_min=cfg["n_min"], seed=cfg["seed"])
    log(f"[diag] {args.workload}: {H} head(s), n={n}, d={d}, causal={causal}")

    out_h, lse_h = ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], **kw)
    out_e, lse_e = ha.exact_attn_forward(Q, K, V, causal=causal)
    err = out_h.float() - out_e.float()
    rel_fro = (err[0].double().flatten(1).norm(dim=1) / out_e[0].double().flatten(1).norm(dim=1))
    max_abs = err[0].abs().flatten(1).max(dim=1).values
    spectral, err_op, p_op, v_op = spectral_error_of(torch, ha, Q, K, V, out_h, out_e, lse_e, causal, args.iters)

    result = {"workload": args.workload, "heads": H, "n": n, "d": d, "causal": causal,
              "b": cfg["b"], "m": cfg["m"], "r": cfg["r"],
              "spectral_error": [float(x) for x in spectral], "err_op_norm": [float(x) for x in err_op],
              "softmax_op_norm": [float(x) for x in p_op], "V_op_norm": [float(x) for x in v_op],
              "rel_frobenius_error": [float(x) for x in rel_fro], "max_abs_error": [float(x) for x in max_abs]}

    if not causal:
        alpha = alpha_of(torch, ha, Q, K, lse_e)
        _, lse_b = ha.hyperattn_forward(Q, K, V, cfg["b"], 0, cfg["r"], **kw)   # mask M^H alone
        kappa, share = kappa_of(torch, lse_e, lse_b)
        result.update({"alpha": [float(x) for x in alpha], "kappa": [float(x) for x in kappa],
                       "mean_block_share_of_row_sum": [float(x) for x in share]})
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
