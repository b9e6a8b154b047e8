"""Seeded synthetic inputs for the HyperAttention forward path.

This module holds input generation only: it draws Q, K, V with the shapes and
value distributions of the benchmark workloads and rounds them once to the
storage dtype.  None of the method's arithmetic (hashing, sorting, softmax,
sampling) lives here, so the CPU oracle and the HIP path can both be fed from
it without sharing any code of the method itself.

Workloads (Q, K, V are [B, H, n, d]):

  iid      Q, K, V ~ N(0, 1) / d**0.25           (the single-layer timing shape
           of the paper's Section 4.2 and the ChatGLM2-like layer shape of
           Section 4.1, with the softmax scale folded into Q and K because the
           paper's attention matrix is exp(Q K^T) with no 1/sqrt(d) factor)
  mixture  Q, K rows drawn from a 64-centre Gaussian mixture per (batch, head):
           centres ~ N(0, 4 I), within-cluster sigma 0.5, cluster k chosen with
           probability proportional to k**-1.1; V ~ N(0, 1).  Uneven LSH
           buckets and large attention entries.
"""
from __future__ import annotations

import numpy as np

DATA_SEED = 1234


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result is fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    bits = bits + np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))
    bits = (bits & np.uint64(0xFFFF0000)).astype(np.uint32)
    return bits.view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable fp32 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def _finish(arrs, dtype):
    if dtype == "bf16":
        return tuple(round_to_bf16(a) for a in arrs)
    if dtype == "fp32":
        return tuple(np.ascontiguousarray(a, dtype=np.float32) for a in arrs)
    raise ValueError(f"unknown dtype {dtype!r}")


def iid_qkv(B, H, n, d, dtype="bf16", seed=DATA_SEED):
    """Q, K, V iid N(0,1)/d**0.25, rounded once to `dtype` (returned as fp32)."""
    rng = np.random.default_rng(seed)
    scale = np.float32(d ** -0.25)
    out = []
    for _ in range(3):
        a = rng.standard_normal((B, H, n, d), dtype=np.float32)
        a *= scale
        out.append(a)
    return _finish(out, dtype)


def mixture_qkv(B, H, n, d, dtype="bf16", seed=DATA_SEED, centres=64,
                centre_sigma=2.0, within_sigma=0.5, zipf_s=1.1):
    """Clustered Q, K (shared centres per (batch, head)), V iid N(0,1)."""
    rng = np.random.default_rng(seed)
    pk = np.arange(1, centres + 1, dtype=np.float64) ** (-zipf_s)
    pk /= pk.sum()
    Q = np.empty((B, H, n, d), dtype=np.float32)
    K = np.empty((B, H, n, d), dtype=np.float32)
    for bi in range(B):
        for hi in range(H):
            C = (centre_sigma * rng.standard_normal((centres, d))).astype(np.float32)
            for dst in (Q, K):
                which = rng.choice(centres, size=n, p=pk)
                noise = rng.standard_normal((n, d), dtype=np.float32)
                dst[bi, hi] = C[which] + np.float32(within_sigma) * noise
    V = rng.standard_normal((B, H, n, d), dtype=np.float32)
    return _finish((Q, K, V), dtype)


# The benchmark configurations: shape, dtype, input law and algorithm parameters.
CONFIGS = {
    "cfg1_n1k_fp32": dict(B=1, H=1, n=1024, d=64, dtype="fp32", law="iid",
                          b=64, m=64, r=7, causal=0, n_min=4096, seed=0),
    "cfg2_n32k": dict(B=1, H=32, n=32768, d=128, dtype="bf16", law="iid",
                      b=256, m=256, r=7, causal=0, n_min=4096, seed=0),
    "cfg3_n32k_causal": dict(B=1, H=32, n=32768, d=128, dtype="bf16", law="iid",
                             b=256, m=256, r=7, causal=1, n_min=4096, seed=0),
    "cfg4_n131k_causal": dict(B=1, H=32, n=131072, d=128, dtype="bf16", law="iid",
                              b=256, m=256, r=7, causal=1, n_min=4096, seed=0),
    "cfg5_n65k_mixture": dict(B=2, H=32, n=65536, d=64, dtype="bf16", law="mixture",
                              b=256, m=512, r=7, causal=0, n_min=4096, seed=0),
}


# The single-layer sweep shape of the paper's speed-up curves (Section 4.2): 12 heads
# of dimension 64, b = m = 256, sequence lengths 4k .. 131k, with and without the causal mask.
SWEEP_LENGTHS = (4096, 8192, 16384, 32768, 65536, 131072)
for _n in SWEEP_LENGTHS:
    for _c in (0, 1):
        CONFIGS[f"sweep_h12_d64_n{_n}" + ("_causal" if _c else "")] = dict(
            B=1, H=12, n=_n, d=64, dtype="bf16", law="iid", b=256, m=256, r=7, causal=_c, n_min=4096, seed=0)


def make_qkv(cfg: dict, seed=DATA_SEED, B=None, H=None, n=None):
    """Inputs for a CONFIGS entry (optionally with B, H or n overridden)."""
    B = cfg["B"] if B is None else B
    H = cfg["H"] if H is None else H
    n = cfg["n"] if n is None else n
    gen = iid_qkv if cfg["law"] == "iid" else mixture_qkv
    return gen(B, H, n, cfg["d"], cfg["dtype"], seed)


def device_qkv(cfg: dict, torch, generator, B=None, H=None):
    """Q, K, V of a CONFIGS entry drawn on the GPU from the same law (torch's generator: not the
    same numbers as the host generators above), in the configuration's dtype.  For heads that no
    CPU reference is computed for."""
    B = cfg["B"] if B is None else B
    H = cfg["H"] if H is None else H
    n, d = cfg["n"], cfg["d"]
    dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    randn = lambda *shape: torch.randn(shape, generator=generator, device="cuda", dtype=torch.float32)
    if cfg["law"] == "iid":
        return [(randn(B, H, n, d) * d ** -0.25).to(dt).contiguous() for _ in range(3)]
    centres, centre_sigma, within_sigma, zipf_s = 64, 2.0, 0.5, 1.1
    C = centre_sigma * randn(B * H, centres, d)
    pk = torch.arange(1, centres + 1, device="cuda", dtype=torch.float32) ** (-zipf_s)
    out = []
    for _ in range(2):
        which = torch.multinomial((pk / pk.sum()).expand(B * H, centres), n, replacement=True, generator=generator)
        rows = torch.gather(C, 1, which[:, :, None].expand(B * H, n, d))
        rows += within_sigma * randn(B * H, n, d)
        out.append(rows.view(B, H, n, d).to(dt).contiguous())
    out.append(randn(B, H, n, d).to(dt).contiguous())
    return out
