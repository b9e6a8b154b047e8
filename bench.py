#!/usr/bin/env python3
"""Benchmark of the HyperAttention forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one whole forward call (hash, sort, block + sampled attention of every
node, causal base case and merge) on one batch of synthetic input that is
already resident in HBM.  The default workload is the long-context target:
causal, 32 heads, n = 131072, d = 128, bf16, b = m = 256, r = 7, n_min = 4096.
Prints ONE JSON line (see the keys below); nothing else goes to stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import synth_inputs  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak
CPU_SAMPLE_HEADS = 4        # heads the oracle is timed on by the cpu_baseline leg



def measured_traffic_bytes(workload, key):
    """HBM bytes per launch of a kernel ("node" / "base") from the rocprofv3 --pmc summary of the
    workload under profiles/ (its lines "traffic <key> FETCH_SIZE <KiB> x <factor> WRITE_SIZE <KiB> x <factor>"),
    or None if no such summary exists."""
    short = workload.split("_")[0]
    folder = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(folder)) if os.path.isdir(folder) else []:
        if not (name.startswith(f"bench_{short}_") and name.endswith("_hbm_traffic.txt")):
            continue
        for line in open(os.path.join(folder, name)):
            f = line.split()
            if len(f) == 10 and f[0] == "traffic" and f[1] == key:
                return int((float(f[3]) * float(f[5]) + float(f[7]) * float(f[9])) * 1024)
    return None


def host_cpu_model():
    """The host processor's name as /proc/cpuinfo gives it (empty if unavailable)."""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return ""


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def device_inputs(cfg, torch, host_heads=1):
    """Q, K, V on the device.  Heads [0, host_heads) of batch 0 come from the
    seeded host generator (so the oracle can be fed the identical rounded
    arrays); the rest is drawn on the device from the same law."""
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    g = torch.Generator(device="cuda")
    g.manual_seed(synth_inputs.DATA_SEED)
    host = synth_inputs.make_qkv(cfg, B=1, H=host_heads)
    out = synth_inputs.device_qkv(cfg, torch, g)
    for i in range(3):
        out[i][0, :host_heads] = torch.from_numpy(host[i][0]).cuda().to(dt)
    return out, host


def algorithmic_work(cfg):
    """Flops and bytes per forward call, from the stage definitions:
    4 d (b + m) flop per query row of every node; 4 n_min^2 d / 2 per causal base
    block; hashing reads every row of Q and K once and writes one byte per row."""
    B, H, n, d, b, m = cfg["B"], cfg["H"], cfg["n"], cfg["d"], cfg["b"], cfg["m"]
    BH = B * H
    esz = 2 if cfg["dtype"] == "bf16" else 4
    w = {}
    if cfg["causal"] and n > cfg["n_min"]:
        levels = int(np.log2(n // cfg["n_min"]))
        node_rows = levels * (n // 2)
        base_blocks = n // cfg["n_min"]
        w["base_flop"] = BH * base_blocks * 4.0 * cfg["n_min"] ** 2 * d / 2
    elif cfg["causal"]:
        node_rows, w["base_flop"] = 0, BH * 4.0 * n * n * d / 2
    else:
        node_rows, w["base_flop"] = n, 0.0
    w["node_flop"] = BH * node_rows * 4.0 * d * (b + m)
    # least HBM bytes of the node attention: every query row is read and its result written once, every
    # block's K and V rows are read once for its b queries (the m sampled rows of a node stay in L2)
    w["node_bytes"] = BH * node_rows * (4 * d * esz + 4)
    w["hash_bytes"] = 2 * BH * n * (d * esz + 1)
    # the sort: every key of every node is read once (1 B) and written as perm (4 B), keys also as pos (4 B)
    w["sort_bytes"] = BH * node_rows * (2 * (1 + 4) + 4) if node_rows else 0
    w["exact_flop"] = BH * 4.0 * n * n * d * (0.5 if cfg["causal"] else 1.0)
    return w


def time_call(torch, fn, warmup, steps):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def sweep(args, torch, ha):
    """The 12-head, d = 64 single-layer sweep (Section 4.2): forward and exact-attention
    time at every length, causal and not.  One JSON line with the whole curve."""
    points = []
    for name in sorted((k for k in synth_inputs.CONFIGS if k.startswith("sweep_")),
                       key=lambda k: (synth_inputs.CONFIGS[k]["causal"], synth_inputs.CONFIGS[k]["n"])):
        cfg = dict(synth_inputs.CONFIGS[name])
        (Q, K, V), _ = device_inputs(cfg, torch)
        B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
        shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
        params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
        ws = ha.alloc_workspace(shape, params)
        out = torch.empty_like(Q)
        lse = torch.empty((B, H, n), dtype=torch.float32, device="cuda")
        kw = dict(causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"], workspace=ws, out=out, lse=lse)
        ms = time_call(torch, lambda: ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], **kw),
                       args.warmup, args.steps)
        ex = time_call(torch, lambda: ha.exact_attn_forward(Q, K, V, causal=cfg["causal"], out=out, lse=lse),
                       1, 3 if n <= 32768 else 2)
        # the same call replayed from a HIP graph (the library only enqueues kernels): the short lengths are
        # bound by the launches of its five kernels
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], **kw)
        gms = time_call(torch, graph.replay, args.warmup, args.steps)
        del graph
        work = algorithmic_work(cfg)
        points.append({"workload": name, "n": n, "causal": bool(cfg["causal"]), "ms": round(ms, 4),
                       "graph_replay_ms": round(gms, 4),
                       "exact_ms": round(ex, 4), "speedup_vs_exact": round(ex / ms, 3),
                       "exact_TFLOPs": round(work["exact_flop"] / (ex * 1e-3) / 1e12, 1)})
        log(f"[bench] {name}: {ms:.3f} ms ({gms:.3f} ms replayed from a graph), exact {ex:.3f} ms, speed-up {ex / ms:.2f}x")
        del Q, K, V, ws, out, lse
    last = points[-1]
    print(json.dumps({
        "metric": "HyperAttention fwd ms", "value": last["ms"], "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": last["ms"], "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": last["workload"], "B": 1, "H": 12, "d": 64, "b": 256, "m": 256, "r": 7, "n_min": 4096,
                   "note": "value is the longest causal point of the sweep"},
        "sweep": points}), flush=True)


def alg2_bench(args, torch, ha):
    """Algorithm 2 as printed (caps, tau) and Lemma 2's value sampling, the options beside the
    Section 4 form, at the unmasked 32-head workload and at the causal one of the same length (where
    Algorithm 4 runs them at every off-diagonal node): time of each next to the main path's."""
    points = {}
    for name in ("cfg2_n32k", "cfg3_n32k_causal"):
        cfg = dict(synth_inputs.CONFIGS[name])
        (Q, K, V), _ = device_inputs(cfg, torch)
        B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
        b, m, r = cfg["b"], cfg["m"], cfg["r"]
        out, lse = torch.empty_like(Q), torch.empty((B, H, n), dtype=torch.float32, device="cuda")
        shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
        ckw = dict(causal=bool(cfg["causal"]), n_min=cfg["n_min"])
        ws = ha.alloc_workspace(shape, ha.make_params(b, m, r, cfg["causal"], cfg["n_min"], cfg["seed"]))
        main_ms = time_call(torch, lambda: ha.hyperattn_forward(Q, K, V, b, m, r, seed=cfg["seed"], workspace=ws, out=out,
                                                                lse=lse, **ckw), args.warmup, args.steps)
        res = {"section4_form_ms": round(main_ms, 4)}
        ws2 = None
        for key, vn in (("caps_ms", False), ("caps_and_value_sampling_ms", True)):
            kw = dict(seed=cfg["seed"], cap_scale=8.0, kappa=1.2, vnorm_sampling=vn, out=out, lse=lse, **ckw)
            _, _, ws2 = ha.hyperattn_forward_alg2(Q, K, V, b, m, r, workspace=ws2, **kw)
            res[key] = round(time_call(torch, lambda: ha.hyperattn_forward_alg2(Q, K, V, b, m, r, workspace=ws2, **kw),
                                       args.warmup, args.steps), 4)
            log(f"[bench] {name} {key}: {res[key]:.3f} ms (Section 4 form: {main_ms:.3f} ms)")
        points[name] = res
        del Q, K, V, out, lse, ws, ws2
    cfg = synth_inputs.CONFIGS["cfg2_n32k"]
    print(json.dumps({
        "metric": "HyperAttention fwd ms", "value": points["cfg2_n32k"]["caps_ms"], "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": points["cfg2_n32k"]["caps_ms"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg2_n32k", "B": cfg["B"], "H": cfg["H"], "n": cfg["n"], "d": cfg["d"], "b": cfg["b"],
                   "m": cfg["m"], "r": cfg["r"], "causal": False,
                   "estimator": "Algorithm 2 as printed: cap_scale 8, kappa 1.2"},
        **points["cfg2_n32k"], "also_cfg3_n32k_causal": points["cfg3_n32k_causal"]}), flush=True)


def backward_bench(args, torch, ha):
    """Forward + backward of the chosen workload (Section 4.2 quotes its speed-ups on that sum),
    with exact attention forward + backward beside it.  One JSON line."""
    cfg = dict(synth_inputs.CONFIGS[args.workload])
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    (Q, K, V), host = device_inputs(cfg, torch)
    g = torch.Generator(device="cuda")
    g.manual_seed(synth_inputs.DATA_SEED + 7)
    G = torch.randn(Q.shape, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    bws = ha.alloc_backward_workspace(shape, params)
    out = torch.empty_like(Q)
    lse = torch.empty((B, H, n), dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(Q) for _ in range(3))
    out32 = torch.empty(Q.shape, dtype=torch.float32, device="cuda")  # unrounded output for the backward's delta
    kw = dict(causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"])
    pa = (cfg["b"], cfg["m"], cfg["r"])

    def fwd():
        ha.hyperattn_forward(Q, K, V, *pa, workspace=ws, out=out, lse=lse, out_f32=out32, **kw)

    def bwd():
        ha.hyperattn_backward(Q, K, V, out, lse, G, *pa, fwd_workspace=ws, bwd_workspace=bws, grads=grads,
                              out_f32=out32, **kw)

    def both():
        fwd()
        bwd()

    fwd_ms = time_call(torch, fwd, args.warmup, args.steps)
    both_ms = time_call(torch, both, args.warmup, args.steps)
    stage = {k: 0.0 for k in ha.binding.BWD_STAGE_NAMES}
    for _ in range(args.steps):
        ms = ha.hyperattn_backward_timed(Q, K, V, out, lse, G, *pa, fwd_workspace=ws, bwd_workspace=bws, grads=grads,
                                         out_f32=out32, **kw)[3]
        for k, v in ms.items():
            stage[k] += v / args.steps
    log(f"[bench] forward {fwd_ms:.3f} ms, forward + backward {both_ms:.3f} ms")
    log("[bench] backward stage ms: " + ", ".join(f"{k} {v:.3f}" for k, v in stage.items()))
    work = algorithmic_work(cfg)
    # five products per (query, key) pair against the forward's two: S, dP, dQ, dK, dV
    bwd_flop = 2.5 * (work["node_flop"] + work["base_flop"])
    bwd_ms = both_ms - fwd_ms
    result = {
        "metric": "HyperAttention fwd+bwd ms", "value": round(both_ms, 4), "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(both_ms, 4), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "B": B, "H": H, "n": n, "d": d, "b": cfg["b"], "m": cfg["m"],
                   "r": cfg["r"], "causal": bool(cfg["causal"]), "n_min": cfg["n_min"], "law": cfg["law"],
                   "pass": "forward + backward"},
        "forward_ms": round(fwd_ms, 4), "backward_ms": round(bwd_ms, 4),
        "backward_stages_ms": {k: round(v, 4) for k, v in stage.items()},
        "roofline": {"bound": "mfma", "kernel": "attn_bwd_kernel (all five passes of one backward call)",
                     "achieved": round(bwd_flop / (bwd_ms * 1e-3) / 1e12, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(bwd_flop / (bwd_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "traffic": None, "flop_per_launch": bwd_flop, "ms_per_launch": round(bwd_ms, 4),
                     "note": "algorithmic flops (5 products per pair); the three-pass scheme executes 8 (3 for dQ, 3 for dK, 2 for dV)"},
    }
    if not args.no_exact:
        eo, el = torch.empty_like(Q), torch.empty_like(lse)
        ews = torch.empty(int(ha.lib().exact_attn_backward_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")

        egrads = tuple(torch.empty_like(Q) for _ in range(3))

        def exact_both():
            ha.exact_attn_forward(Q, K, V, causal=cfg["causal"], out=eo, lse=el, out_f32=out32)
            ha.exact_attn_backward(Q, K, V, eo, el, G, causal=cfg["causal"], workspace=ews, grads=egrads, out_f32=out32)

        ex_ms = time_call(torch, exact_both, 1, 2)
        result["exact_fwd_bwd_ms"] = round(ex_ms, 3)
        result["speedup_vs_exact"] = round(ex_ms / both_ms, 3)
        log(f"[bench] exact attention forward + backward {ex_ms:.2f} ms -> speed-up {ex_ms / both_ms:.2f}x")
        del eo, el, ews, egrads
    if not args.no_cpu_baseline:
        from oracle import hyperattn_oracle as orc
        Qh, Kh, Vh = host
        Gh = G[0, :1].float().cpu().numpy()[None]
        t0 = time.perf_counter()
        orc.hyperattn_forward(Qh, Kh, Vh, b=cfg["b"], m=cfg["m"], r=cfg["r"], causal=bool(cfg["causal"]),
                              n_min=cfg["n_min"], seed=cfg["seed"])
        ref = orc.hyperattn_backward(Qh, Kh, Vh, Gh, b=cfg["b"], m=cfg["m"], r=cfg["r"], causal=bool(cfg["causal"]),
                                     n_min=cfg["n_min"], seed=cfg["seed"])
        cpu_s = time.perf_counter() - t0
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
        errs = [float(np.linalg.norm(grads[i][0, 0].float().cpu().numpy() - ref[i][0, 0]) / np.linalg.norm(ref[i][0, 0]))
                for i in range(3)]
        result["cpu_baseline"] = {"value": round(cpu_s * 1e3 * B * H, 1), "unit": "ms", "cores": int(cores),
                                  "kind": "oracle",
                                  "sample": f"forward + backward of head 0 of batch 0 ({cpu_s:.1f} s measured), "
                                            f"multiplied by B*H = {B * H} heads"}
        result["parity_sample_rel_fro_err"] = {"dQ": errs[0], "dK": errs[1], "dV": errs[2]}
        log(f"[bench] oracle fwd+bwd {cpu_s:.1f} s for one head; relative Frobenius errors dQ/dK/dV {errs}")
    print(json.dumps(result), flush=True)


def probes(args, torch, ha):
    """The issue-rate probes of the library (measurement aid): cycles per instruction of what the
    attention loop consists of, and what that makes of one 64-key tile of the d = 128 kernel."""
    buf = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
    ha.ha_measure_issue_rates(buf)                      # warm-up
    raw = ha.ha_measure_issue_rates(buf)
    r = {k: round(max(v), 1) for k, v in raw.items()}   # the slower half of the workgroup
    per = {"v_exp_f32": r["exp_x64"] / 64, "v_fma_f32": r["fma_x64"] / 64, "v_cvt_pk_bf16_f32": r["cvt_pk_bf16_x64"] / 64,
           "v_max3_f32": r["max3_x64"] / 64, "v_mfma_f32_32x32x16_bf16": r["mfma_x16"] / 16}
    # two waves per SIMD issue the same loop, so a trip of both takes the printed cycles: per wave half of it
    per = {k: round(v / 2, 2) for k, v in per.items()}
    lds = {"ds_read_b128_B_per_clk_per_CU": round(65536 / r["lds_read_b128_64KiB"], 1),
           "ds_read_b64_tr_b16_B_per_clk_per_CU": round(32768 / r["lds_read_tr_b64_32KiB"], 1),
           "ds_write_b128_B_per_clk_per_CU": round(65536 / r["lds_write_b128_64KiB"], 1)}
    # one 64-key tile of one wave at d = 128: 32 MFMAs; 32 fma + 32 exp + 32 add + 16 cvt + 17 max3 + ~12 others;
    # 16 KiB of K fragments (b128 reads), 16 KiB of V^T fragments (transposing b64 reads), and 1/4 (four-wave
    # workgroups) of the 32 KiB tile written.  Per CU and round of eight wave-tiles (two per SIMD):
    mfma = 2 * 32 * per["v_mfma_f32_32x32x16_bf16"]
    valu = 2 * (32 * per["v_exp_f32"] + 16 * per["v_cvt_pk_bf16_f32"] + 17 * per["v_max3_f32"] +
                (32 + 32 + 12) * per["v_fma_f32"])
    lds_cyc = 8 * (16384 / lds["ds_read_b128_B_per_clk_per_CU"] + 16384 / lds["ds_read_b64_tr_b16_B_per_clk_per_CU"] +
                   8192 / lds["ds_write_b128_B_per_clk_per_CU"])
    tile = {"mfma_pipe_cycles_per_SIMD": round(mfma), "vector_issue_cycles_per_SIMD": round(valu),
            "lds_cycles_per_CU": round(lds_cyc)}
    log(f"[bench] cycles per instruction and wave: {per}")
    log(f"[bench] LDS: {lds}")
    log(f"[bench] one round of eight 64-key wave-tiles (d = 128): {tile}")
    print(json.dumps({"metric": "issue-rate probes", "unit": "shader cycles", "n_gpus": 1,
                      "cycles_per_trip": raw, "cycles_per_instruction_per_wave": per, "lds": lds,
                      "round_of_eight_wave_tiles_d128": tile}), flush=True)


def phases(args, torch, ha):
    """Where the workgroups of the two attention launches spend their cycles: the forward pass through
    the instrumented instantiation of the attention kernel (ha.hyperattn_forward_stamped), whose
    workgroups record the shader clock at their phase boundaries."""
    cfg = dict(synth_inputs.CONFIGS[args.workload])
    if args.heads > 0 or args.seq > 0:
        cfg["H"] = args.heads if args.heads > 0 else cfg["H"]
        cfg["n"] = args.seq if args.seq > 0 else cfg["n"]
    if cfg["dtype"] != "bf16":
        sys.exit("bench.py --phases: the instrumented kernel is the bf16 MFMA kernel")
    (Q, K, V), _ = device_inputs(cfg, torch)
    B, H, n, d = Q.shape
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    kw = dict(causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"], workspace=ws)
    call = (Q, K, V, cfg["b"], cfg["m"], cfg["r"])
    for _ in range(max(1, args.warmup)):
        ha.hyperattn_forward_stamped(*call, **kw)
    stage = {k: [] for k in ("node_attn", "causal_base", "total")}
    for _ in range(max(1, args.steps)):     # what the product instantiations take, for comparison
        ms = ha.hyperattn_forward_timed(*call, **kw)[2]
        for k in stage:
            stage[k].append(ms[k])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    _, _, node_st, base_st = ha.hyperattn_forward_stamped(*call, **kw)
    e1.record()
    torch.cuda.synchronize()

    def summary(st, groups):
        st = st.cpu().numpy().astype(np.int64)
        if st.shape[0] == 0:
            return None
        c = st[:, :5]
        ph = np.diff(c, axis=1)                     # list, gathers + first scores, loop, epilogue
        life = c[:, 4] - c[:, 0]
        ticks = st[:, 6] - st[:, 5]                 # 10 ns units
        tiles = ha.stamp_place(st[:, 7])[0]
        rows = []
        for name, sel in groups(tiles):
            if not sel.any():
                continue
            # the loop forms tiles - 1 score tiles (the first one is computed ahead of it) and tiles P V products
            loop_tiles = np.maximum(tiles[sel] - 0.5, 0.5)
            rows.append({"workgroups": name, "count": int(sel.sum()), "tiles": float(tiles[sel].mean()),
                         "cycles_life": float(life[sel].mean()),
                         "cycles_key_list": float(ph[sel, 0].mean()),
                         "cycles_gathers_first_scores": float(ph[sel, 1].mean()),
                         "cycles_loop": float(ph[sel, 2].mean()),
                         "cycles_loop_per_tile": float((ph[sel, 2] / loop_tiles).mean()),
                         "cycles_epilogue": float(ph[sel, 3].mean()),
                         "shader_clock_GHz": float((life[sel] / np.maximum(ticks[sel], 1)).mean() / 10.0)})
        return rows

    def residency(st):
        """How the launch's workgroups reached the CUs, from where and when each ran: share of the launch during
        which a CU held 0 / 1 / 2 of them, time until a finished workgroup was replaced, and the work (key tiles)
        each shader engine of an XCD was given."""
        st = st.cpu().numpy().astype(np.int64)
        if st.shape[0] == 0:
            return None
        tiles, xcd, se, cu = ha.stamp_place(st[:, 7])
        t0, t1 = st[:, 5], st[:, 6]
        start, span = t0.min(), t1.max() - t0.min()
        key = (xcd * 8 + se) * 16 + cu
        held = np.zeros(3)
        gaps, ends = [], []
        for k in np.unique(key):
            a, b = np.sort(t0[key == k]), np.sort(t1[key == k])
            ev = np.concatenate([np.stack([a, np.ones_like(a)], 1), np.stack([b, -np.ones_like(b)], 1)])
            ev = ev[np.argsort(ev[:, 0], kind="stable")]
            c, last = 0, start
            for t, dv in ev:
                held[min(c, 2)] += t - last
                last, c = t, c + int(dv)
            held[0] += start + span - last
            if len(a) > 2:
                gaps.append(a[2:] - b[:-2])      # the i-th end frees a slot for the (i + 2)-th start (two slots per CU)
            ends.append(b.max() - start)
        gaps = np.concatenate(gaps) if gaps else np.zeros(1)
        per_se = [[int(tiles[(xcd == x) & (se == e)].sum()) for e in np.unique(se)] for x in np.unique(xcd)]
        xcd_end = [float((t1[xcd == x].max() - start) / span) for x in np.unique(xcd)]
        return {"CUs": int(len(np.unique(key))), "span_ms": float(span) * 1e-5,
                "share_of_launch_with_0_1_2_resident": [float(v) for v in held / held.sum()],
                "replacement_us_mean_median_p90": [float(gaps.mean()) * 0.01, float(np.median(gaps)) * 0.01,
                                                   float(np.percentile(gaps, 90)) * 0.01],
                "workgroups_per_engine_xcd0": [int(((xcd == xcd.min()) & (se == e)).sum()) for e in np.unique(se)],
                "key_tiles_per_engine_by_xcd": per_se,
                "xcd_end_over_span": xcd_end,
                "cu_last_end_over_span_min_mean": [float(np.min(ends) / span), float(np.mean(ends) / span)]}

    node = summary(node_st, lambda t: [("all", t >= 0)])
    base = summary(base_st, lambda t: [("all", t >= 0), ("2-16 tiles", t <= 16), ("17-48 tiles", (t > 16) & (t <= 48)),
                                       ("49-64 tiles", t > 48)])
    res = {"metric": "attention workgroup phases", "unit": "shader cycles (mean over the launch's workgroups)",
           "n_gpus": 1, "config": {"workload": args.workload, "B": B, "H": H, "n": n, "d": d},
           "node_launch": node, "base_case_launch": base,
           "node_residency": residency(node_st), "base_case_residency": residency(base_st),
           "stamped_forward_ms": e0.elapsed_time(e1),
           "product_stage_ms_median": {k: float(np.median(v)) for k, v in stage.items()}}
    for k in ("node_launch", "base_case_launch"):
        for row in res[k] or []:
            log(f"[bench] {k} {row}")
    for k in ("node_residency", "base_case_residency"):
        if res[k]:
            log(f"[bench] {k} {res[k]}")
    print(json.dumps(res), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4_n131k_causal", choices=sorted(synth_inputs.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-exact", action="store_true")
    ap.add_argument("--backward", action="store_true", help="time forward + backward instead of the forward alone")
    ap.add_argument("--sweep", action="store_true", help="time the 12-head d=64 sweep shape at every length instead")
    ap.add_argument("--alg2", action="store_true", help="time Algorithm 2 as printed / Lemma 2's value sampling instead")
    ap.add_argument("--probes", action="store_true", help="run the library's issue-rate probes instead")
    ap.add_argument("--phases", action="store_true", help="cycle stamps of the attention workgroups' phases instead")
    ap.add_argument("--heads", type=int, default=0, help="override the workload's head count (profiling runs whose "
                                                          "32-bit hardware counters a full workload would overflow)")
    ap.add_argument("--seq", type=int, default=0, help="override the workload's sequence length (same purpose)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (heads would shard over GPUs with no communication); "
                 "use --gpus 1")

    import torch
    import paper_2310_05869_amd as ha
    ha.lib()  # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    if args.probes:
        return probes(args, torch, ha)
    if args.phases:
        return phases(args, torch, ha)
    if args.sweep:
        return sweep(args, torch, ha)
    if args.alg2:
        return alg2_bench(args, torch, ha)
    if args.backward:
        return backward_bench(args, torch, ha)

    cfg = dict(synth_inputs.CONFIGS[args.workload])
    if args.heads > 0 or args.seq > 0:
        cfg["H"] = args.heads if args.heads > 0 else cfg["H"]
        cfg["n"] = args.seq if args.seq > 0 else cfg["n"]
        args.workload += f"_H{cfg['H']}_n{cfg['n']}"
    B, H, n, d = cfg["B"], cfg["H"], cfg["n"], cfg["d"]
    log(f"[bench] workload {args.workload}: B{B} H{H} n{n} d{d} {cfg['dtype']} b{cfg['b']} m{cfg['m']} r{cfg['r']} "
        f"causal={cfg['causal']} n_min={cfg['n_min']}")
    # heads of batch 0 that the oracle is timed on (the cpu_baseline leg): about 10-30 s of host work
    cpu_heads = 1 if args.no_cpu_baseline else min(H, CPU_SAMPLE_HEADS)
    (Q, K, V), host = device_inputs(cfg, torch, host_heads=cpu_heads)
    shape = ha.make_shape(B, H, n, d, ha.HA_BF16 if cfg["dtype"] == "bf16" else ha.HA_FP32)
    params = ha.make_params(cfg["b"], cfg["m"], cfg["r"], cfg["causal"], cfg["n_min"], cfg["seed"])
    ws = ha.alloc_workspace(shape, params)
    out = torch.empty_like(Q)
    lse = torch.empty((B, H, n), dtype=torch.float32, device="cuda")
    kw = dict(causal=cfg["causal"], n_min=cfg["n_min"], seed=cfg["seed"], workspace=ws, out=out, lse=lse)

    def step():
        ha.hyperattn_forward(Q, K, V, cfg["b"], cfg["m"], cfg["r"], **kw)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    log(f"[bench] {ms_per_step:.3f} ms per forward")

    # per-stage durations from HIP events recorded on the launch stream
    stage = {k: 0.0 for k in ha.binding.STAGE_NAMES}
    totals = []
    for _ in range(args.steps):
        _, _, ms = ha.hyperattn_forward_timed(Q, K, V, cfg["b"], cfg["m"], cfg["r"], **kw)
        totals.append(ms["total"])
        for k, v in ms.items():
            stage[k] += v / args.steps
    log("[bench] stage ms: " + ", ".join(f"{k} {v:.3f}" for k, v in stage.items()))

    head0 = out[0, :cpu_heads].float().cpu().numpy()  # for the parity sample of the cpu_baseline leg
    gpu_codes = None
    if ha.ha_workspace_layout(shape, params).levels > 0:
        views = ha.workspace_views(ws, shape, params)
        gpu_codes = np.stack([views["codes_q"][:cpu_heads].cpu().numpy(), views["codes_k"][:cpu_heads].cpu().numpy()])
    work = algorithmic_work(cfg)
    stages_out = {k: round(v, 4) for k, v in stage.items()}
    tflops = lambda flop, ms: flop / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
    node_tf = tflops(work["node_flop"], stage["node_attn"])
    base_tf = tflops(work["base_flop"], stage["causal_base"])
    hash_gbs = work["hash_bytes"] / (stage["lsh_hash"] * 1e-3) / 1e9 if stage["lsh_hash"] > 0 else 0.0
    sort_gbs = work["sort_bytes"] / (stage["seg_sort"] * 1e-3) / 1e9 if stage["seg_sort"] > 0 else 0.0
    hs_ms = stage["lsh_hash"] + stage["seg_sort"]
    hash_sort_gbs = (work["hash_bytes"] + work["sort_bytes"]) / (hs_ms * 1e-3) / 1e9 if hs_ms > 0 else 0.0
    # the dominant kernel: the causal base case when there is one, else the node attention
    if stage["causal_base"] >= stage["node_attn"]:
        dom, dom_tf, dom_flop, dom_ms, key = ("attn_mfma_kernel<exact> (causal base case)", base_tf, work["base_flop"],
                                              stage["causal_base"], "base")
    else:
        dom, dom_tf, dom_flop, dom_ms, key = ("attn_mfma_kernel<node> (block + sampled)", node_tf, work["node_flop"],
                                              stage["node_attn"], "node")
    node_gbs = work["node_bytes"] / (stage["node_attn"] * 1e-3) / 1e9 if stage["node_attn"] > 0 else 0.0
    # Which roofline bounds the dominant kernel: the node attention of an unmasked problem needs
    # 4 d (b + m) flop and 4 d esz bytes per query row; at the chip's balance (2.5 PFLOP/s : 8 TB/s) that
    # is HBM-bound whenever b + m <= 312 esz, i.e. for every unmasked workload here.  The exact base
    # case (n_min / 2 keys per row on average) is bound by the matrix cores.
    hbm_bound = key == "node" and work["node_flop"] / PEAK_BF16_TFLOPS / 1e12 < work["node_bytes"] / PEAK_HBM_GBS / 1e9
    if hbm_bound:
        roofline = {"bound": "hbm", "kernel": dom, "achieved": round(node_gbs, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(node_gbs / PEAK_HBM_GBS, 4),
                    "traffic": measured_traffic_bytes(args.workload, key),
                    "bytes_per_launch": work["node_bytes"], "ms_per_launch": round(dom_ms, 4),
                    "mfma_frac": round(dom_tf / PEAK_BF16_TFLOPS, 4)}
    else:
        roofline = {"bound": "mfma", "kernel": dom, "achieved": round(dom_tf, 2), "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(dom_tf / PEAK_BF16_TFLOPS, 4),
                    "traffic": measured_traffic_bytes(args.workload, key),
                    "flop_per_launch": dom_flop, "ms_per_launch": round(dom_ms, 4)}

    result = {
        "metric": "HyperAttention fwd ms", "value": round(ms_per_step, 4), "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "B": B, "H": H, "n": n, "d": d, "b": cfg["b"], "m": cfg["m"],
                   "r": cfg["r"], "causal": bool(cfg["causal"]), "n_min": cfg["n_min"], "law": cfg["law"]},
        "roofline": roofline,
        "stages_ms": stages_out,
        "event_ms_median": round(float(np.median(totals)), 4), "event_ms_min": round(float(np.min(totals)), 4),
        "stage_rates": {"node_attn_TFLOPs": round(node_tf, 2), "node_attn_frac_mfma": round(node_tf / PEAK_BF16_TFLOPS, 4),
                        "node_attn_GBs": round(node_gbs, 1), "node_attn_frac_hbm": round(node_gbs / PEAK_HBM_GBS, 4),
                        "causal_base_TFLOPs": round(base_tf, 2), "causal_base_frac_mfma": round(base_tf / PEAK_BF16_TFLOPS, 4),
                        "lsh_hash_GBs": round(hash_gbs, 1), "lsh_hash_frac_hbm": round(hash_gbs / PEAK_HBM_GBS, 4),
                        "seg_sort_GBs": round(sort_gbs, 1), "seg_sort_frac_hbm": round(sort_gbs / PEAK_HBM_GBS, 4),
                        "hash_plus_sort_GBs": round(hash_sort_gbs, 1),
                        "hash_plus_sort_frac_hbm": round(hash_sort_gbs / PEAK_HBM_GBS, 4)},
        "tokens_per_s": round(B * n / (ms_per_step * 1e-3), 1),
    }

    # what this GPU sustains on code that does nothing else: MFMA chains in registers, streaming reads
    cal = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    cal.zero_()
    mfma_tf = ha.ha_measure_mfma_rate(cal, iters=4000)   # about 5 ms: as long as the dominant kernel runs
    read_gbs, copy_gbs = ha.ha_measure_hbm_rate(cal)
    del cal
    result["attainable"] = {"mfma_bf16_TFLOPs": round(mfma_tf, 1), "hbm_read_GBs": round(read_gbs, 1),
                            "hbm_copy_GBs": round(copy_gbs, 1)}
    if hbm_bound:
        roofline["frac_of_attainable"] = round(node_gbs / read_gbs, 4) if read_gbs > 0 else None
    else:
        roofline["frac_of_attainable"] = round(dom_tf / mfma_tf, 4) if mfma_tf > 0 else None
    result["stage_rates"]["lsh_hash_frac_of_attainable_read"] = round(hash_gbs / read_gbs, 4) if read_gbs > 0 else None
    log(f"[bench] attainable: MFMA {mfma_tf:.0f} TFLOP/s, HBM read {read_gbs:.0f} GB/s, copy {copy_gbs:.0f} GB/s")

    if not args.no_exact:
        eo = torch.empty_like(Q)
        el = torch.empty_like(lse)
        ha.exact_attn_forward(Q, K, V, causal=cfg["causal"], out=eo, lse=el)
        torch.cuda.synchronize()
        reps = 2
        t0 = time.perf_counter()
        for _ in range(reps):
            ha.exact_attn_forward(Q, K, V, causal=cfg["causal"], out=eo, lse=el)
        torch.cuda.synchronize()
        exact_ms = (time.perf_counter() - t0) * 1e3 / reps
        result["exact_attn_ms"] = round(exact_ms, 3)
        result["exact_attn_TFLOPs"] = round(tflops(work["exact_flop"], exact_ms), 2)
        result["speedup_vs_exact"] = round(exact_ms / ms_per_step, 3)
        log(f"[bench] exact attention {exact_ms:.2f} ms -> speedup {exact_ms / ms_per_step:.2f}x")
        del eo, el

    if args.workload == "cfg4_n131k_causal" and not args.no_exact:
        # the metric is quoted at n = 32k and 131k causal: the 32k point beside the headline workload
        del Q, K, V, out, lse, ws
        c3 = dict(synth_inputs.CONFIGS["cfg3_n32k_causal"])
        (Q3, K3, V3), _ = device_inputs(c3, torch)
        sh3 = ha.make_shape(c3["B"], c3["H"], c3["n"], c3["d"], ha.HA_BF16)
        ws3 = ha.alloc_workspace(sh3, ha.make_params(c3["b"], c3["m"], c3["r"], c3["causal"], c3["n_min"], c3["seed"]))
        o3 = torch.empty_like(Q3)
        l3 = torch.empty((c3["B"], c3["H"], c3["n"]), dtype=torch.float32, device="cuda")
        kw3 = dict(causal=1, n_min=c3["n_min"], seed=c3["seed"], workspace=ws3, out=o3, lse=l3)
        ms3 = time_call(torch, lambda: ha.hyperattn_forward(Q3, K3, V3, c3["b"], c3["m"], c3["r"], **kw3), 3, 20)
        ex3 = time_call(torch, lambda: ha.exact_attn_forward(Q3, K3, V3, causal=True, out=o3, lse=l3), 1, 5)
        result["also_cfg3_n32k_causal"] = {"ms": round(ms3, 4), "exact_attn_ms": round(ex3, 4),
                                           "speedup_vs_exact": round(ex3 / ms3, 3)}
        log(f"[bench] cfg3 (n=32768 causal): {ms3:.3f} ms, exact {ex3:.3f} ms, speed-up {ex3 / ms3:.2f}x")
        del Q3, K3, V3, o3, l3, ws3

    if not args.no_cpu_baseline:
        # The oracle (tests' reference, untuned) on the host cores, on head 0 of batch 0
        # of this very workload; scaled by the head count to the whole job.
        from oracle import hyperattn_oracle as orc
        Qh, Kh, Vh = host
        stages = {}
        okw = dict(b=cfg["b"], m=cfg["m"], r=cfg["r"], causal=bool(cfg["causal"]), n_min=cfg["n_min"], seed=cfg["seed"])
        t0 = time.perf_counter()
        ro, rl = orc.hyperattn_forward(Qh, Kh, Vh, stages=stages, **okw)
        cpu_s = time.perf_counter() - t0
        # bucket codes: sign bits the GPU resolved differently from the oracle (allowed only where the oracle's
        # |projection| < 1e-6); such bits are replayed in the oracle before the outputs are compared
        flips, unexplained = [], 0
        if gpu_codes is not None:
            inv = np.argsort(orc.gray_rank_table(cfg["r"]))
            for t in range(2):
                g, o = gpu_codes[t].astype(np.int64), stages["codes"][t]
                for bh, row in zip(*np.nonzero(g != o)):
                    diff = int(inv[g[bh, row]]) ^ int(inv[o[bh, row]])
                    for k in range(cfg["r"]):
                        if (diff >> k) & 1:
                            flips.append((t, int(bh), int(row), k))
                            unexplained += int(abs(stages["proj"][t, bh, row, k]) >= 1e-6)
            if flips:
                ro, rl = orc.hyperattn_forward(Qh, Kh, Vh, flip=flips, **okw)
            result["sign_bits"] = {"checked": int(2 * cpu_heads * n * cfg["r"]), "near_zero_disagreements": len(flips),
                                   "disagreements_at_1e-6_or_more": unexplained}
        got = head0.astype(np.float64)
        err = float(np.abs(got - ro[0]).max())
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
        try:
            from threadpoolctl import threadpool_info
            nt = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
            threads = max(nt) if nt else cores
        except Exception:
            threads = cores
        result["cpu_baseline"] = {"value": round(cpu_s * 1e3 * B * H / cpu_heads, 1), "unit": "ms", "cores": int(cores),
                                  "blas_threads": int(threads), "cpu": host_cpu_model(), "kind": "oracle",
                                  "sample": f"heads 0..{cpu_heads - 1} of batch 0 of the same workload ({cpu_s:.1f} s "
                                            f"measured), scaled to B*H = {B * H} heads"}
        result["parity_sample_max_abs_err"] = err
        log(f"[bench] oracle {cpu_s:.1f} s for {cpu_heads} head(s) on {cores} cores ({threads} BLAS threads); GPU-vs-oracle "
            f"max abs err on them {err:.2e}; sign bits that differ: {len(flips)} ({unexplained} not near zero)")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
