"""ctypes binding of libhyperattn.so: argument marshalling only.

Every function has the name and meaning of the C entry point it wraps (see
include/hyperattn.h).  PyTorch supplies device memory and the current HIP
stream; every step of the computation runs in the library's kernels.  There is
no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_uint64, c_void_p

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhyperattn.so")

HA_BF16, HA_FP32 = 0, 1


class HaShape(ctypes.Structure):
    _fields_ = [("B", c_int32), ("H", c_int32), ("n", c_int32), ("d", c_int32), ("dtype", c_int32)]


class HaParams(ctypes.Structure):
    _fields_ = [("b", c_int32), ("m", c_int32), ("r", c_int32), ("causal", c_int32), ("n_min", c_int32),
                ("seed", c_uint64)]


class HaWsLayout(ctypes.Structure):
    _fields_ = [("levels", c_int32), ("total_nodes", c_int32), ("n_cov", c_int64),
                ("codes_q", c_size_t), ("codes_k", c_size_t), ("perm_q", c_size_t), ("perm_k", c_size_t),
                ("pos_k", c_size_t), ("samples", c_size_t), ("samp_blk", c_size_t), ("proj", c_size_t), ("sort_hist", c_size_t),
                ("part_o", c_size_t),
                ("part_l", c_size_t), ("total_bytes", c_size_t)]


class HaBwdWsLayout(ctypes.Structure):
    _fields_ = [(k, c_size_t) for k in ("delta", "acc_a", "acc_b", "samp_k", "samp_v", "total_bytes")]


class HaAlg2Options(ctypes.Structure):
    _fields_ = [("cap_scale", c_float), ("kappa", c_float), ("vnorm_sampling", c_int32)]


class HaAlg2WsLayout(ctypes.Structure):
    _fields_ = [(k, c_size_t) for k in ("forward_bytes", "pos_q", "tau_rows", "log_unmasked_t", "log_tau", "vnorm_w",
                                        "vnorm_prefix", "vnorm_samples", "vnorm_logw",
                                        "log_unmasked_parts",
                                        "total_bytes")]


class HyperAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_SIGNATURES = {
    "ha_workspace_layout": (c_int, [POINTER(HaShape), POINTER(HaParams), POINTER(HaWsLayout)]),
    "ha_workspace_bytes": (c_size_t, [POINTER(HaShape), POINTER(HaParams)]),
    "hyperattn_forward": (c_int, [c_void_p] * 5 + [POINTER(HaShape), POINTER(HaParams), c_void_p, c_size_t, c_void_p]),
    "hyperattn_forward_static": (c_int, [c_void_p] * 5 + [POINTER(HaShape), POINTER(HaParams), c_void_p]),
    "ha_static_scratch_bytes": (c_size_t, []),
    "hyperattn_forward_ex": (c_int, [c_void_p] * 5 + [POINTER(HaShape), POINTER(HaParams), c_void_p, c_void_p,
                                                     c_void_p, c_size_t, c_void_p]),
    "hyperattn_forward_timed": (c_int, [c_void_p] * 5 + [POINTER(HaShape), POINTER(HaParams), c_void_p, c_size_t,
                                                        c_void_p, POINTER(c_float)]),
    "ha_forward_workgroups": (c_int, [POINTER(HaShape), POINTER(HaParams), POINTER(c_int64), POINTER(c_int64)]),
    "hyperattn_forward_stamped": (c_int, [c_void_p] * 5 + [POINTER(HaShape), POINTER(HaParams), c_void_p, c_size_t,
                                                          c_void_p, c_void_p, c_size_t, c_void_p, c_size_t]),
    "exact_attn_forward": (c_int, [c_void_p] * 5 + [POINTER(HaShape), c_int, c_void_p]),
    "ha_make_projection": (c_int, [c_uint64, c_int32, c_int32, POINTER(c_float)]),
    "ha_make_samples": (c_int, [c_uint64, c_int32, c_int32, c_int32, c_int32, POINTER(c_int32)]),
    "ha_lsh_hash": (c_int, [c_void_p, c_void_p, c_int64, c_int32, c_int32, c_void_p, c_int32, c_void_p]),
    "ha_seg_sort": (c_int, [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p]),
    "ha_gather_rows": (c_int, [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int32, c_void_p]),
    "ha_block_attn": (c_int, [c_void_p] * 5 + [c_int32] * 5 + [c_void_p]),
    "ha_sampled_attn": (c_int, [c_void_p] * 7 + [c_int32] * 6 + [c_void_p]),
    "ha_merge_unpermute": (c_int, [c_void_p] * 7 + [c_int32] * 4 + [c_void_p]),
    "ha_backward_workspace_layout": (c_int, [POINTER(HaShape), POINTER(HaParams), POINTER(HaBwdWsLayout)]),
    "ha_backward_workspace_bytes": (c_size_t, [POINTER(HaShape), POINTER(HaParams)]),
    "hyperattn_forward_train": (c_int, [c_void_p] * 6 + [POINTER(HaShape), POINTER(HaParams), c_void_p, c_size_t,
                                                        c_void_p]),
    "exact_attn_forward_train": (c_int, [c_void_p] * 6 + [POINTER(HaShape), c_int, c_void_p]),
    "hyperattn_backward": (c_int, [c_void_p] * 10 + [POINTER(HaShape), POINTER(HaParams), c_void_p, c_size_t, c_void_p,
                                                    c_size_t, c_void_p]),
    "hyperattn_backward_timed": (c_int, [c_void_p] * 10 + [POINTER(HaShape), POINTER(HaParams), c_void_p, c_size_t,
                                                          c_void_p, c_size_t, c_void_p, POINTER(c_float)]),
    "exact_attn_backward": (c_int, [c_void_p] * 10 + [POINTER(HaShape), c_int, c_void_p, c_size_t, c_void_p]),
    "exact_attn_backward_workspace_bytes": (c_size_t, [POINTER(HaShape)]),
    "ha_alg2_workspace_layout": (c_int, [POINTER(HaShape), POINTER(HaParams), POINTER(HaAlg2WsLayout)]),
    "ha_alg2_workspace_bytes": (c_size_t, [POINTER(HaShape), POINTER(HaParams)]),
    "hyperattn_forward_alg2": (c_int, [c_void_p] * 5 + [POINTER(HaShape), POINTER(HaParams), POINTER(HaAlg2Options),
                                                       c_void_p, c_size_t, c_void_p]),
    "ha_measure_mfma_rate": (c_int, [c_void_p, c_size_t, c_int32, POINTER(c_float), c_void_p]),
    "ha_measure_hbm_rate": (c_int, [c_void_p, c_size_t, POINTER(c_float), POINTER(c_float), c_void_p]),
    "ha_issue_probe_count": (c_int32, []),
    "ha_measure_issue_rates": (c_int, [c_void_p, c_size_t, POINTER(c_float), c_void_p]),
    "ha_strerror": (c_char_p, [c_int]),
}

_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2310_05869_amd.build`")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def strerror(status: int) -> str:
    return lib().ha_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise HyperAttnError(status, where)


# ---------------------------------------------------------------- host-only calls
def make_shape(B, H, n, d, dtype) -> HaShape:
    return HaShape(B, H, n, d, dtype)


def make_params(b, m, r, causal=False, n_min=4096, seed=0) -> HaParams:
    return HaParams(b, m, r, int(bool(causal)), n_min, seed)


def ha_workspace_layout(shape: HaShape, params: HaParams) -> HaWsLayout:
    lay = HaWsLayout()
    _check(lib().ha_workspace_layout(ctypes.byref(shape), ctypes.byref(params), ctypes.byref(lay)),
           "ha_workspace_layout")
    return lay


def ha_workspace_bytes(shape: HaShape, params: HaParams) -> int:
    return int(lib().ha_workspace_bytes(ctypes.byref(shape), ctypes.byref(params)))


def ha_make_projection(seed: int, d: int, r: int) -> np.ndarray:
    R = np.empty((d, r), dtype=np.float32)
    _check(lib().ha_make_projection(seed, d, r, R.ctypes.data_as(POINTER(c_float))), "ha_make_projection")
    return R


def ha_make_samples(seed: int, level: int, node: int, n_keys: int, m: int) -> np.ndarray:
    idx = np.empty(max(m, 1), dtype=np.int32)
    _check(lib().ha_make_samples(seed, level, node, n_keys, m, idx.ctypes.data_as(POINTER(c_int32))),
           "ha_make_samples")
    return idx[:m]


# ---------------------------------------------------------------- device calls
def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return HA_BF16
    if t.dtype == torch.float32:
        return HA_FP32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _dev(t, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(stream):
    torch = _torch()
    return (torch.cuda.current_stream() if stream is None else stream).cuda_stream


def _expect(t, name, shape, dtype, like):
    """The kernels take sizes from Q alone: every other tensor must have the shape, dtype and device they assume."""
    if t is None:
        return
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if t.dtype != dtype:
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    if t.device != like.device:
        raise ValueError(f"{name} is on {t.device}, expected {like.device}")


def _expect_qkv(Q, **others):
    """others: name=tensor pairs that must match Q in shape, dtype and device (None entries are skipped)."""
    if Q.dim() != 4:
        raise ValueError(f"Q has shape {tuple(Q.shape)}, expected [B, H, n, d]")
    for name, t in others.items():
        _expect(t, name, Q.shape, Q.dtype, Q)


def _expect_f32(Q, shape, **others):
    torch = _torch()
    for name, t in others.items():
        _expect(t, name, shape, torch.float32, Q)


def _on_stream(stream, *tensors):
    """Memory this call allocated itself and lets go of on return must not be handed out again by the
    caching allocator while kernels on a stream other than the current one still use it."""
    torch = _torch()
    if stream is not None and stream != torch.cuda.current_stream():
        for t in tensors:
            if t is not None:
                t.record_stream(stream)


def _check_samples(samples, shape: HaShape, params: HaParams, Q):
    """int32 [total_nodes, m], every index inside its node (the C call can only clamp: it never reads
    device memory on the host)."""
    torch = _torch()
    lay = ha_workspace_layout(shape, params)
    _expect(samples, "samples", (lay.total_nodes, params.m), torch.int32, Q)
    if samples.numel() == 0:
        return
    if params.causal:
        level = torch.floor(torch.log2(torch.arange(1, lay.total_nodes + 1, device=samples.device).float())).long()
        size = (shape.n >> (level + 1)).to(torch.int32)[:, None]
    else:
        size = shape.n
    if bool((samples < 0).any()) or bool((samples >= size).any()):
        raise HyperAttnError(-3, "hyperattn_forward: a sample index lies outside its node")


def alloc_workspace(shape: HaShape, params: HaParams, device="cuda"):
    torch = _torch()
    nbytes = ha_workspace_bytes(shape, params)
    if nbytes == 0:
        _check(lib().ha_workspace_layout(ctypes.byref(shape), ctypes.byref(params), ctypes.byref(HaWsLayout())),
               "ha_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def hyperattn_forward(Q, K, V, b, m, r, causal=False, n_min=4096, seed=0, R=None, samples=None,
                      workspace=None, out=None, lse=None, stream=None, out_f32=None):
    """out, lse = HyperAttention(Q, K, V).  Q, K, V: [B, H, n, d] device tensors
    (bf16 or fp32).  R (float32 [d, r]) / samples (int32 [total_nodes, m]) are
    optional device tensors overriding the seed-derived draws.  out_f32 (float32
    [B, H, n, d]), if given, receives the output before its rounding to bf16
    (hyperattn_forward_train): pass it on to hyperattn_backward."""
    torch = _torch()
    _expect_qkv(Q, K=K, V=V, out=out)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    params = make_params(b, m, r, causal, n_min, seed)
    _expect_f32(Q, (B, H, n), lse=lse)
    _expect_f32(Q, (B, H, n, d), out_f32=out_f32)
    _expect_f32(Q, (d, r), R=R)
    if samples is not None:
        _check_samples(samples, shape, params, Q)
    own_ws = workspace is None
    if own_ws:
        workspace = alloc_workspace(shape, params, Q.device)
    if out is None:
        out = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((B, H, n), dtype=torch.float32, device=Q.device)
    _on_stream(stream, workspace if own_ws else None)
    ptrs = [_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"), _dev(lse, "lse")]
    if out_f32 is not None:
        if R is not None or samples is not None:
            raise ValueError("out_f32 goes with the seed-derived draws")
        st = lib().hyperattn_forward_train(*ptrs, _dev(out_f32, "out_f32"), ctypes.byref(shape), ctypes.byref(params),
                                           workspace.data_ptr(), workspace.numel(), _stream(stream))
    elif R is None and samples is None:
        st = lib().hyperattn_forward(*ptrs, ctypes.byref(shape), ctypes.byref(params), workspace.data_ptr(),
                                     workspace.numel(), _stream(stream))
    else:
        st = lib().hyperattn_forward_ex(*ptrs, ctypes.byref(shape), ctypes.byref(params),
                                        None if R is None else _dev(R, "R"),
                                        None if samples is None else _dev(samples, "samples"),
                                        workspace.data_ptr(), workspace.numel(), _stream(stream))
    _check(st, "hyperattn_forward")
    return out, lse


def ha_static_scratch_bytes() -> int:
    return int(lib().ha_static_scratch_bytes())


def hyperattn_forward_static(Q, K, V, out, lse, b, m, r, causal=False, n_min=4096, seed=0, stream=None):
    """hyperattn_forward on the library's built-in scratch array: the call
    allocates nothing, so the caller passes out and lse."""
    _expect_qkv(Q, K=K, V=V, out=out)
    _expect_f32(Q, tuple(Q.shape[:3]), lse=lse)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    params = make_params(b, m, r, causal, n_min, seed)
    st = lib().hyperattn_forward_static(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"), _dev(lse, "lse"),
                                        ctypes.byref(shape), ctypes.byref(params), _stream(stream))
    _check(st, "hyperattn_forward_static")
    return out, lse


STAGE_NAMES = ("prep", "lsh_hash", "seg_sort", "node_attn", "causal_base", "total")


def hyperattn_forward_timed(Q, K, V, b, m, r, causal=False, n_min=4096, seed=0, workspace=None, out=None,
                            lse=None, stream=None):
    """As hyperattn_forward, but waits for the result and also returns the
    per-stage milliseconds (dict keyed by STAGE_NAMES) from HIP events."""
    torch = _torch()
    _expect_qkv(Q, K=K, V=V, out=out)
    _expect_f32(Q, tuple(Q.shape[:3]), lse=lse)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    params = make_params(b, m, r, causal, n_min, seed)
    if workspace is None:
        workspace = alloc_workspace(shape, params, Q.device)
    if out is None:
        out = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((B, H, n), dtype=torch.float32, device=Q.device)
    ms = (c_float * 6)()
    st = lib().hyperattn_forward_timed(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"), _dev(lse, "lse"),
                                       ctypes.byref(shape), ctypes.byref(params), workspace.data_ptr(),
                                       workspace.numel(), _stream(stream), ms)
    _check(st, "hyperattn_forward_timed")
    return out, lse, dict(zip(STAGE_NAMES, [float(x) for x in ms]))


STAMP_WORDS = 8
STAMP_NAMES = ("cycles_entry", "cycles_list", "cycles_loop", "cycles_epilogue", "cycles_end", "ticks_entry", "ticks_end",
               "tiles_and_place")


def stamp_place(word):
    """Splits word 7 of stamp records (an int64 numpy array or tensor): tiles, XCD, shader engine, CU."""
    return word & 0xFFFF, (word >> 48) & 0xF, (word >> (16 + 13)) & 0x7, (word >> (16 + 8)) & 0xF


def ha_forward_workgroups(shape, params):
    """(node workgroups, base-case workgroups) of the forward pass's two attention launches."""
    nw, bw = c_int64(0), c_int64(0)
    _check(lib().ha_forward_workgroups(ctypes.byref(shape), ctypes.byref(params), ctypes.byref(nw), ctypes.byref(bw)),
           "ha_forward_workgroups")
    return int(nw.value), int(bw.value)


def hyperattn_forward_stamped(Q, K, V, b, m, r, causal=False, n_min=4096, seed=0, workspace=None, out=None, lse=None,
                              stream=None):
    """As hyperattn_forward (bf16 tensors), through the instrumented instantiation of the attention kernel.
    Returns (out, lse, node_stamps, base_stamps): int64 tensors [workgroups, STAMP_WORDS] in the order of
    STAMP_NAMES, one row per workgroup of the node launch / the base-case launch."""
    torch = _torch()
    _expect_qkv(Q, K=K, V=V, out=out)
    _expect_f32(Q, tuple(Q.shape[:3]), lse=lse)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    params = make_params(b, m, r, causal, n_min, seed)
    if workspace is None:
        workspace = alloc_workspace(shape, params, Q.device)
    if out is None:
        out = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((B, H, n), dtype=torch.float32, device=Q.device)
    nw, bw = ha_forward_workgroups(shape, params)
    node_st = torch.zeros((nw, STAMP_WORDS), dtype=torch.int64, device=Q.device)
    base_st = torch.zeros((bw, STAMP_WORDS), dtype=torch.int64, device=Q.device)
    _check(lib().hyperattn_forward_stamped(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"), _dev(lse, "lse"),
                                           ctypes.byref(shape), ctypes.byref(params), workspace.data_ptr(),
                                           workspace.numel(), _stream(stream),
                                           node_st.data_ptr() if nw else None, node_st.numel() * 8,
                                           base_st.data_ptr() if bw else None, base_st.numel() * 8),
           "hyperattn_forward_stamped")
    return out, lse, node_st, base_st


def exact_attn_forward(Q, K, V, causal=False, out=None, lse=None, stream=None, out_f32=None):
    torch = _torch()
    _expect_qkv(Q, K=K, V=V, out=out)
    _expect_f32(Q, tuple(Q.shape[:3]), lse=lse)
    _expect_f32(Q, tuple(Q.shape), out_f32=out_f32)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    if out is None:
        out = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((B, H, n), dtype=torch.float32, device=Q.device)
    if out_f32 is not None:
        _check(lib().exact_attn_forward_train(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"), _dev(lse, "lse"),
                                              _dev(out_f32, "out_f32"), ctypes.byref(shape), int(bool(causal)),
                                              _stream(stream)), "exact_attn_forward_train")
        return out, lse
    _check(lib().exact_attn_forward(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"), _dev(lse, "lse"),
                                    ctypes.byref(shape), int(bool(causal)), _stream(stream)), "exact_attn_forward")
    return out, lse


def workspace_views(workspace, shape: HaShape, params: HaParams):
    """Typed views of the workspace regions after a forward call."""
    torch = _torch()
    lay = ha_workspace_layout(shape, params)
    BH, n, d = shape.B * shape.H, shape.n, shape.d
    cov = lay.levels * BH * lay.n_cov

    def view(off, count, dtype, shp):
        esz = torch.empty((), dtype=dtype).element_size()
        return workspace[off:off + count * esz].view(dtype).view(*shp)

    v = {
        "layout": lay,
        "codes_q": view(lay.codes_q, BH * n, torch.uint8, (BH, n)),
        "codes_k": view(lay.codes_k, BH * n, torch.uint8, (BH, n)),
        "proj": view(lay.proj, d * params.r, torch.float32, (d, params.r)),
    }
    if cov:
        for name in ("perm_q", "perm_k", "pos_k"):
            v[name] = view(getattr(lay, name), cov, torch.int32, (lay.levels, BH, lay.n_cov))
        if params.m and lay.total_nodes:
            v["samples"] = view(lay.samples, lay.total_nodes * params.m, torch.int32, (lay.total_nodes, params.m))
            v["samp_blk"] = view(lay.samp_blk, BH * lay.total_nodes * params.m, torch.int32,
                                 (BH, lay.total_nodes, params.m))
        if params.causal:
            pdt = torch.bfloat16 if shape.dtype == HA_BF16 else torch.float32
            v["part_o"] = view(lay.part_o, cov * d, pdt, (lay.levels, BH, lay.n_cov, d))
            v["part_l"] = view(lay.part_l, cov, torch.float32, (lay.levels, BH, lay.n_cov))
    return v


def ha_lsh_hash(X, R, stream=None):
    """codes (uint8 [rows]) of the rows of X ([..., d]); R: float32 [d, r] device tensor."""
    torch = _torch()
    d = X.shape[-1]
    rows = X.numel() // d
    codes = torch.empty(rows, dtype=torch.uint8, device=X.device)
    _check(lib().ha_lsh_hash(_dev(X, "X"), codes.data_ptr(), rows, d, _dtype_code(X), _dev(R, "R"), R.shape[1],
                             _stream(stream)), "ha_lsh_hash")
    return codes.view(X.shape[:-1])


def ha_seg_sort(codes, stream=None):
    """codes: uint8 [n_seg, seg_len] -> (perm, pos) int32 [n_seg, seg_len]."""
    torch = _torch()
    n_seg, seg_len = codes.shape
    perm = torch.empty((n_seg, seg_len), dtype=torch.int32, device=codes.device)
    pos = torch.empty_like(perm)
    _check(lib().ha_seg_sort(_dev(codes, "codes"), perm.data_ptr(), pos.data_ptr(), n_seg, seg_len,
                             _stream(stream)), "ha_seg_sort")
    return perm, pos


def ha_gather_rows(src, idx, stream=None):
    """src: [groups, n, d]; idx: int32 [groups, n] -> dst[g, p] = src[g, idx[g, p]]."""
    torch = _torch()
    groups, n, d = src.shape
    dst = torch.empty_like(src)
    _check(lib().ha_gather_rows(_dev(src, "src"), _dev(idx, "idx"), dst.data_ptr(), groups, n, d,
                                _dtype_code(src), _stream(stream)), "ha_gather_rows")
    return dst


def ha_block_attn(Qs, Ks, Vs, b, stream=None):
    torch = _torch()
    groups, n, d = Qs.shape
    o = torch.empty((groups, n, d), dtype=torch.float32, device=Qs.device)
    l = torch.empty((groups, n), dtype=torch.float32, device=Qs.device)
    _check(lib().ha_block_attn(_dev(Qs, "Qs"), _dev(Ks, "Ks"), _dev(Vs, "Vs"), o.data_ptr(), l.data_ptr(),
                               groups, n, d, _dtype_code(Qs), b, _stream(stream)), "ha_block_attn")
    return o, l


def ha_sampled_attn(Qs, K, V, samples, pos_k, b, stream=None):
    torch = _torch()
    groups, n, d = Qs.shape
    m = samples.numel()
    o = torch.empty((groups, n, d), dtype=torch.float32, device=Qs.device)
    l = torch.empty((groups, n), dtype=torch.float32, device=Qs.device)
    _check(lib().ha_sampled_attn(_dev(Qs, "Qs"), _dev(K, "K"), _dev(V, "V"), _dev(samples, "samples"),
                                 _dev(pos_k, "pos_k"), o.data_ptr(), l.data_ptr(), groups, n, d,
                                 _dtype_code(Qs), b, m, _stream(stream)), "ha_sampled_attn")
    return o, l


def ha_merge_unpermute(o_b, lse_b, o_r, lse_r, perm_q, dtype, stream=None):
    torch = _torch()
    groups, n, d = o_b.shape
    out = torch.empty((groups, n, d), dtype=dtype, device=o_b.device)
    lse = torch.empty((groups, n), dtype=torch.float32, device=o_b.device)
    _check(lib().ha_merge_unpermute(_dev(o_b, "o_b"), _dev(lse_b, "lse_b"), _dev(o_r, "o_r"), _dev(lse_r, "lse_r"),
                                    _dev(perm_q, "perm_q"), out.data_ptr(), lse.data_ptr(), groups, n, d,
                                    _dtype_code(out), _stream(stream)), "ha_merge_unpermute")
    return out, lse


def ha_measure_mfma_rate(buf, iters=2000, stream=None) -> float:
    """bf16 matrix-core TFLOP/s of register-resident MFMA chains; buf: device tensor >= 512 KiB."""
    val = c_float(0.0)
    _check(lib().ha_measure_mfma_rate(_dev(buf, "buf"), buf.numel() * buf.element_size(), int(iters),
                                      ctypes.byref(val), _stream(stream)), "ha_measure_mfma_rate")
    return float(val.value)


def ha_measure_hbm_rate(buf, stream=None):
    """(read GB/s, copy GB/s) of streaming kernels over buf, a device tensor well beyond the caches."""
    rd, cp = c_float(0.0), c_float(0.0)
    _check(lib().ha_measure_hbm_rate(_dev(buf, "buf"), buf.numel() * buf.element_size(), ctypes.byref(rd),
                                     ctypes.byref(cp), _stream(stream)), "ha_measure_hbm_rate")
    return float(rd.value), float(cp.value)


ISSUE_PROBES = ("exp_x64", "fma_x64", "cvt_pk_bf16_x64", "max3_x64", "mfma_x16", "mfma_x16_fma4", "mfma_x16_fma7",
                "mfma_x16_exp1_fma3", "mfma_x16_exp1_fma4", "split_mfma16_vs_exp16_fma48", "lds_read_b128_64KiB",
                "lds_read_tr_b64_32KiB", "lds_write_b128_64KiB")


def ha_issue_probe_count() -> int:
    return int(lib().ha_issue_probe_count())


def ha_measure_issue_rates(buf, stream=None):
    """{probe: (cycles per trip of the first wave of waves 0-3, of waves 4-7)}; see include/hyperattn.h."""
    n = ha_issue_probe_count()
    assert n == len(ISSUE_PROBES)
    vals = (c_float * (2 * n))()
    _check(lib().ha_measure_issue_rates(_dev(buf, "buf"), buf.numel() * buf.element_size(), vals, _stream(stream)),
           "ha_measure_issue_rates")
    return {name: (float(vals[2 * i]), float(vals[2 * i + 1])) for i, name in enumerate(ISSUE_PROBES)}


# ---------------------------------------------------------------- backward pass
BWD_STAGE_NAMES = ("delta", "dq_nodes", "dq_base", "dkv_block", "dkv_sampled", "dkv_base", "sums", "total")


def ha_backward_workspace_bytes(shape: HaShape, params: HaParams) -> int:
    lay = HaBwdWsLayout()
    _check(lib().ha_backward_workspace_layout(ctypes.byref(shape), ctypes.byref(params), ctypes.byref(lay)),
           "ha_backward_workspace_layout")
    return int(lay.total_bytes)


def alloc_backward_workspace(shape: HaShape, params: HaParams, device="cuda"):
    return _torch().empty(ha_backward_workspace_bytes(shape, params), dtype=_torch().uint8, device=device)


def _backward_call(timed, Q, K, V, out, lse, d_out, b, m, r, causal, n_min, seed, fwd_workspace, bwd_workspace,
                   grads, stream, out_f32=None):
    torch = _torch()
    dQ, dK, dV = grads if grads is not None else (torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V))
    _expect_qkv(Q, K=K, V=V, out=out, d_out=d_out, dQ=dQ, dK=dK, dV=dV)
    _expect_f32(Q, tuple(Q.shape[:3]), lse=lse)
    _expect_f32(Q, tuple(Q.shape), out_f32=out_f32)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    params = make_params(b, m, r, causal, n_min, seed)
    own_ws = bwd_workspace is None
    if own_ws:
        bwd_workspace = alloc_backward_workspace(shape, params, Q.device)
    _on_stream(stream, bwd_workspace if own_ws else None)
    args = [_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"),
            None if out_f32 is None else _dev(out_f32, "out_f32"), _dev(lse, "lse"), _dev(d_out, "d_out"),
            _dev(dQ, "dQ"), _dev(dK, "dK"), _dev(dV, "dV"), ctypes.byref(shape), ctypes.byref(params),
            fwd_workspace.data_ptr(), fwd_workspace.numel(), bwd_workspace.data_ptr(), bwd_workspace.numel(),
            _stream(stream)]
    if not timed:
        _check(lib().hyperattn_backward(*args), "hyperattn_backward")
        return dQ, dK, dV
    ms = (c_float * 8)()
    _check(lib().hyperattn_backward_timed(*args, ms), "hyperattn_backward_timed")
    return dQ, dK, dV, dict(zip(BWD_STAGE_NAMES, [float(x) for x in ms]))


def hyperattn_backward(Q, K, V, out, lse, d_out, b, m, r, causal=False, n_min=4096, seed=0, fwd_workspace=None,
                       bwd_workspace=None, grads=None, stream=None, out_f32=None):
    """dQ, dK, dV of sum(out * d_out).  out, lse and fwd_workspace are what
    hyperattn_forward produced / used for the same arguments (bf16 or fp32 tensors);
    out_f32 (bf16 tensors only), if the forward wrote one, makes delta = <d_out, out>
    free of the output's bf16 rounding."""
    if fwd_workspace is None:
        raise ValueError("hyperattn_backward needs the workspace of the forward call")
    return _backward_call(False, Q, K, V, out, lse, d_out, b, m, r, causal, n_min, seed, fwd_workspace, bwd_workspace,
                          grads, stream, out_f32)


def hyperattn_backward_timed(Q, K, V, out, lse, d_out, b, m, r, causal=False, n_min=4096, seed=0, fwd_workspace=None,
                             bwd_workspace=None, grads=None, stream=None, out_f32=None):
    """As hyperattn_backward, but waits and also returns per-stage milliseconds (BWD_STAGE_NAMES)."""
    if fwd_workspace is None:
        raise ValueError("hyperattn_backward_timed needs the workspace of the forward call")
    return _backward_call(True, Q, K, V, out, lse, d_out, b, m, r, causal, n_min, seed, fwd_workspace, bwd_workspace,
                          grads, stream, out_f32)


def exact_attn_backward(Q, K, V, out, lse, d_out, causal=False, workspace=None, grads=None, stream=None, out_f32=None):
    torch = _torch()
    dQ, dK, dV = grads if grads is not None else (torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V))
    _expect_qkv(Q, K=K, V=V, out=out, d_out=d_out, dQ=dQ, dK=dK, dV=dV)
    _expect_f32(Q, tuple(Q.shape[:3]), lse=lse)
    _expect_f32(Q, tuple(Q.shape), out_f32=out_f32)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    own_ws = workspace is None
    if own_ws:
        workspace = torch.empty(int(lib().exact_attn_backward_workspace_bytes(ctypes.byref(shape))), dtype=torch.uint8,
                                device=Q.device)
    _on_stream(stream, workspace if own_ws else None)
    _check(lib().exact_attn_backward(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"),
                                     None if out_f32 is None else _dev(out_f32, "out_f32"), _dev(lse, "lse"),
                                     _dev(d_out, "d_out"), _dev(dQ, "dQ"), _dev(dK, "dK"), _dev(dV, "dV"),
                                     ctypes.byref(shape), int(bool(causal)), workspace.data_ptr(), workspace.numel(),
                                     _stream(stream)), "exact_attn_backward")
    return dQ, dK, dV


# ---------------------------------------------------------------- Algorithm 2 as printed / Lemma 2
def ha_alg2_workspace_layout(shape: HaShape, params: HaParams) -> HaAlg2WsLayout:
    lay = HaAlg2WsLayout()
    _check(lib().ha_alg2_workspace_layout(ctypes.byref(shape), ctypes.byref(params), ctypes.byref(lay)),
           "ha_alg2_workspace_layout")
    return lay


def hyperattn_forward_alg2(Q, K, V, b, m, r, seed=0, cap_scale=0.0, kappa=0.0, vnorm_sampling=False, workspace=None,
                           out=None, lse=None, stream=None, causal=False, n_min=4096):
    """HyperAttention with Algorithm 2's caps and, optionally, Lemma 2's value sampling by squared
    row norm (at every off-diagonal node of Algorithm 4 when causal).  Returns (out, log d~, workspace)."""
    torch = _torch()
    _expect_qkv(Q, K=K, V=V, out=out)
    _expect_f32(Q, tuple(Q.shape[:3]), lse=lse)
    B, H, n, d = Q.shape
    shape = make_shape(B, H, n, d, _dtype_code(Q))
    params = make_params(b, m, r, causal, n_min, seed)
    if workspace is None:
        workspace = torch.empty(int(ha_alg2_workspace_layout(shape, params).total_bytes), dtype=torch.uint8,
                                device=Q.device)
    if out is None:
        out = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((B, H, n), dtype=torch.float32, device=Q.device)
    opt = HaAlg2Options(float(cap_scale), float(kappa), int(bool(vnorm_sampling)))
    _check(lib().hyperattn_forward_alg2(_dev(Q, "Q"), _dev(K, "K"), _dev(V, "V"), _dev(out, "out"), _dev(lse, "lse"),
                                        ctypes.byref(shape), ctypes.byref(params), ctypes.byref(opt),
                                        workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "hyperattn_forward_alg2")
    return out, lse, workspace


def alg2_workspace_views(workspace, shape: HaShape, params: HaParams):
    """Typed views of the option kernels' regions after hyperattn_forward_alg2: the per-node regions
    (nodes in heap order), and vnorm_w of the last level processed (the only level of an unmasked problem)."""
    torch = _torch()
    lay = ha_alg2_workspace_layout(shape, params)
    fwd = ha_workspace_layout(shape, params)
    BH, m, nodes = shape.B * shape.H, params.m, fwd.total_nodes

    def view(off, count, dtype, shp):
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        return workspace[off:off + nbytes].view(dtype).view(shp)

    return {"layout": lay,
            "tau_rows": view(lay.tau_rows, nodes * m, torch.int32, (nodes, m)),
            "log_tau": view(lay.log_tau, BH * nodes, torch.float32, (BH, nodes)),
            "vnorm_w": view(lay.vnorm_w, BH * fwd.n_cov, torch.float64, (BH, fwd.n_cov)),
            "vnorm_samples": view(lay.vnorm_samples, BH * nodes * m, torch.int32, (BH, nodes, m)),
            "vnorm_logw": view(lay.vnorm_logw, BH * nodes * m, torch.float32, (BH, nodes, m))}
