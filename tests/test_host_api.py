"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, rejects bad arguments before touching the
device, lays out the workspace as documented, and its random draws are
bit-identical to the oracle's independently written generator."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import hyperattn_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ha():
    import paper_2310_05869_amd as mod
    if not os.path.exists(mod.binding.LIB_PATH):
        from paper_2310_05869_amd import build
        build.build_library()
    mod.lib()
    return mod


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hyperattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ha_\w+|hyperattn_\w+|exact_attn_\w+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound(ha):
    declared = _declared_functions()
    assert "hyperattn_forward" in declared and "ha_lsh_hash" in declared
    handle = ctypes.CDLL(ha.binding.LIB_PATH)
    for name in declared:
        assert hasattr(handle, name), f"{name} declared in hyperattn.h but not exported"
    assert sorted(ha.exported_symbols()) == declared


def test_struct_layouts_match_header(ha):
    assert ctypes.sizeof(ha.HaShape) == 20
    assert ctypes.sizeof(ha.HaParams) == 32 and ha.HaParams.seed.offset == 24


@pytest.mark.parametrize("seed,d,r", [(0, 128, 7), (0, 64, 7), (12345, 128, 8), (2 ** 63 + 5, 64, 1)])
def test_projection_bit_identical_to_oracle(ha, seed, d, r):
    R = ha.ha_make_projection(seed, d, r)
    np.testing.assert_array_equal(R.astype(np.float64), orc.make_projection(seed, d, r))


@pytest.mark.parametrize("seed,level,node,n_keys,m", [(0, 0, 0, 32768, 256), (0, 4, 15, 4096, 256), (7, 2, 3, 1000, 33),
                                                      (1, 0, 0, 1, 5), (3, 1, 0, 2 ** 24, 512)])
def test_samples_bit_identical_to_oracle(ha, seed, level, node, n_keys, m):
    np.testing.assert_array_equal(ha.ha_make_samples(seed, level, node, n_keys, m),
                                  orc.make_samples(seed, level, node, n_keys, m))


def test_workspace_layout(ha):
    sh = ha.make_shape(1, 32, 131072, 128, ha.HA_BF16)
    p = ha.make_params(256, 256, 7, True, 4096, 0)
    lay = ha.ha_workspace_layout(sh, p)
    assert (lay.levels, lay.total_nodes, lay.n_cov) == (5, 31, 65536)
    offs = [lay.codes_q, lay.codes_k, lay.perm_q, lay.perm_k, lay.pos_k, lay.samples, lay.proj, lay.part_o,
            lay.part_l, lay.total_bytes]
    assert all(o % 256 == 0 for o in offs) and offs == sorted(offs)
    assert lay.part_l - lay.part_o == 5 * 32 * 65536 * 128 * 2     # bf16 tensors: bf16 partial outputs
    assert ha.ha_workspace_bytes(sh, p) == lay.total_bytes
    # unmasked: one level covering all n rows, no partial buffers
    p2 = ha.make_params(256, 256, 7, False, 4096, 0)
    lay2 = ha.ha_workspace_layout(ha.make_shape(1, 32, 32768, 128, ha.HA_BF16), p2)
    assert (lay2.levels, lay2.total_nodes, lay2.n_cov) == (1, 1, 32768)
    assert lay2.part_l == lay2.part_o
    # causal with n <= n_min: exact attention only
    lay3 = ha.ha_workspace_layout(ha.make_shape(1, 2, 1024, 64, ha.HA_BF16), p)
    assert lay3.levels == 0 and lay3.total_nodes == 0


def test_backward_workspace_layout(ha):
    """The backward keeps one accumulated fp32 row per tensor row and pass (two buffers, the first one used by dQ
    and then by dK), delta, and the sampled keys' rows per query chunk: not one buffer per level."""
    sh = ha.make_shape(1, 32, 131072, 128, ha.HA_BF16)
    p = ha.make_params(256, 256, 7, True, 4096, 0)
    lay = ha.binding.HaBwdWsLayout()
    assert ha.lib().ha_backward_workspace_layout(ctypes.byref(sh), ctypes.byref(p), ctypes.byref(lay)) == 0
    rows = 32 * 131072
    assert lay.acc_a - lay.delta == rows * 4 and lay.acc_b - lay.acc_a == rows * 128 * 4
    assert lay.samp_k - lay.acc_b == rows * 128 * 4
    # per level: 32 heads x 2^l nodes x ceil(s / 2048) chunks x 256 samples, s = n >> (l + 1): 32 chunks per head and level
    samp_rows = 5 * 32 * 32 * 256
    assert lay.samp_v - lay.samp_k == samp_rows * 128 * 4 and lay.total_bytes - lay.samp_v == samp_rows * 128 * 4
    assert lay.total_bytes == ha.ha_backward_workspace_bytes(sh, p) < 6 * 2 ** 30
    # fp32 tensors have a backward pass too, with the same buffers
    assert ha.ha_backward_workspace_bytes(ha.make_shape(1, 32, 131072, 128, ha.HA_FP32), p) == lay.total_bytes
    # exact attention (the recursion that never splits): delta only
    p0 = ha.make_params(1, 0, 1, True, 131072, 0)
    assert ha.ha_backward_workspace_bytes(sh, p0) == rows * 4


def test_forward_workgroup_counts(ha):
    """Records of the stamped forward: one per 128-query tile of every node (levels x half the rows when causal)
    and of the base case; none for fp32 tensors, which run the kernel without matrix cores."""
    p = ha.make_params(256, 256, 7, True, 4096, 0)
    assert ha.ha_forward_workgroups(ha.make_shape(1, 32, 131072, 128, ha.HA_BF16), p) == (5 * 32 * 65536 // 128, 32 * 131072 // 128)
    assert ha.ha_forward_workgroups(ha.make_shape(1, 32, 131072, 128, ha.HA_FP32), p) == (0, 0)
    pu = ha.make_params(256, 256, 7, False, 4096, 0)
    assert ha.ha_forward_workgroups(ha.make_shape(2, 4, 32768, 64, ha.HA_BF16), pu) == (8 * 32768 // 128, 0)
    assert ha.ha_forward_workgroups(ha.make_shape(1, 0, 32768, 64, ha.HA_BF16), pu) == (0, 0)
    nw, bw = ctypes.c_int64(0), ctypes.c_int64(0)
    bad = ha.make_shape(1, 1, 1000, 64, ha.HA_BF16)
    assert ha.lib().ha_forward_workgroups(ctypes.byref(bad), ctypes.byref(pu), ctypes.byref(nw), ctypes.byref(bw)) == -3
    assert ha.lib().ha_forward_workgroups(ctypes.byref(bad), ctypes.byref(pu), None, ctypes.byref(bw)) != 0


@pytest.mark.parametrize("shape,params,status", [
    ((1, 1, 1024, 96, 0), (64, 64, 7, 0, 4096, 0), -3),     # d not 64/128
    ((1, 1, 1000, 64, 0), (64, 64, 7, 0, 4096, 0), -3),     # n % b
    ((1, 1, 1024, 64, 0), (64, 64, 9, 0, 4096, 0), -3),     # r > 8
    ((1, 1, 1024, 64, 0), (64, 64, 0, 0, 4096, 0), -3),     # r < 1
    ((1, 1, 1024, 64, 0), (64, 5000, 7, 0, 4096, 0), -3),   # m too large
    ((1, 1, 1024, 64, 0), (0, 64, 7, 0, 4096, 0), -3),      # b < 1
    ((1, 1, 3072, 64, 0), (64, 64, 7, 1, 1024, 0), -3),     # n / n_min not a power of two
    ((1, 1, 2048, 64, 0), (96, 64, 7, 1, 1024, 0), -3),     # n_min % b
    ((1, 1, 2048, 64, 0), (64, 64, 7, 1, 0, 0), -3),        # n_min < 1
    ((1, 1, 1024, 64, 2), (64, 64, 7, 0, 4096, 0), -2),     # dtype
])
def test_bad_arguments_are_rejected_on_the_host(ha, shape, params, status):
    sh = ha.make_shape(*shape)
    p = ha.make_params(*params)
    lay = ha.HaWsLayout()
    assert ha.lib().ha_workspace_layout(ctypes.byref(sh), ctypes.byref(p), ctypes.byref(lay)) == status
    assert ha.ha_workspace_bytes(sh, p) == 0
    # the forward call reports the same error before any pointer is used
    assert ha.lib().hyperattn_forward(None, None, None, None, None, ctypes.byref(sh), ctypes.byref(p), None, 0,
                                      None) == status


def test_null_pointers_and_strerror(ha):
    sh = ha.make_shape(1, 1, 1024, 64, 0)
    p = ha.make_params(64, 64, 7)
    assert ha.lib().hyperattn_forward(None, None, None, None, None, ctypes.byref(sh), ctypes.byref(p), None, 0,
                                      None) == -1
    assert ha.lib().hyperattn_forward(None, None, None, None, None, None, None, None, 0, None) == -1
    assert ha.lib().exact_attn_forward(None, None, None, None, None, ctypes.byref(sh), 0, None) == -1
    assert ha.lib().ha_make_projection(0, 64, 7, None) == -1
    assert ha.lib().ha_lsh_hash(None, None, 10, 64, 0, None, 7, None) == -1
    assert ha.lib().ha_lsh_hash(None, None, 10, 65, 0, None, 7, None) == -3
    assert ha.lib().ha_seg_sort(None, None, None, 1, 2 ** 25, None) == -3
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert ha.strerror(code) and ha.strerror(code) != "unknown status"
    assert ha.strerror(-99) == "unknown status"


def test_misaligned_arrays_are_rejected_on_the_host(ha):
    """Tensors must start at a 16-byte boundary, float / index arrays at a 4-byte one; the check
    runs on the host before anything is enqueued (the addresses here are never dereferenced)."""
    sh = ha.make_shape(1, 1, 1024, 64, 0)
    p = ha.make_params(64, 64, 7)
    ok = 0x7F0000000000
    fwd = ha.lib().hyperattn_forward
    assert fwd(ok + 8, ok, ok, ok, ok, ctypes.byref(sh), ctypes.byref(p), ok, 1 << 30, None) == -6
    assert fwd(ok, ok, ok + 2, ok, ok, ctypes.byref(sh), ctypes.byref(p), ok, 1 << 30, None) == -6
    assert fwd(ok, ok, ok, ok, ok + 2, ctypes.byref(sh), ctypes.byref(p), ok, 1 << 30, None) == -6
    assert ha.lib().exact_attn_forward(ok, ok + 4, ok, ok, ok, ctypes.byref(sh), 0, None) == -6
    assert ha.lib().ha_lsh_hash(ok + 4, ok, 10, 64, 0, ok, 7, None) == -6
    assert ha.lib().ha_seg_sort(ok, ok + 1, ok, 1, 16, None) == -6
    assert "aligned" in ha.strerror(-6)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2310_05869_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), (dirpath, f)
