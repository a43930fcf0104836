"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before touching a GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2410_13344_amd import binding as B
from paper_2410_13344_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2410_13344_amd.build import build_library
        build_library()
    return B.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cerberus.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cerberus_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert {"cerberus_init", "cerberus_verify_step", "cerberus_ar_step", "cerberus_gate", "cerberus_accept"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def _cfg(**kw):
    return B.make_config(synth.make_config("tiny", **kw), B.CERBERUS_BF16, 1, 256)


def test_workspace_bytes_and_host_validation(L):
    parent, rank = synth.make_tree("tiny")
    tree, keep = B.make_tree(parent, rank)
    n = B.cerberus_workspace_bytes(_cfg(), tree)
    assert n > 0 and n % 256 == 0
    # bf16 mode carries a packed copy of every matrix; fp32 mode does not
    n32 = B.cerberus_workspace_bytes(B.make_config(synth.make_config("tiny"), B.CERBERUS_F32, 1, 256), tree)
    assert 0 < n32 < n
    # shapes the kernels do not support
    assert B.cerberus_workspace_bytes(_cfg(head_dim=48), tree) == 0
    assert b"head_dim" in L.cerberus_last_error()
    assert B.cerberus_workspace_bytes(_cfg(d_model=128), tree) == 0
    assert B.cerberus_workspace_bytes(_cfg(topk=1), tree) == 0          # rank 3 needs topk >= 4
    assert B.cerberus_workspace_bytes(_cfg(n_cerb_heads=3), tree) == 0  # tree depth 4 > 3 heads
    bad_parent = list(parent)
    bad_parent[5] = 9                                                  # parent after child
    t2, k2 = B.make_tree(bad_parent, rank)
    assert B.cerberus_workspace_bytes(_cfg(), t2) == 0
    deep, k3 = B.make_tree([-1] + list(range(64)), [0] * 65)
    assert B.cerberus_workspace_bytes(_cfg(), deep) == 0               # a chain deeper than the heads
    # a 4-ary tree in breadth-first order: 192 nodes are the most the library takes
    for n, ok in ((192, True), (193, False)):
        t4, k4 = B.make_tree([-1] + [(i - 1) // 4 for i in range(1, n)], [0] + [(i - 1) % 4 for i in range(1, n)])
        assert (B.cerberus_workspace_bytes(_cfg(), t4) > 0) == ok, n


def test_init_rejects_null_arguments_without_a_gpu(L):
    parent, rank = synth.make_tree("tiny")
    tree, keep = B.make_tree(parent, rank)
    cfg = _cfg()
    ctx = C.c_void_p()
    rc = L.cerberus_init(C.byref(ctx), C.byref(cfg), None, C.byref(tree), None, 0)
    assert rc == -1 and ctx.value is None
    assert L.cerberus_init(None, C.byref(cfg), None, C.byref(tree), None, 0) == -1
    assert L.cerberus_verify_step(None, None, 1, None) == -1
    assert L.cerberus_gate(None, None, 1, None, None, None) == -1
    assert L.cerberus_set_param(None, b"attn_mfma", 1) == -1


def test_binding_constants_match_the_header():
    text = open(os.path.join(ROOT, "include", "cerberus.h")).read()
    for name in ("CERBERUS_MAX_TREE", "CERBERUS_MAX_HEADS", "CERBERUS_MAX_TOPK", "CERBERUS_MAX_BATCH", "CERBERUS_F32",
                 "CERBERUS_BF16", "CERBERUS_DEV_KV_OVERFLOW", "CERBERUS_DEV_BAD_TOKEN", "CERBERUS_DEV_LOG_FULL"):
        m = re.search(r"\b" + name + r"\s*=\s*(-?\d+)", text)
        assert m, name
        assert getattr(B, name) == int(m.group(1)), name
