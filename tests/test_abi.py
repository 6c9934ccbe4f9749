"""Host-only checks of the C ABI: the library loads, exports every declared
symbol, and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

from helpers import tiny_cfg


@pytest.fixture(scope="module")
def B():
    from paper_2406_02657_amd import binding
    return binding


def test_exports_every_declared_symbol(B, repo_root):
    hdr = open(os.path.join(repo_root, "include", "bt.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(bt_[a-z_]+)\s*\(", hdr))
    assert {"bt_create", "bt_prefill", "bt_decode_step", "bt_workspace_bytes", "bt_get_logits"} <= names
    for n in names:
        assert hasattr(B.lib, n), n


def _cfg(B, **kw):
    cfg = tiny_cfg(d_model=64, n_heads=2, d_ff=128, **kw)
    return B.make_config(cfg, max_batch=2, max_blocks=8)


def test_workspace_bytes_and_bad_configs(B):
    n = C.c_size_t(0)
    assert B.lib.bt_workspace_bytes(C.byref(_cfg(B)), C.byref(n)) == 0 and n.value > 0
    assert B.lib.bt_workspace_bytes(None, C.byref(n)) == B.BT_ERR_ARG
    bad = []
    c = _cfg(B); c.n_heads = 3; bad.append(c)              # D % H
    c = _cfg(B); c.n_heads = 8; bad.append(c)              # d_head = 8 unsupported
    c = _cfg(B); c.block_len = 3; bad.append(c)            # D % L_B
    c = _cfg(B); c.rotary_dims = 3; bad.append(c)          # odd rotary
    c = _cfg(B); c.rotary_dims = 64; bad.append(c)         # > d_head
    c = _cfg(B); c.prefix_len = 0; bad.append(c)           # P = 0 needs L_B = 1
    c = _cfg(B); c.dtype = 7; bad.append(c)
    c = _cfg(B); c.max_batch = 0; bad.append(c)
    c = _cfg(B); c.max_blocks = 0; bad.append(c)
    c = _cfg(B); c.dtype = B.BT_BF16; c.d_ff = 72; bad.append(c)
    for c in bad:
        assert B.lib.bt_workspace_bytes(C.byref(c), C.byref(n)) == B.BT_ERR_ARG
    c = _cfg(B); c.block_len = 1; c.prefix_len = 0
    assert B.lib.bt_workspace_bytes(C.byref(c), C.byref(n)) == 0


def test_workspace_grows_with_capacity(B):
    n1, n2 = C.c_size_t(0), C.c_size_t(0)
    c = _cfg(B)
    B.lib.bt_workspace_bytes(C.byref(c), C.byref(n1))
    c.max_blocks = 64
    B.lib.bt_workspace_bytes(C.byref(c), C.byref(n2))
    assert n2.value > n1.value


def test_create_rejects_null_and_small_workspace(B):
    c = _cfg(B)
    w = B.bt_weights()
    h = C.c_void_p()
    assert B.lib.bt_create(C.byref(c), C.byref(w), 4096, 1 << 30, None, C.byref(h)) == B.BT_ERR_ARG   # null weights
    assert B.lib.bt_create(C.byref(c), C.byref(w), None, 1 << 30, None, C.byref(h)) == B.BT_ERR_ARG   # null workspace
    assert B.lib.bt_create(C.byref(c), C.byref(w), 4097, 1 << 30, None, C.byref(h)) == B.BT_ERR_ARG   # misaligned
    assert h.value is None
    # null model handles
    assert B.lib.bt_prefill(None, None, 1, 4) == B.BT_ERR_ARG
    assert B.lib.bt_decode_step(None, 1, None) == B.BT_ERR_ARG
    assert b"aligned" in B.lib.bt_last_error(None)          # the reason of this thread's last failed create
    c.struct_size = 12
    assert B.lib.bt_create(C.byref(c), C.byref(w), 4096, 1 << 30, None, C.byref(h)) == B.BT_ERR_ARG
    assert b"struct_size" in B.lib.bt_last_error(None)
    c = _cfg(B)
    big = _cfg(B); big.max_batch = 4096; big.max_blocks = 4096
    assert B.lib.bt_create_static(C.byref(big), C.byref(w), None, C.byref(h)) == B.BT_ERR_CAPACITY
    assert b"BT_STATIC_WORKSPACE_BYTES" in B.lib.bt_last_error(None) and h.value is None
    B.lib.bt_destroy(None)


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message before touching any GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
