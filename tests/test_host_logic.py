"""Host-side checks that need no GPU: the library loads, exports what the header declares, and its
argument validation and KV bookkeeping behave as include/jupiter_stage.h says.  No kernel is launched:
device pointers are fake (never dereferenced by host logic)."""
import ctypes
import os
import re

import pytest

from paper_2504_08242_amd import binding as jb
from paper_2504_08242_amd import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x7000_0000_0000)  # 256-byte aligned, never touched


def declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            names += re.findall(r"JUP_API[^;(]*?\b(jup_[a-z0-9_]+)\s*\(", text)
    return names


def test_library_exports_every_declared_entry_point():
    names = declared_functions()
    assert "jup_stage_create" in names and "jup_stage_prefill_chunk" in names and "jup_kv_reset" in names
    L = jb.lib()
    for n in names:
        assert hasattr(L, n), n


def cfg_of(d, dtype):
    return jb.make_config(d, dtype)


def test_size_queries():
    L = jb.lib()
    c = cfg_of(si.LLAMA7B_STAGE, "bf16")
    per_layer = (4 * 4096 * 4096 + 3 * 4096 * 11008 + 2 * 4096) * 2
    assert L.jup_stage_packed_bytes(ctypes.byref(c)) >= 8 * per_layer
    assert L.jup_stage_packed_bytes(ctypes.byref(c)) < 8 * per_layer + (1 << 20)
    assert L.jup_kv_bytes(ctypes.byref(c), 2048) == 8 * 2 * 32 * 2048 * 128 * 2
    t = cfg_of(si.TINY, "f32")
    assert L.jup_kv_bytes(ctypes.byref(t), 128) == 2 * 2 * 4 * 128 * 64 * 4
    assert L.jup_stage_workspace_bytes(ctypes.byref(t), 0) == 0
    assert L.jup_stage_workspace_bytes(ctypes.byref(t), 128) > 128 * 256 * 4
    bad = cfg_of(dict(si.TINY, n_heads=3), "f32")
    assert L.jup_stage_packed_bytes(ctypes.byref(bad)) == 0 and L.jup_kv_bytes(ctypes.byref(bad), 8) == 0
    # 4-bit stage: half a byte per weight plus one fp32 scale per 128 weights; activations and cache stay bf16
    w = cfg_of(si.LLAMA7B_STAGE, "w4")
    n_weights = 4 * 4096 * 4096 + 3 * 4096 * 11008
    per_layer_w4 = n_weights // 2 + n_weights // 128 * 4 + 2 * 4096 * 2
    assert 8 * per_layer_w4 <= L.jup_stage_packed_bytes(ctypes.byref(w)) < 8 * per_layer_w4 + (1 << 20)
    assert L.jup_kv_bytes(ctypes.byref(w), 2048) == L.jup_kv_bytes(ctypes.byref(c), 2048)
    assert L.jup_stage_workspace_bytes(ctypes.byref(w), 64) == L.jup_stage_workspace_bytes(ctypes.byref(c), 64)
    # with the bf16 copy for long chunks: two more bytes per weight; the field belongs to 4-bit stages only
    x = jb.make_config(si.LLAMA7B_STAGE, "w4", w4_expanded=True)
    assert (8 * (per_layer_w4 + 2 * n_weights) <= L.jup_stage_packed_bytes(ctypes.byref(x))
            < 8 * (per_layer_w4 + 2 * n_weights) + (1 << 20))
    assert L.jup_stage_workspace_bytes(ctypes.byref(x), 512) == L.jup_stage_workspace_bytes(ctypes.byref(c), 512)
    x.w4_expanded = 2
    assert L.jup_stage_packed_bytes(ctypes.byref(x)) == 0
    c.w4_expanded = 1
    assert L.jup_stage_packed_bytes(ctypes.byref(c)) == 0
    c.w4_expanded = 0
    w.dtype = 3
    assert L.jup_stage_packed_bytes(ctypes.byref(w)) == 0


@pytest.mark.parametrize("change,dtype", [
    (dict(n_heads=3), "f32"), (dict(head_dim=63, d_model=252), "f32"), (dict(d_ffn=0), "f32"),
    (dict(rope_theta=0.0), "f32"), (dict(n_layers=-1), "f32"),
    (dict(), "bf16"),  # the tiny shape (head_dim 64) is not a matrix-core shape
    (dict(), "w4"),
])
def test_stage_create_rejects_bad_configurations_before_touching_the_device(change, dtype):
    L = jb.lib()
    c = cfg_of(dict(si.TINY, **change), dtype)
    layers = (jb.LayerWeights * 2)()
    out = ctypes.c_void_p()
    rc = L.jup_stage_create(ctypes.byref(c), layers, FAKE, 1 << 40, FAKE, 1 << 40, 32, None, ctypes.byref(out))
    assert rc == jb.JUP_EINVAL and not out.value and jb.last_error()


def test_stage_create_rejects_null_and_small_buffers():
    L = jb.lib()
    c = cfg_of(si.TINY, "f32")
    layers = (jb.LayerWeights * 2)()
    for l in layers:
        for n in jb.WEIGHT_NAMES:
            setattr(l, n, FAKE.value)
    out = ctypes.c_void_p()
    pb = L.jup_stage_packed_bytes(ctypes.byref(c))
    wb = L.jup_stage_workspace_bytes(ctypes.byref(c), 32)
    assert L.jup_stage_create(ctypes.byref(c), layers, FAKE, pb - 1, FAKE, wb, 32, None, ctypes.byref(out)) == jb.JUP_EINVAL
    assert "packed" in jb.last_error()
    assert L.jup_stage_create(ctypes.byref(c), layers, FAKE, pb, FAKE, wb - 1, 32, None, ctypes.byref(out)) == jb.JUP_EINVAL
    assert L.jup_stage_create(ctypes.byref(c), layers, None, pb, FAKE, wb, 32, None, ctypes.byref(out)) == jb.JUP_EINVAL
    assert L.jup_stage_create(ctypes.byref(c), layers, ctypes.c_void_p(FAKE.value + 8), pb, FAKE, wb, 32, None,
                              ctypes.byref(out)) == jb.JUP_EINVAL
    assert L.jup_stage_create(ctypes.byref(c), layers, FAKE, pb, FAKE, wb, 0, None, ctypes.byref(out)) == jb.JUP_EINVAL
    layers[1].w_up = None
    assert L.jup_stage_create(ctypes.byref(c), layers, FAKE, pb, FAKE, wb, 32, None, ctypes.byref(out)) == jb.JUP_EINVAL
    assert "layer 1" in jb.last_error()
    assert L.jup_stage_create(None, layers, FAKE, pb, FAKE, wb, 32, None, ctypes.byref(out)) == jb.JUP_EINVAL
    # bfloat16 dtypes: weight pointers must be 16-byte aligned (checked on the host, before any copy kernel)
    b = cfg_of(dict(si.LLAMA7B_STAGE, n_layers=1), "bf16")
    one = (jb.LayerWeights * 1)()
    for n in jb.WEIGHT_NAMES:
        setattr(one[0], n, FAKE.value)
    one[0].wk = FAKE.value + 8
    pb = L.jup_stage_packed_bytes(ctypes.byref(b))
    wb = L.jup_stage_workspace_bytes(ctypes.byref(b), 32)
    assert L.jup_stage_create(ctypes.byref(b), one, FAKE, pb, FAKE, wb, 32, None, ctypes.byref(out)) == jb.JUP_EINVAL
    assert "16-byte aligned" in jb.last_error() and not out.value


def make_kv(max_positions, dtype="f32", cfg=si.TINY):
    L = jb.lib()
    c = cfg_of(cfg, dtype)
    h = ctypes.c_void_p()
    rc = L.jup_kv_create(ctypes.byref(c), max_positions, FAKE, L.jup_kv_bytes(ctypes.byref(c), max_positions),
                         ctypes.byref(h))
    assert rc == jb.JUP_OK and h.value
    return h


def test_kv_create_validation():
    L = jb.lib()
    c = cfg_of(si.TINY, "f32")
    h = ctypes.c_void_p()
    nb = L.jup_kv_bytes(ctypes.byref(c), 64)
    assert L.jup_kv_create(ctypes.byref(c), 64, FAKE, nb - 1, ctypes.byref(h)) == jb.JUP_EINVAL
    assert L.jup_kv_create(ctypes.byref(c), 0, FAKE, nb, ctypes.byref(h)) == jb.JUP_EINVAL
    assert L.jup_kv_create(ctypes.byref(c), 64, None, nb, ctypes.byref(h)) == jb.JUP_EINVAL
    assert L.jup_kv_len(None) == -1 and L.jup_kv_capacity(None) == -1
    assert L.jup_kv_destroy(None) == jb.JUP_OK


def test_position_rules():
    """Holes, capacity, overwrite-from-here and the empty chunk (Sec. IV-A.2: s_i needs all of s_1..s_{i-1})."""
    L = jb.lib()
    kv = make_kv(100)
    assert L.jup_kv_len(kv) == 0 and L.jup_kv_capacity(kv) == 100
    assert L.jup_kv_check_append(kv, 32, 0) == jb.JUP_OK
    assert L.jup_kv_check_append(kv, 32, 1) == jb.JUP_EPOS        # hole
    assert "hole" in jb.last_error()
    assert L.jup_kv_check_append(kv, 101, 0) == jb.JUP_ECAP
    assert L.jup_kv_check_append(kv, 100, 0) == jb.JUP_OK          # exactly full
    assert L.jup_kv_check_append(kv, -1, 0) == jb.JUP_EINVAL
    assert L.jup_kv_check_append(kv, 1, -1) == jb.JUP_EINVAL
    assert L.jup_kv_check_append(kv, 0, 0) == jb.JUP_OK
    assert L.jup_kv_check_append(None, 1, 0) == jb.JUP_EINVAL
    assert L.jup_kv_truncate(kv, 1) == jb.JUP_EPOS                 # cannot grow by truncating
    assert L.jup_kv_truncate(kv, 0) == jb.JUP_OK
    assert L.jup_kv_reset(kv) == jb.JUP_OK
    assert L.jup_kv_destroy(kv) == jb.JUP_OK


def test_prefill_chunk_argument_errors_leave_the_cache_untouched():
    L = jb.lib()
    kv = make_kv(16)
    # no stage: rejected before anything else
    assert L.jup_stage_prefill_chunk(None, FAKE, 4, 0, kv, FAKE, None) == jb.JUP_EINVAL
    assert L.jup_kv_len(kv) == 0
    L.jup_kv_destroy(kv)


def test_prefill_branches_without_a_stage_is_rejected():
    L = jb.lib()
    kv = make_kv(16)
    pos = (ctypes.c_int32 * 1)(0)
    kvs = (ctypes.c_void_p * 1)(kv)
    assert L.jup_stage_prefill_branches(None, 1, FAKE, 4, pos, kvs, FAKE, None) == jb.JUP_EINVAL
    assert L.jup_kv_len(kv) == 0
    L.jup_kv_destroy(kv)


def test_tree_and_keep_argument_errors_need_no_device():
    """Everything jup_kv_keep() rejects is rejected on the host; an empty cache has nothing to keep."""
    L = jb.lib()
    kv = make_kv(16)
    par = (ctypes.c_int32 * 3)(-1, 0, 1)
    assert L.jup_stage_prefill_tree(None, FAKE, 3, 0, par, kv, FAKE, None) == jb.JUP_EINVAL
    assert L.jup_kv_keep(None, 0, 0, None, None) == jb.JUP_EINVAL
    one = (ctypes.c_int32 * 1)(0)
    assert L.jup_kv_keep(kv, 0, 1, one, None) == jb.JUP_EPOS       # entry 0 does not exist
    assert L.jup_kv_keep(kv, 1, 0, None, None) == jb.JUP_EPOS      # base behind the end
    assert L.jup_kv_keep(kv, 0, 65, one, None) == jb.JUP_EINVAL    # more than a tree holds
    assert L.jup_kv_keep(kv, 0, 1, None, None) == jb.JUP_EINVAL
    assert L.jup_kv_keep(kv, 0, 0, None, None) == jb.JUP_OK        # nothing kept, nothing moved, no launch
    assert L.jup_kv_len(kv) == 0
    L.jup_kv_destroy(kv)


def test_prefill_chunks_without_a_stage_is_rejected():
    L = jb.lib()
    kv = make_kv(16)
    n = (ctypes.c_int32 * 2)(4, 4)
    assert L.jup_stage_prefill_chunks(None, FAKE, 2, n, 0, kv, FAKE, None) == jb.JUP_EINVAL
    assert L.jup_stage_enable_overlap(None, 2, FAKE, 1 << 20) == jb.JUP_EINVAL
    assert L.jup_kv_len(kv) == 0
    L.jup_kv_destroy(kv)


def test_fork_rules():
    """Outline branches share the prompt's cache read-only (Sec. V-B)."""
    L = jb.lib()
    parent = make_kv(64)
    child = ctypes.c_void_p()
    # nothing cached yet: cannot share 8 positions
    assert L.jup_kv_fork(parent, 8, 32, FAKE, 1 << 30, ctypes.byref(child)) == jb.JUP_EPOS
    assert L.jup_kv_fork(parent, 0, 32, FAKE, 1 << 30, ctypes.byref(child)) == jb.JUP_OK
    assert L.jup_kv_len(child) == 0 and L.jup_kv_capacity(child) == 32
    # a fork of a fork is refused
    grand = ctypes.c_void_p()
    assert L.jup_kv_fork(child, 0, 8, FAKE, 1 << 30, ctypes.byref(grand)) == jb.JUP_EINVAL
    # the parent cannot be destroyed while the fork lives
    assert L.jup_kv_destroy(parent) == jb.JUP_EINVAL
    assert L.jup_kv_destroy(child) == jb.JUP_OK
    assert L.jup_kv_destroy(parent) == jb.JUP_OK
    c = cfg_of(si.TINY, "f32")
    p2 = make_kv(64)
    assert L.jup_kv_fork_bytes(p2, 0, 24) == L.jup_kv_bytes(ctypes.byref(c), 24)
    assert L.jup_kv_fork_bytes(p2, 8, 8) == 0
    assert L.jup_kv_fork(p2, 0, 24, FAKE, L.jup_kv_fork_bytes(p2, 0, 24) - 1, ctypes.byref(child)) == jb.JUP_EINVAL
    assert L.jup_kv_destroy(p2) == jb.JUP_OK


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(jb, "_lib", None)
    monkeypatch.setattr(jb, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        jb.lib()
