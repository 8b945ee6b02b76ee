"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes workspaces, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import workloads as W
from paper_2404_16710_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_functions():
    src = open(os.path.join(ROOT, "include", "ls.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ls_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _header_functions()
    assert set(names) >= {"ls_load_weights", "ls_prefill", "ls_draft", "ls_verify", "ls_generate"}
    for n in names:
        assert hasattr(lib, n), n
    assert set(B.EXPORTS) == set(names)


def test_workspace_sizes_follow_the_configuration():
    lib = B.lib()
    for name in ("c1", "c2", "c3", "c4", "c5"):
        w = W.get_workload(name)
        m = w.model
        max_seq = w.n_prompt + w.n_new + 17
        cfg = B.config_struct(m, max_seq)
        n = lib.ls_workspace_bytes(C.byref(cfg))
        kv = 2 * m.n_layers * m.kv_dim * max_seq * m.elem_bytes
        rows = min(max_seq, 2048)                       # prompt rows the GEMM prefill keeps at once
        pf = rows * (4 * m.d_model + m.elem_bytes * (m.d_model + 2 * m.q_dim + m.ffn_dim))
        assert kv + pf < n < kv + pf + (64 << 20), (name, n, kv, pf)


@pytest.mark.parametrize("field,value", [("head_dim", 96), ("n_kv_heads", 3), ("d_model", 250), ("vocab", 1001),
                                         ("max_draft", 16), ("max_draft", 0), ("dtype", 7), ("max_seq", 1),
                                         ("max_seq", 1 << 20), ("n_layers", 0), ("rms_eps", 0.0)])
def test_invalid_configurations_are_rejected(field, value):
    lib = B.lib()
    cfg = B.config_struct(W.get_workload("c1").model, 128)
    setattr(cfg, field, value)
    assert lib.ls_workspace_bytes(C.byref(cfg)) == 0
    ctx = C.c_void_p()
    w = B.ls_weights()
    assert lib.ls_load_weights(C.byref(cfg), C.byref(w), C.c_void_p(256), 1 << 30, C.byref(ctx)) == -1
    assert not ctx.value


def test_null_and_misaligned_arguments_are_rejected_without_a_gpu():
    lib = B.lib()
    cfg = B.config_struct(W.get_workload("c1").model, 128)
    ctx = C.c_void_p()
    w = B.ls_weights()                                      # all pointers null
    assert lib.ls_load_weights(C.byref(cfg), C.byref(w), C.c_void_p(256), 1 << 30, C.byref(ctx)) == -1
    assert lib.ls_load_weights(C.byref(cfg), None, C.c_void_p(256), 1 << 30, C.byref(ctx)) == -1
    assert lib.ls_load_weights(C.byref(cfg), C.byref(w), None, 1 << 30, C.byref(ctx)) == -1
    assert lib.ls_load_weights(C.byref(cfg), C.byref(w), C.c_void_p(257), 1 << 30, C.byref(ctx)) == -1
    for fn, args in (("ls_prefill", (None, None, 4, None)), ("ls_draft", (None, 1, 1, None)),
                     ("ls_verify", (None, 1, 1, None)), ("ls_get_state", (None, None, None, None, None)),
                     ("ls_debug_capture", (None, None)), ("ls_set_launch", (None, 1)),
                     ("ls_set_prompt_tiles", (None, 64)), ("ls_debug_spin_limit", (None, 1)),
                     ("ls_debug_kv_policy", (None, 1))):
        assert getattr(lib, fn)(*args) == -1, fn
    # the read-only stream reference: null or misaligned pointers, no workgroups, a size that does not split evenly
    for args in ((None, 1 << 24, C.c_void_p(256), 256, None), (C.c_void_p(256), 1 << 24, None, 256, None),
                 (C.c_void_p(264), 1 << 24, C.c_void_p(256), 256, None), (C.c_void_p(256), 1 << 24, C.c_void_p(256), 0, None),
                 (C.c_void_p(256), (1 << 24) + 16, C.c_void_p(256), 256, None), (C.c_void_p(256), 0, C.c_void_p(256), 256, None)):
        assert lib.ls_debug_read(*args) == -1, args
    assert b"capacity" in lib.ls_strerror(-3) and b"ok" == lib.ls_strerror(0)
    lib.ls_destroy(None)                                     # harmless


def test_static_workspace_variant_rejects_what_does_not_fit_before_touching_the_device():
    lib = B.lib()
    limit = lib.ls_static_workspace_limit()
    assert limit == 8 << 20
    w = B.ls_weights()
    st = B.ls_stats()
    small = B.config_struct(W.get_workload("c1").model, 113)
    assert 0 < lib.ls_workspace_bytes(C.byref(small)) <= limit
    big = B.config_struct(W.get_workload("c2").model, 785)
    assert lib.ls_workspace_bytes(C.byref(big)) > limit
    args = (None, 4, 4, 1, 1, -1, None, C.byref(st), None)
    assert lib.ls_generate_static(C.byref(big), C.byref(w), *args) == -3      # LS_E_CAPACITY
    bad = B.config_struct(W.get_workload("c1").model, 113)
    bad.head_dim = 96
    assert lib.ls_generate_static(C.byref(bad), C.byref(w), *args) == -1      # LS_E_ARG
    assert lib.ls_generate_static(None, C.byref(w), *args) == -1


def test_binding_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    w = W.get_workload("c1")
    with pytest.raises(RuntimeError):
        B.LsModel(w.model, W.make_weights(w), max_seq=128)
