"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/ll.h declares, sizes workspaces, and turns bad calls into
error codes before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2604_23467_amd import binding as b
from paper_2604_23467_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ll.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ll_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = b.load()
    names = declared_functions()
    assert len(names) >= 12 and "ll_init" in names and "ll_decode_step" in names
    for n in names:
        assert hasattr(lib, n), "libll.so does not export %s" % n
    assert sorted(b.EXPORTS) == names, "binding.EXPORTS out of step with include/ll.h"


def test_workspace_bytes_is_pure_and_monotone():
    tiny = b.ll_workspace_bytes(wl.tiny_cfg(max_seq=64))
    tiny2 = b.ll_workspace_bytes(wl.tiny_cfg(max_seq=128))
    big = b.ll_workspace_bytes(wl.llama7b_cfg())
    assert 0 < tiny < tiny2 < big
    assert tiny % 256 == 0 and big % 256 == 0
    # the 7B KV cache alone: 32 layers x 2 x 32 heads x 1024 x 128 fp16
    assert big > 32 * 2 * 32 * 1024 * 128 * 2


@pytest.mark.parametrize("patch", [
    dict(head_dim=32, n_heads=8), dict(head_dim=64, n_heads=3), dict(ffn_hidden=100),
    dict(max_seq=1), dict(vocab=0), dict(n_layers=0), dict(rope_theta=0.0), dict(rms_eps=-1.0),
])
def test_bad_configs_are_rejected(patch):
    cfg = wl.tiny_cfg()
    cfg.update(patch)
    assert b.ll_workspace_bytes(cfg) == 0
    lib = b.load()
    c = b.make_config(cfg)
    w = b.LLWeights()
    assert lib.ll_init(C.byref(c), C.byref(w), None, 0, None) == b.LL_E_BAD_CONFIG
    assert b.ll_last_error() != ""


def test_calls_before_init_fail_cleanly():
    lib = b.load()
    assert lib.ll_decode_step() == b.LL_E_NOT_INIT
    assert lib.ll_decode_n(3, None) == b.LL_E_NOT_INIT
    toks = (C.c_int32 * 2)(1, 2)
    assert lib.ll_prefill(toks, 2) == b.LL_E_NOT_INIT
    assert lib.ll_reset() == b.LL_E_NOT_INIT
    assert lib.ll_shutdown() == b.LL_E_NOT_INIT
    assert lib.ll_max_prompt() == b.LL_E_NOT_INIT
    assert lib.ll_position() == b.LL_E_NOT_INIT
    assert lib.ll_dbg_force_next_token(0) == b.LL_E_NOT_INIT
    assert "not initialised" in b.ll_last_error()


def test_init_rejects_null_arguments_before_touching_the_device():
    lib = b.load()
    c = b.make_config(wl.tiny_cfg())
    assert lib.ll_init(C.byref(c), None, None, 0, None) == b.LL_E_BAD_ARG
    w = b.LLWeights()                       # all pointers null
    assert lib.ll_init(C.byref(c), C.byref(w), None, 0, None) == b.LL_E_BAD_ARG
    assert lib.ll_init(None, C.byref(w), None, 0, None) == b.LL_E_BAD_CONFIG


def test_binding_has_no_oracle_dependency():
    """The product path must not route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2604_23467_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
                assert "liboracle" not in src, f


def test_batch_calls_need_an_instance():
    """No ll_init, no GPU: every batched-decoding call reports LL_E_NOT_INIT (the size query: 0)."""
    import ctypes as C
    from paper_2604_23467_amd import binding as b
    lib = b.load()
    assert lib.ll_batch_pool_bytes(16, 8) == 0
    out = (C.c_int32 * 16)()
    first = C.c_int32(0)
    ms = C.c_float(0)
    logits = (C.c_float * 4)()
    for rc in (lib.ll_batch_open(4, 16, 8, C.c_void_p(256), 1 << 20), lib.ll_batch_add(out, 1, C.byref(first)),
               lib.ll_batch_step(out), lib.ll_batch_remove(0), lib.ll_batch_close(),
               lib.ll_batch_dbg_get_logits(0, logits), lib.ll_batch_dbg_force_next_token(0, 0),
               lib.ll_batch_dbg_time_steps(1, C.byref(ms))):
        assert rc == b.LL_E_NOT_INIT
