"""ll_prefill_static (the prefill whose kernels keep their scratch in the library's static device
array) against ll_prefill, through the C ABI: two calls in a row, the second with a smaller input.
Needs a real MI355X: run with ``-m gpu``."""
import numpy as np
import pytest

from paper_2604_23467_amd import workloads as wl
from parity_utils import check_greedy_token, check_kv, check_logits, check_token

pytestmark = pytest.mark.gpu


def _snapshot(s, n):
    return dict(logits=s.ll_dbg_get_logits(), hidden=s.ll_dbg_get_hidden(),
                kv=[s.ll_dbg_get_kv(layer, which, n) for layer in range(s.cfg["n_layers"]) for which in range(2)])


def test_static_scratch_prefill_matches_ll_prefill(oracle32):
    import torch
    from paper_2604_23467_amd import binding
    assert torch.cuda.is_available(), "this test needs a GPU"
    cfg = wl.custom_cfg(2, 2, 128, 344, 300, 100)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=31, gain_jitter=0.1), np.float16)
    w_t = wl.weights_to_torch(w, device="cuda:0", dtype=torch.float16)
    prompts = [wl.make_tokens(n, cfg["vocab"], seed=700 + n) for n in (27, 9)]     # 32-row, then 16-row kernels
    with binding.Session(cfg, w_t) as s:
        want = []
        for p in prompts:                       # the existing entry point first
            s.ll_reset()
            t1 = s.ll_prefill(p)
            snap = _snapshot(s, len(p))
            want.append((t1, snap, s.ll_decode_n(3).tolist(), s.ll_dbg_get_logits()))
        for p, (t1, snap, toks, last_logits) in zip(prompts, want):     # two calls in a row, the second smaller
            s.ll_reset()
            got_t1 = s.ll_prefill_static(p)
            got = _snapshot(s, len(p))
            assert got_t1 == t1 and s.ll_position() == len(p)
            # same kernels on the same inputs, fixed summation order: the same bits
            assert np.array_equal(got["logits"], snap["logits"]) and np.array_equal(got["hidden"], snap["hidden"])
            for a, b in zip(got["kv"], snap["kv"]):
                assert np.array_equal(a, b)
            check_greedy_token(got_t1, got["logits"], "static prefill(%d)" % len(p))
            # and against the oracle, to the parity bar
            om = oracle32.model(cfg, w)
            t_ref, l_ref, h_ref = om.prefill(p)
            check_logits(got["logits"], l_ref, "static prefill(%d) logits" % len(p))
            check_token(got_t1, t_ref, l_ref, "static prefill(%d)" % len(p))
            for layer in range(cfg["n_layers"]):
                for which in range(2):
                    check_kv(got["kv"][2 * layer + which], om.kv(layer, which), "static prefill(%d) layer %d" % (len(p), layer))
            om.close()
            # decoding continues from the context it left
            assert s.ll_decode_n(3).tolist() == toks and np.array_equal(s.ll_dbg_get_logits(), last_logits)
        # limits: a clear error and an untouched context
        s.ll_reset()
        with pytest.raises(binding.LLError) as e:
            s.ll_prefill_static(wl.make_tokens(33, cfg["vocab"], seed=1))
        assert e.value.code == binding.LL_E_CAPACITY and "32" in str(e.value)
        assert s.ll_position() == 0
        s.ll_prefill_static(prompts[1])
        with pytest.raises(binding.LLError) as e:
            s.ll_prefill_static(prompts[1])               # non-empty context, as ll_prefill
        assert e.value.code == binding.LL_E_STATE


def test_static_scratch_prefill_rejects_a_model_that_does_not_fit():
    """A vocabulary whose logits alone exceed the 4 MiB array."""
    import torch
    from paper_2604_23467_amd import binding
    cfg = wl.custom_cfg(1, 2, 64, 136, 1100000, 16)
    w_t = wl.make_weights_torch(cfg, seed=2, device="cuda:0")
    with binding.Session(cfg, w_t) as s:
        p = wl.make_tokens(5, cfg["vocab"], seed=5)
        with pytest.raises(binding.LLError) as e:
            s.ll_prefill_static(p)
        assert e.value.code == binding.LL_E_CAPACITY and "scratch" in str(e.value)
        assert s.ll_position() == 0 and s.ll_prefill(p) >= 0      # the workspace path still serves it
