"""GPU parity of in-graph stochastic sampling: the HIP sampler against the CPU
oracle (oracle/sampling.py) on the SAME logits (the GPU's own, read back through
the debug hook), so that only the sampler is compared.

Where floating point decides the token (a running sum against a target), the GPU
sums in fp32 in another order than the fp64 oracle.  A GPU token is accepted when
it is the oracle's, or when the oracle's interval of the running sum for that
token, widened by 1e-5 of the total (and the nucleus mass target moved by the
same relative amount), contains the target; at least 95 % must match exactly."""
import numpy as np
import pytest

from oracle import sampling as sp
from paper_2604_23467_amd import workloads as wl

pytestmark = pytest.mark.gpu
REL = 1e-5


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def _session(cfg, w_np, flags=0):
    from paper_2604_23467_amd import binding
    return binding.Session(cfg, wl.weights_to_torch(wl.weights_astype(w_np, np.float16), "cuda:0"), flags=flags)


def _accept(tok, logits, temperature, top_k, top_p, u):
    ref, _ = sp.sample(logits, temperature, top_k, top_p, u)
    if tok == ref:
        return True, True
    for p in (top_p, max(top_p * (1 - REL), 1e-12), min(top_p * (1 + REL), 1.0)):
        _, info = sp.sample(logits, temperature, top_k, p, u)
        where = np.flatnonzero(info["idx"] == tok)
        if where.size == 0:
            continue
        r = int(where[0])
        lo = info["csum"][r - 1] if r > 0 else 0.0
        hi = info["csum"][r]
        eps = REL * info["total"]
        if lo - eps <= info["target"] <= hi + eps:
            return True, False
    return False, False


def _run(sess, prompt, steps, temperature, top_k, top_p, seed):
    sess.ll_reset()
    sess.ll_set_sampling(temperature, top_k, top_p, seed)
    toks, exact = [], 0
    for i in range(steps + 1):
        tok = sess.ll_prefill(prompt) if i == 0 else sess.ll_decode_step()
        logits = sess.ll_dbg_get_logits()
        ok, same = _accept(tok, logits, temperature, top_k, top_p, sp.uniform(seed, i))
        assert ok, "draw %d: token %d not a valid draw (T=%g k=%d p=%g)" % (i, tok, temperature, top_k, top_p)
        exact += same
        toks.append(tok)
    return toks, exact


SETTINGS = [(1.0, 0, 1.0), (0.7, 40, 1.0), (1.3, 0, 0.9), (0.8, 50, 0.95), (2.0, 5, 0.5), (1.0, 1000, 0.3)]


@pytest.mark.parametrize("vocab", [1024, 5001, 32000])
def test_sampler_matches_oracle_on_the_gpu_logits(torch_cuda, vocab):
    cfg = wl.custom_cfg(1, 2, 64, 136, vocab, 80)
    w = wl.make_weights_numpy(cfg, seed=51, emb_std=1.0)
    w["lm_head"] = (w["lm_head"] * 30.0).astype(w["lm_head"].dtype)     # logits a few units wide
    w = wl.weights_astype(w, np.float16)
    prompt = wl.make_tokens(6, vocab, seed=3)
    total = exact = 0
    with _session(cfg, w) as s:
        for j, (t, k, p) in enumerate(SETTINGS):
            toks, ex = _run(s, prompt, 40, t, k, p, seed=1000 + j)
            assert len(set(toks)) > 3                                      # it does sample
            total += len(toks)
            exact += ex
    assert exact >= 0.95 * total, (exact, total)


def test_equal_logits_exercise_the_tie_rules(torch_cuda):
    """A zero LM head makes every logit equal: top-k keeps the k lowest ids and the draw is
    uniform over them in index order, token = floor(u * k), exactly."""
    cfg = wl.custom_cfg(1, 2, 64, 136, 3000, 40)
    w = wl.make_weights_numpy(cfg, seed=52)
    w["lm_head"][:] = 0
    with _session(cfg, wl.weights_astype(w, np.float16)) as s:
        for k in (7, 64, 2999):
            s.ll_reset()
            s.ll_set_sampling(1.0, k, 1.0, 99)
            toks = [s.ll_prefill([1, 2, 3])] + [s.ll_decode_step() for _ in range(20)]
            want = [int(np.floor(np.float32(sp.uniform(99, i)) * np.float32(k))) for i in range(21)]
            assert all(0 <= t < k for t in toks)
            assert sum(a == b for a, b in zip(toks, want)) >= 20, (toks, want)   # fp32 running sums of ones are exact below 2^24
        # top-p on equal logits: ceil(p * V) lowest ids survive
        s.ll_reset()
        s.ll_set_sampling(1.0, 0, 0.01, 5)
        toks = [s.ll_prefill([1, 2, 3])] + [s.ll_decode_step() for _ in range(30)]
        assert max(toks) <= 31 and len(set(toks)) > 5


def test_ties_among_a_few_large_logits(torch_cuda):
    """Two groups of ids share one LM-head row each (r and -r), the rest is zero: whichever group is
    positive forms ~100 equal largest logits scattered over the vocabulary, so the cut runs through
    ties that sit in different threads' ranges; the draw must be the oracle's, exactly."""
    cfg = wl.custom_cfg(1, 2, 64, 136, 3000, 40)
    w = wl.make_weights_numpy(cfg, seed=53)
    r = w["lm_head"][0].copy() * 8
    w["lm_head"][:] = 0
    w["lm_head"][5::29] = r
    w["lm_head"][11::31] = -r
    with _session(cfg, wl.weights_astype(w, np.float16)) as s:
        for k, p in ((7, 1.0), (64, 1.0), (64, 0.5), (150, 1.0), (150, 0.9)):
            s.ll_reset()
            s.ll_set_sampling(1.0, k, p, 17)
            for i in range(12):
                tok = s.ll_prefill([4, 5, 6]) if i == 0 else s.ll_decode_step()
                logits = s.ll_dbg_get_logits()
                assert (logits == logits.max()).sum() >= 90
                ok, same = _accept(tok, logits, 1.0, k, p, sp.uniform(17, i))
                assert ok, (k, p, i, tok)


def test_streams_are_reproducible_and_seeded(torch_cuda):
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=3)
    w["lm_head"] = w["lm_head"] * 40.0
    prompt = wl.make_tokens(9, cfg["vocab"], seed=9)
    runs = {}
    for name, flags in (("graph", 0), ("eager", 1)):
        with _session(cfg, w, flags) as s:
            s.ll_set_sampling(0.9, 30, 0.9, 42)
            a = [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(25)]
            s.ll_reset()                                   # the setting survives, the stream restarts
            b = [s.ll_prefill(prompt)] + s.ll_decode_n(25).tolist()
            s.ll_reset()
            s.ll_set_sampling(0.9, 30, 0.9, 43)
            c = [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(25)]
            s.ll_reset()
            s.ll_set_sampling(0.0, 0, 1.0, 0)
            g = [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(10)]
            s.ll_reset()
            s.ll_set_sampling(0.5, 1, 1.0, 7)              # top-k = 1 is greedy whatever the draw
            g1 = [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(10)]
            runs[name] = (a, b, c, g, g1)
    for a, b, c, g, g1 in runs.values():
        assert a == b and a != c and g == g1
    assert runs["graph"][0] == runs["eager"][0] and runs["graph"][3] == runs["eager"][3]
    with _session(cfg, w) as s:                            # never set: greedy, as before
        assert [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(10)] == runs["graph"][3]


def test_sampling_error_paths(torch_cuda):
    from paper_2604_23467_amd import binding as b
    cfg = wl.custom_cfg(1, 2, 64, 136, 33000, 12)
    w = wl.make_weights_numpy(cfg, seed=5)
    with _session(cfg, w) as s:
        with pytest.raises(b.LLError) as e:
            s.ll_set_sampling(1.0, 0, 1.0, 1)
        assert e.value.code == b.LL_E_CAPACITY
        s.ll_set_sampling(0.0, 0, 1.0, 1)                  # greedy is fine at any vocabulary
        for bad in ((-1.0, 0, 1.0), (float("nan"), 0, 1.0), (1.0, -2, 1.0), (1.0, 0, 0.0), (1.0, 0, 1.01)):
            with pytest.raises(b.LLError) as e:
                s.ll_set_sampling(*bad, 1)
            assert e.value.code == b.LL_E_BAD_ARG
    cfg = wl.tiny_cfg(max_seq=32)
    with _session(cfg, wl.make_weights_numpy(cfg, seed=1), flags=b.LL_FLAG_PERSISTENT) as s:
        with pytest.raises(b.LLError) as e:
            s.ll_set_sampling(1.0, 0, 1.0, 1)
        assert e.value.code == b.LL_E_STATE
        assert s.ll_prefill([1, 2, 3]) >= 0
