"""Pins of the sampling oracle (oracle/sampling.py) against things it does not
define itself: published Philox vectors, closed forms, limiting cases that
reduce to argmax or to a uniform draw, and the frequencies of many draws."""
import json
import os

import numpy as np
import pytest
from oracle import sampling as sp

HERE = os.path.dirname(os.path.abspath(__file__))


def test_philox_known_answers():
    kat = json.load(open(os.path.join(HERE, "golden", "philox4x32_10_kat.json")))
    for v in kat["vectors"]:
        got = sp.philox4x32_10([int(x, 16) for x in v["counter"]], [int(x, 16) for x in v["key"]])
        assert ["%08x" % x for x in got] == v["out"]


def test_uniform_is_a_24_bit_fraction_and_depends_on_seed_and_index():
    us = [sp.uniform(7, i) for i in range(2000)]
    assert all(0.0 <= u < 1.0 and (u * 2 ** 24) == int(u * 2 ** 24) for u in us)
    assert abs(np.mean(us) - 0.5) < 0.03 and abs(np.var(us) - 1 / 12) < 0.01
    assert sp.uniform(7, 5) != sp.uniform(8, 5) and sp.uniform(7, 5) != sp.uniform(7, 6)
    assert sp.uniform((1 << 32) + 7, 5) != sp.uniform(7, 5)          # the high word is key material


def test_equal_logits_give_a_uniform_draw_in_index_order():
    # e_i all equal: the running sum crosses u * n at token floor(u * n)
    z = np.full(50, 1.25, dtype=np.float32)
    for u in (0.0, 0.019, 0.5, 0.98, 0.999999):
        tok, _ = sp.sample(z, 1.0, 0, 1.0, u)
        assert tok == int(np.floor(u * 50))
    # top-k on ties keeps the k lowest indices
    tok, info = sp.sample(z, 1.0, 7, 1.0, 0.999)
    assert list(np.flatnonzero(info["cand"])) == list(range(7)) and tok == 6


def test_limits_reduce_to_argmax():
    rng = np.random.default_rng(0)
    z = rng.normal(size=300).astype(np.float32)
    best = int(np.argmax(z))
    for u in (0.0, 0.3, 0.99):
        assert sp.sample(z, 1.0, 1, 1.0, u)[0] == best            # top-k = 1
        assert sp.sample(z, 1e-4, 0, 1.0, u)[0] == best           # temperature -> 0
        assert sp.sample(z, 1.0, 0, 1e-9, u)[0] == best           # nucleus of vanishing mass
    assert sp.sample_step(z, 0.0, 0, 1.0, 1, 0)[0] == best        # greedy switch


def test_top_k_and_top_p_sets_against_a_sorted_brute_force():
    rng = np.random.default_rng(1)
    for trial in range(20):
        v = int(rng.integers(5, 400))
        z = rng.normal(scale=2.0, size=v).astype(np.float32)
        z[rng.integers(0, v, size=3)] = z[0]                      # some exact ties
        k = int(rng.integers(0, v + 3))
        p = float(rng.uniform(0.05, 1.0))
        _, info = sp.sample(z, 0.7, k, p, 0.5)
        zz = (z * np.float32(1.0 / 0.7)).astype(np.float32)
        order = sorted(range(v), key=lambda i: (-float(zz[i]), i))
        cand = order[:k] if 0 < k < v else order
        assert set(np.flatnonzero(info["cand"])) == set(cand)
        prob = np.exp(zz[cand].astype(np.float64) - float(zz[cand[0]]))
        prob /= prob.sum()
        # minimal prefix of the sorted candidates whose mass reaches p
        r = int(np.searchsorted(np.cumsum(prob), p - 1e-12)) + 1
        keep = set(cand[:min(r, len(cand))])
        got = set(np.flatnonzero(info["keep"]))
        assert got == keep or abs(np.cumsum(prob)[len(got) - 1] - p) < 1e-9 or abs(np.cumsum(prob)[len(keep) - 1] - p) < 1e-9


def test_draw_frequencies_match_the_softmax_probabilities():
    z = np.array([2.0, 0.5, 1.0, -1.0, 0.0, 1.5], dtype=np.float32)
    t = 0.8
    p = np.exp(z.astype(np.float64) / t)
    p /= p.sum()
    n = 40000
    counts = np.zeros(6)
    for i in range(n):
        counts[sp.sample_step(z, t, 0, 1.0, 12345, i)[0]] += 1
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    assert chi2 < 25.0, (chi2, counts / n, p)                      # 5 degrees of freedom: P(chi2 > 25) ~ 1e-4


def test_top_p_renormalises_inside_the_nucleus():
    z = np.log(np.array([0.5, 0.3, 0.15, 0.05])).astype(np.float32)
    _, info = sp.sample(z, 1.0, 0, 0.7, 0.0)
    assert list(np.flatnonzero(info["keep"])) == [0, 1]           # 0.5 < 0.7 <= 0.8
    # inside {0, 1}: token 0 with probability 0.5 / 0.8
    assert sp.sample(z, 1.0, 0, 0.7, 0.62)[0] == 0 and sp.sample(z, 1.0, 0, 0.7, 0.63)[0] == 1


def test_index_order_walk_and_last_token_fallback():
    z = np.log(np.array([0.1, 0.6, 0.3])).astype(np.float32)
    assert [sp.sample(z, 1.0, 0, 1.0, u)[0] for u in (0.05, 0.1, 0.69, 0.7, 0.99)] == [0, 1, 1, 2, 2]
    tok, info = sp.sample(z, 1.0, 0, 1.0, 1.0)                    # u = 1 cannot be drawn; the walk still ends inside
    assert tok == 2


@pytest.mark.parametrize("bad", [dict(temperature=-1.0), dict(top_k=-1), dict(top_p=0.0), dict(top_p=1.5)])
def test_binding_rejects_bad_sampling_parameters_without_a_gpu(bad):
    from paper_2604_23467_amd import binding
    args = dict(temperature=1.0, top_k=0, top_p=1.0, seed=1)
    args.update(bad)
    with pytest.raises(binding.LLError):
        binding.ll_set_sampling_raw(**args)                       # not initialised or bad argument: an error either way
