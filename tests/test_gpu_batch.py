"""Batched lock-step decoding over the paged KV cache against the CPU oracle: every sequence of
the batch is an independent oracle run (batching must not change what a sequence computes).
Same acceptance as the single-sequence parity tests, teacher-forced per slot."""
import numpy as np
import pytest

from paper_2604_23467_amd import workloads as wl
from parity_utils import check_logits, check_token

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need a GPU"
    return torch


def _session(cfg, w_np, flags=0):
    import torch
    from paper_2604_23467_amd import binding
    return binding.Session(cfg, wl.weights_to_torch(w_np, device="cuda:0", dtype=torch.float16), flags=flags)


class Seq:
    """One sequence on both sides: its slot in the batch and its oracle model."""

    def __init__(self, sess, oracle, cfg, w, prompt, label):
        self.om = oracle.model(cfg, w)
        self.label = label
        self.t_ref, self.l_ref, _ = self.om.prefill(prompt)
        self.slot, t_gpu = sess.ll_batch_add(prompt)
        check_token(t_gpu, self.t_ref, self.l_ref, "%s first token" % label)
        if t_gpu != self.t_ref:
            sess.ll_batch_dbg_force_next_token(self.slot, self.t_ref)
        self.steps = 0

    def advance_oracle(self):
        self.t_ref, self.l_ref, _ = self.om.step(self.t_ref)
        self.steps += 1

    def check(self, sess, toks):
        what = "%s step %d (slot %d)" % (self.label, self.steps, self.slot)
        stat = check_logits(sess.ll_batch_dbg_get_logits(self.slot), self.l_ref, what + " logits")
        check_token(toks[self.slot], self.t_ref, self.l_ref, what)
        if toks[self.slot] != self.t_ref:
            sess.ll_batch_dbg_force_next_token(self.slot, self.t_ref)
        return stat


def _step_all(sess, seqs):
    for q in seqs:
        q.advance_oracle()
    toks = sess.ll_batch_step()
    occupied = {q.slot for q in seqs}
    assert all((t >= 0) == (b in occupied) for b, t in enumerate(toks)), toks
    return [q.check(sess, toks) for q in seqs]


@pytest.mark.parametrize("flags", [0, 1, 32], ids=["graph", "eager", "lean-workspace"])
def test_tiny_batch_with_sequences_joining_and_leaving(torch_cuda, oracle32, flags):
    """Pages of 8 positions, so every sequence crosses several page borders; a sequence joins while
    others are running, one leaves and its pages serve a newcomer."""
    cfg = wl.tiny_cfg(max_seq=96)
    w = wl.make_weights_numpy(cfg, seed=0)
    prompts = [wl.make_tokens(n, cfg["vocab"], seed=100 + n) for n in (5, 12, 33, 1, 20)]
    worst = 0.0
    with _session(cfg, w, flags) as s:
        s.ll_batch_open(4, 8, 40)
        a = Seq(s, oracle32, cfg, w, prompts[0], "A")
        b = Seq(s, oracle32, cfg, w, prompts[1], "B")
        assert (a.slot, b.slot) == (0, 1)
        for _ in range(10):
            worst = max(worst, max(x[1] for x in _step_all(s, [a, b])))
        c = Seq(s, oracle32, cfg, w, prompts[2], "C")          # 33 tokens: the GEMM prefill path, 5 pages
        d = Seq(s, oracle32, cfg, w, prompts[3], "D")          # one-token prompt
        for _ in range(12):
            worst = max(worst, max(x[1] for x in _step_all(s, [a, b, c, d])))
        s.ll_batch_remove(b.slot)
        e = Seq(s, oracle32, cfg, w, prompts[4], "E")
        assert e.slot == b.slot
        for _ in range(9):
            worst = max(worst, max(x[1] for x in _step_all(s, [a, c, d, e])))
        s.ll_batch_close()
        # the single-sequence calls still work afterwards
        assert s.ll_reset() == 0 and s.ll_prefill(prompts[0]) >= 0 and s.ll_decode_step() >= 0
    for q in (a, b, c, d, e):
        q.om.close()
    print("tiny batch worst rel-L2 %.2e" % worst)


def test_batch_of_16_on_a_7b_shaped_layer(torch_cuda, oracle32):
    """One LLaMA-2-7B-shaped layer with the full vocabulary, 16 sequences of different lengths."""
    cfg = wl.custom_cfg(1, 32, 128, 11008, 32000, 96)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=7), np.float16)
    lens = [3, 40, 17, 8, 25, 1, 33, 12, 5, 29, 16, 2, 37, 21, 9, 31]
    with _session(cfg, w) as s:
        s.ll_batch_open(16, 16, 16 * 4 + 1)
        seqs = [Seq(s, oracle32, cfg, w, wl.make_tokens(n, cfg["vocab"], seed=n), "len%d" % n) for n in lens]
        assert [q.slot for q in seqs] == list(range(16))
        worst = 0.0
        for _ in range(4):
            worst = max(worst, max(x[1] for x in _step_all(s, seqs)))
        ms = s.ll_batch_dbg_time_steps(3) / 3
        assert 0.0 < ms < 50.0
        s.ll_batch_close()
    for q in seqs:
        q.om.close()
    print("7B-layer batch worst rel-L2 %.2e" % worst)


def test_32_slot_batch_on_the_tiny_model(torch_cuda, oracle32):
    """More than 16 slots: the step runs 32 rows (two token blocks); 20 sequences, 12 free slots."""
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=4)
    with _session(cfg, w) as s:
        s.ll_batch_open(32, 4, 20 * 12 + 1)
        seqs = [Seq(s, oracle32, cfg, w, wl.make_tokens(1 + (7 * i) % 23, cfg["vocab"], seed=300 + i), "s%d" % i)
                for i in range(20)]
        assert [q.slot for q in seqs] == list(range(20))
        worst = 0.0
        for _ in range(9):
            worst = max(worst, max(x[1] for x in _step_all(s, seqs)))
        s.ll_batch_close()
    for q in seqs:
        q.om.close()
    print("32-slot batch worst rel-L2 %.2e" % worst)


def test_batched_steps_are_bit_reproducible(torch_cuda):
    """The batched step sums in a fixed order too: two identical batches give identical logits."""
    cfg = wl.custom_cfg(1, 32, 128, 1024, 512, 64)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=8), np.float16)
    prompts = [wl.make_tokens(n, cfg["vocab"], seed=50 + n) for n in (3, 11, 20, 6, 15)]
    runs = []
    with _session(cfg, w) as s:
        for rep in range(2):
            s.ll_batch_open(8, 8, 60)
            slots = [s.ll_batch_add(p)[0] for p in prompts]
            toks = [s.ll_batch_step() for _ in range(5)]
            runs.append((toks, [s.ll_batch_dbg_get_logits(b).tobytes() for b in slots]))
            s.ll_batch_close()
    assert runs[0] == runs[1]


def test_stochastic_selection_per_slot(torch_cuda):
    """ll_set_sampling applies to the batch as well: every slot draws with its own index (tokens its
    sequence has produced), so a sequence that joins later starts its stream at index 1 while the
    others are further along.  Checked like the single-sequence sampler: the oracle's draw on the
    GPU's own logits, with the rounding-aware acceptance rule."""
    from oracle import sampling as sp
    from test_gpu_sampling import _accept
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=3)
    w["lm_head"] = w["lm_head"] * 40.0
    T, k, p, seed = 0.9, 30, 0.9, 42
    with _session(cfg, w) as s:
        s.ll_set_sampling(T, k, p, seed)
        s.ll_batch_open(3, 8, 30)
        drawn = {}
        exact = total = 0

        def add(prompt):
            slot, tok = s.ll_batch_add(prompt)
            ok, same = _accept(tok, s.ll_dbg_get_logits(), T, k, p, sp.uniform(seed, 0))   # the prefill's draw: index 0
            assert ok, ("first token", slot, tok)
            drawn[slot] = 1
            return slot

        def step():
            nonlocal exact, total
            toks = s.ll_batch_step()
            for slot in list(drawn):
                ok, same = _accept(toks[slot], s.ll_batch_dbg_get_logits(slot), T, k, p, sp.uniform(seed, drawn[slot]))
                assert ok, ("slot %d draw %d: token %d is not a valid draw" % (slot, drawn[slot], toks[slot]))
                exact += same
                total += 1
                drawn[slot] += 1
            return toks

        a = add(wl.make_tokens(9, cfg["vocab"], seed=9))
        b = add(wl.make_tokens(4, cfg["vocab"], seed=10))
        first = [step() for _ in range(6)]
        c = add(wl.make_tokens(13, cfg["vocab"], seed=11))
        for _ in range(10):
            step()
        assert exact >= 0.95 * total, (exact, total)
        assert len({t[a] for t in first} | {t[b] for t in first}) > 3          # not a constant stream
        # greedy again: the setting is read from device memory by the same captured step
        s.ll_set_sampling(0.0, 0, 1.0, 0)
        toks = s.ll_batch_step()
        for slot in (a, b, c):
            lg = s.ll_batch_dbg_get_logits(slot)
            assert toks[slot] == int(np.flatnonzero(lg == lg.max())[0])
        s.ll_batch_close()


def test_batch_capacity_and_error_paths(torch_cuda):
    from paper_2604_23467_amd import binding as b
    cfg = wl.tiny_cfg(max_seq=40)
    w = wl.make_weights_numpy(cfg, seed=2)
    p = wl.make_tokens(6, cfg["vocab"], seed=1)
    with _session(cfg, w) as s:
        for call in (lambda: s.ll_batch_step(), lambda: s.ll_batch_add(p), lambda: s.ll_batch_remove(0)):
            s.max_batch = 2
            with pytest.raises(b.LLError) as e:
                call()
            assert e.value.code == b.LL_E_STATE
        for bad in ((0, 8, 4), (33, 8, 4), (2, 0, 4), (2, 8, 1)):
            with pytest.raises(b.LLError):
                s.ll_batch_open(*bad)
        s.ll_batch_open(2, 8, 4)                       # 3 usable pages of 8 positions
        with pytest.raises(b.LLError) as e:
            s.ll_batch_open(2, 8, 4)
        assert e.value.code == b.LL_E_STATE
        with pytest.raises(b.LLError) as e:
            s.ll_batch_step()                          # empty batch
        assert e.value.code == b.LL_E_STATE
        s0, _ = s.ll_batch_add(p)                      # 7 positions: 1 page
        s1, _ = s.ll_batch_add(wl.make_tokens(9, cfg["vocab"], seed=3))    # 10 positions: 2 pages, pool now empty
        with pytest.raises(b.LLError) as e:
            s.ll_batch_add(p)                          # no slot left
        assert e.value.code == b.LL_E_CAPACITY
        assert s.ll_batch_step()[0] >= 0               # positions 6 and 9: inside the pages held
        assert s.ll_batch_step()[0] >= 0               # positions 7 and 10
        with pytest.raises(b.LLError) as e:
            s.ll_batch_step()                          # slot 0 reaches position 8: needs a page, none free
        assert e.value.code == b.LL_E_CAPACITY
        with pytest.raises(b.LLError) as e:
            s.ll_batch_remove(5)
        assert e.value.code == b.LL_E_BAD_ARG
        s.ll_batch_remove(s1)
        toks = s.ll_batch_step()                       # now it can take one
        assert toks[s0] >= 0 and toks[s1] == -1
        with pytest.raises(b.LLError) as e:
            s.ll_batch_add(list(wl.make_tokens(40, cfg["vocab"], seed=4)))   # 41 positions > max_seq
        assert e.value.code == b.LL_E_CAPACITY
        s.ll_batch_close()
    for flags in (b.LL_FLAG_PERSISTENT, b.LL_FLAG_PER_LENGTH_GRAPHS):      # step graphs of their own: not combined
        with _session(cfg, w, flags) as s:
            with pytest.raises(b.LLError) as e:
                s.ll_batch_open(2, 8, 4)
            assert e.value.code == b.LL_E_STATE

