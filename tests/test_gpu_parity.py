"""Parity of the HIP path (called through the C ABI) against the CPU oracle on
the same seeded inputs.  Needs a real MI355X: run with ``-m gpu``."""
import numpy as np
import pytest

from paper_2604_23467_amd import workloads as wl
from parity_utils import (LOGIT_REL_L2, check_greedy_token, check_kv, check_logits, check_token, gated_steps, max_abs,
                          oracle_trace, rel_l2, run_teacher_forced, top2_margin)

pytestmark = pytest.mark.gpu
DEFAULT_MODE = 1      # what ll_init picks without LL_FLAG_PERSISTENT / LL_FLAG_MULTIKERNEL


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need a GPU"
    return torch


def _session(cfg, w_np, flags=0):
    import torch
    from paper_2604_23467_amd import binding
    w_t = wl.weights_to_torch(w_np, device="cuda:0", dtype=torch.float16)
    return binding.Session(cfg, w_t, flags=flags)


# ------------------------------------------------------------ config 1: tiny model
@pytest.mark.parametrize("flags", [4, 2, 1, 0, 8, 16, 17],
                         ids=["persistent", "multikernel", "eager", "default", "per-length-graphs", "fused-attn-oproj", "fused-eager"])
def test_tiny_config_prefill_and_16_steps(torch_cuda, oracle32, flags):
    """2 layers, d=256, 4x64 heads, FFN 688, vocab 1024, fp32 weights seed 0,
    10-token prompt seed 0, prefill + 16 greedy steps.  The oracle keeps the
    original fp32 weights; the GPU gets them rounded to fp16."""
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=0)
    prompt = wl.make_tokens(10, cfg["vocab"], seed=0)
    om = oracle32.model(cfg, w)
    with _session(cfg, w, flags) as s:
        assert s.ll_decode_mode() == {4: 0, 2: 1, 1: 2, 0: DEFAULT_MODE, 8: 3, 16: DEFAULT_MODE, 17: 2}[flags]
        stats = run_teacher_forced(s, om, prompt, 16, "tiny")
        assert s.ll_position() == 26 and om.pos == 26
        # the token comparison with the oracle must have been binding somewhere
        assert gated_steps(stats) > 0, [round(x[2], 3) for x in stats]
        # K/V rows the GPU cached (fp16) against the oracle's, both layers, element by element
        for layer in range(cfg["n_layers"]):
            for which in (0, 1):
                check_kv(s.ll_dbg_get_kv(layer, which, 26), om.kv(layer, which), "tiny layer %d %s" % (layer, "KV"[which]))
    om.close()
    print("tiny worst max-abs %.2e rel-L2 %.2e" % (max(x[0] for x in stats), max(x[1] for x in stats)))


def test_tiny_config_fp16_rounded_weights_isolate_kernel_error(torch_cuda, oracle32):
    """Same run against the oracle on fp16-rounded weights: what is left is the
    kernels' own error (fp16 KV cache / prefill activations, summation order)."""
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=0)
    w16 = wl.weights_astype(w, np.float16)
    prompt = wl.make_tokens(10, cfg["vocab"], seed=0)
    om = oracle32.model(cfg, w16)
    with _session(cfg, w) as s:
        stats = run_teacher_forced(s, om, prompt, 16, "tiny-fp16w")
    om.close()
    assert max(x[1] for x in stats) < 5e-3


# ------------------------------------------------------------ shapes, tails, buckets
SHAPES = [
    # (n_layers, n_heads, head_dim, ffn, vocab, max_seq, prompt_len, steps)
    (1, 2, 128, 344, 777, 80, 1, 3),        # head_dim 128, odd vocab, single-token prompt
    (2, 4, 64, 688, 1024, 200, 63, 2),      # just under a 64-row tile
    (2, 4, 64, 688, 1024, 200, 64, 2),      # exactly one tile
    (2, 4, 64, 688, 1024, 200, 65, 2),      # one row into the next bucket
    (1, 3, 128, 1000, 501, 300, 150, 4),    # d=384 (K not a multiple of 512), ragged FFN
    (2, 2, 64, 136, 33, 40, 7, 30),         # tiny everything, decode to near max_seq
    (1, 2, 64, 4616, 100, 48, 5, 3),        # FFN rows of 10 chunks: down projection split in 2 K segments
    (1, 2, 64, 8712, 100, 48, 5, 3),        # 18 chunks: 3 K segments, ragged last one
]


@pytest.mark.parametrize("flags", [4, 2, 18], ids=["persistent", "multikernel", "fused-attn-oproj"])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "L%d_H%dx%d_F%d_V%d_S%d_p%d" % s[:7])
def test_shapes_tails_and_buckets(torch_cuda, oracle32, shape, flags):
    n_layers, H, dh, F, V, max_seq, n_prompt, steps = shape
    cfg = wl.custom_cfg(n_layers, H, dh, F, V, max_seq)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=21, gain_jitter=0.1), np.float16)
    prompt = wl.make_tokens(n_prompt, V, seed=n_prompt)
    om = oracle32.model(cfg, w)
    with _session(cfg, w, flags) as s:
        run_teacher_forced(s, om, prompt, steps, "shape")
        for which in range(2):
            check_kv(s.ll_dbg_get_kv(n_layers - 1, which, n_prompt + steps), om.kv(n_layers - 1, which), "shape %s" % "KV"[which])
    om.close()


@pytest.mark.parametrize("n_prompt", [5, 20])
def test_short_prompt_wide_model(torch_cuda, oracle32, n_prompt):
    """d_model 4224 > 4096: the short-prompt Q/K/V and gate/up projections cannot keep their
    activations in registers and take the general kernel."""
    cfg = wl.custom_cfg(1, 33, 128, 64, 64, 40)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=41, gain_jitter=0.1), np.float16)
    prompt = wl.make_tokens(n_prompt, cfg["vocab"], seed=n_prompt)
    om = oracle32.model(cfg, w)
    with _session(cfg, w) as s:
        run_teacher_forced(s, om, prompt, 2, "wide")
        for which in range(2):
            check_kv(s.ll_dbg_get_kv(0, which, n_prompt + 2), om.kv(0, which), "wide %s" % "KV"[which])
    om.close()


@pytest.mark.parametrize("flags", [0, 1, 32], ids=["graph", "eager", "lean-workspace"])
@pytest.mark.parametrize("n_prompt", [2, 15, 16, 17, 31, 32, 33, 50])
def test_short_prompt_row_blocks(torch_cuda, oracle32, n_prompt, flags):
    """Prompts around the 16 / 32 / 64-row boundaries of the short-prompt kernels, head_dim 128
    and an FFN width whose K range ends inside an MFMA step; every K and V cache row is compared."""
    cfg = wl.custom_cfg(2, 2, 128, 344, 300, 100)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=31, gain_jitter=0.1), np.float16)
    prompt = wl.make_tokens(n_prompt, cfg["vocab"], seed=100 + n_prompt)
    om = oracle32.model(cfg, w)
    with _session(cfg, w, flags) as s:
        run_teacher_forced(s, om, prompt, 2, "short")
        for layer in range(2):
            for which in range(2):
                check_kv(s.ll_dbg_get_kv(layer, which, n_prompt + 2), om.kv(layer, which),
                         "short prompt %d layer %d %s" % (n_prompt, layer, "KV"[which]))
    om.close()


def test_larger_activations_exercise_softmax_and_rope(torch_cuda, oracle32):
    """Weights scaled up so attention is far from uniform and RoPE matters."""
    cfg = wl.custom_cfg(2, 4, 64, 256, 300, 160)
    w = wl.make_weights_numpy(cfg, seed=22, gain_jitter=0.2, emb_std=1.0)
    for L in w["layers"]:
        for k in ("wq", "wk"):
            L[k] *= 6.0
    w = wl.weights_astype(w, np.float16)
    prompt = wl.make_tokens(90, cfg["vocab"], seed=5)
    om = oracle32.model(cfg, w)
    with _session(cfg, w) as s:
        run_teacher_forced(s, om, prompt, 20, "sharp")
    om.close()


# ------------------------------------------------------------ runtime behaviour
def test_graph_replay_equals_eager_and_decode_n(torch_cuda):
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=3)
    prompt = wl.make_tokens(12, cfg["vocab"], seed=9)
    runs = {}
    for name, flags in (("graph", 4), ("multi", 2), ("eager", 1)):
        with _session(cfg, w, flags) as s:
            t1 = s.ll_prefill(prompt)
            toks = [t1] + [s.ll_decode_step() for _ in range(10)]
            logits = s.ll_dbg_get_logits()
            s.ll_reset()
            assert s.ll_position() == 0
            t1b = s.ll_prefill(prompt)
            toks_n = [t1b] + s.ll_decode_n(10).tolist()
            logits_n = s.ll_dbg_get_logits()
            runs[name] = (toks, logits, toks_n, logits_n)
    g, m, e = runs["graph"], runs["multi"], runs["eager"]
    for r in (g, m, e):
        assert r[0] == r[2]                           # decode_n == repeated decode_step, reset works
    assert g[0] == e[0] == m[0]
    # every kernel sums in a fixed order, so the modes differ by nothing but how launches are issued
    assert max_abs(m[1], e[1]) < 1e-4 and max_abs(g[1], e[1]) < 1e-4 and max_abs(g[1], g[3]) < 1e-4


@pytest.mark.parametrize("n_prompt", [9, 27, 200])
def test_runs_are_bit_reproducible(torch_cuda, n_prompt):
    """No kernel on the path accumulates in arrival order (no floating-point atomics): the same
    prompt gives the same bits, run after run and instance after instance; one 7B-shaped layer, so
    that the short-prompt projections run with their full 256 workgroups."""
    from paper_2604_23467_amd import binding
    cfg = wl.llama7b_cfg(n_layers=1, vocab=512, max_seq=256)
    w_t = wl.make_weights_torch(cfg, seed=5, device="cuda:0", emb_std=1.0)
    prompt = wl.make_tokens(n_prompt, cfg["vocab"], seed=n_prompt)
    runs = []
    for inst in range(2):
        with binding.Session(cfg, w_t) as s:
            for rep in range(3):
                s.ll_reset()
                t1 = s.ll_prefill(prompt)
                lp, hp = s.ll_dbg_get_logits(), s.ll_dbg_get_hidden()
                toks = s.ll_decode_n(3).tolist()
                runs.append((t1, toks, lp.tobytes(), hp.tobytes(), s.ll_dbg_get_logits().tobytes(),
                             s.ll_dbg_get_kv(0, 0, n_prompt + 3).tobytes()))
    assert all(r == runs[0] for r in runs[1:])


@pytest.mark.parametrize("flags", [0, 1], ids=["graph", "eager"])
@pytest.mark.parametrize("n_prompt,max_seq", [(600, 1200), (1025, 1200), (1052, 2000), (1112, 2000), (2124, 3500)])
def test_chunked_prefill_of_long_prompts(torch_cuda, oracle32, n_prompt, max_seq, flags):
    """600 tokens fill part of the largest (1024-row) bucket; prompts beyond it are fed in chunks:
    1024 + a 1-row, a 28-row (short-prompt kernels at a position offset) and an 88-row chunk, and two
    full chunks + 76 rows, in instances of different capacity."""
    cfg = wl.custom_cfg(2, 2, 64, 136, 200, max_seq)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=61, gain_jitter=0.1, emb_std=0.5), np.float16)
    prompt = wl.make_tokens(n_prompt, cfg["vocab"], seed=n_prompt)
    om = oracle32.model(cfg, w)
    with _session(cfg, w, flags) as s:
        assert s.ll_max_prompt() == max_seq - 1
        run_teacher_forced(s, om, prompt, 3, "chunked")
        for which in range(2):
            check_kv(s.ll_dbg_get_kv(1, which, n_prompt + 3), om.kv(1, which), "chunked %s" % "KV"[which])
    om.close()


def test_per_length_graph_buffer_replays_the_same_tokens(torch_cuda):
    """The paper's mechanism (one graph per KV length, rolling buffer of 8, next length captured
    while the current one replays) must generate what the single graph generates."""
    from paper_2604_23467_amd import binding as b
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=3)
    prompt = wl.make_tokens(12, cfg["vocab"], seed=9)
    with _session(cfg, w) as s:
        ref = [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(30)]
    with _session(cfg, w, b.LL_FLAG_PER_LENGTH_GRAPHS) as s:
        assert s.ll_decode_mode() == b.LL_MODE_PER_LENGTH_GRAPHS
        got = [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(20)] + s.ll_decode_n(10).tolist()
        st = s.ll_dbg_graph_stats()
        # the first step captures its own graph; every later one finds the graph captured during the step before
        assert got == ref and st["blocking_captures"] == 1 and st["overlapped_captures"] == 30
        assert st["buffered_replays"] == 29 and st["capture_ms"] > 0
        s.ll_reset()                       # lengths 12..19 left the 8-deep buffer long ago: the cycle restarts
        again = [s.ll_prefill(prompt)] + [s.ll_decode_step() for _ in range(5)]
        assert again == ref[:6] and s.ll_dbg_graph_stats()["blocking_captures"] == 2
        s.ll_reset()
        s.ll_prefill(prompt[:11])          # lengths 11.. : 11 is new, 12..17 are still buffered
        s.ll_decode_n(4)
        st2 = s.ll_dbg_graph_stats()
        assert st2["blocking_captures"] == 3 and st2["overlapped_captures"] == 35
    for bad in (b.LL_FLAG_PER_LENGTH_GRAPHS | b.LL_FLAG_EAGER, b.LL_FLAG_PER_LENGTH_GRAPHS | b.LL_FLAG_PERSISTENT):
        with pytest.raises(b.LLError) as e:
            _session(cfg, w, bad)
        assert e.value.code == b.LL_E_BAD_CONFIG


@pytest.mark.parametrize("flags", [0, 1, 4, 16], ids=["graph", "eager", "persistent", "fused-attn-oproj"])
@pytest.mark.parametrize("n_prompt", [9, 70])
def test_poisoned_scratch_changes_nothing(torch_cuda, flags, n_prompt):
    """Every scratch buffer is written before it is read: with NaN patterns planted in all of them
    before the prefill and between the decode steps, tokens and logits come out bit-identical."""
    cfg = wl.custom_cfg(2, 4, 64, 688, 512, 128)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=4, gain_jitter=0.1), np.float16)
    prompt = wl.make_tokens(n_prompt, cfg["vocab"], seed=2)
    with _session(cfg, w, flags) as s:
        ref = [(s.ll_prefill(prompt), s.ll_dbg_get_logits())]
        for _ in range(6):
            ref.append((s.ll_decode_step(), s.ll_dbg_get_logits()))
        s.ll_reset()
        s.ll_dbg_poison_scratch()
        got = [(s.ll_prefill(prompt), s.ll_dbg_get_logits())]
        for _ in range(6):
            s.ll_dbg_poison_scratch()
            got.append((s.ll_decode_step(), s.ll_dbg_get_logits()))
    for (t0, l0), (t1, l1) in zip(ref, got):
        assert t0 == t1 and np.isfinite(l1).all() and np.array_equal(l0, l1)


def test_prefill_matches_token_by_token_decode(torch_cuda, oracle32):
    """The MFMA prefill and the GEMV decode path are two implementations of the
    same layer: feeding the prompt through decode steps must give the same
    logits and cache as one prefill call."""
    cfg = wl.custom_cfg(2, 4, 64, 688, 512, 128)
    w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=4, gain_jitter=0.1), np.float16)
    prompt = wl.make_tokens(40, cfg["vocab"], seed=2)
    with _session(cfg, w) as s:
        s.ll_prefill(prompt)
        lp = s.ll_dbg_get_logits()
        kp = s.ll_dbg_get_kv(1, 0, 40)
        s.ll_reset()
        s.ll_prefill(prompt[:1])
        for t in prompt[1:]:
            s.ll_dbg_force_next_token(int(t))
            s.ll_decode_step()
        ld = s.ll_dbg_get_logits()
        kd = s.ll_dbg_get_kv(1, 0, 40)
    assert rel_l2(lp, ld) < 5e-3 and rel_l2(kp, kd) < 3e-3


def test_error_paths_on_device(torch_cuda):
    from paper_2604_23467_amd import binding as b
    cfg = wl.custom_cfg(1, 2, 64, 136, 50, 12)
    w = wl.make_weights_numpy(cfg, seed=5)
    with _session(cfg, w) as s:
        assert s.ll_max_prompt() == 11
        with pytest.raises(b.LLError) as e:
            s.ll_decode_step()                          # empty context
        assert e.value.code == b.LL_E_STATE
        with pytest.raises(b.LLError) as e:
            s.ll_prefill(np.array([1, 50], dtype=np.int32))   # token out of range
        assert e.value.code == b.LL_E_BAD_ARG
        with pytest.raises(b.LLError) as e:
            s.ll_prefill(np.arange(12, dtype=np.int32))       # n + 1 > max_seq
        assert e.value.code == b.LL_E_CAPACITY
        assert s.ll_position() == 0                           # failed calls left the state alone
        s.ll_prefill(np.arange(5, dtype=np.int32))
        with pytest.raises(b.LLError) as e:
            s.ll_prefill(np.arange(5, dtype=np.int32))        # non-empty context
        assert e.value.code == b.LL_E_STATE
        s.ll_decode_n(7)                                      # fills the cache to max_seq = 12
        assert s.ll_position() == 12
        with pytest.raises(b.LLError) as e:
            s.ll_decode_step()
        assert e.value.code == b.LL_E_CAPACITY
        # a second init while one is live is refused
        lib = b.load()
        assert lib.ll_init(s._cfg, s._w, None, 0, None) == b.LL_E_ALREADY_INIT
        s.ll_reset()
        assert s.ll_prefill(np.arange(3, dtype=np.int32)) >= 0


# ------------------------------------------------------------ config 2: one 7B-shaped layer
@pytest.mark.parametrize("kv_len", [10, 25, 50, 128, 250, 500])      # one length per prefill bucket
def test_one_7b_layer_decode_step(torch_cuda, oracle32, kv_len):
    """d=4096, 32x128 heads, FFN 11008, fp16 N(0,0.02) weights.  The cache is
    filled by prefilling kv_len random hidden states (token i's embedding is an
    N(0,1) row, vocab = kv_len + 1); the step under test feeds row kv_len at
    position kv_len and attends kv_len + 1 keys.  Hidden state and logits
    (through a random LM head) are compared."""
    import torch
    from paper_2604_23467_amd import binding
    cfg = wl.llama7b_cfg(n_layers=1, vocab=kv_len + 1, max_seq=kv_len + 2)
    w_t = wl.make_weights_torch(cfg, seed=0, device="cuda:0", emb_std=1.0)
    w_np = wl.weights_to_numpy(w_t)
    prompt = np.arange(kv_len, dtype=np.int32)
    om = oracle32.model(cfg, w_np)
    om.prefill(prompt)
    _, l_ref, h_ref = om.step(kv_len)
    with binding.Session(cfg, w_t) as s:
        s.ll_prefill(prompt)
        s.ll_dbg_force_next_token(kv_len)
        s.ll_decode_step()
        h = s.ll_dbg_get_hidden()
        lg = s.ll_dbg_get_logits()
        k_gpu = s.ll_dbg_get_kv(0, 0, kv_len + 1)
        v_gpu = s.ll_dbg_get_kv(0, 1, kv_len + 1)
    check_logits(h, h_ref, "7B layer kv=%d hidden" % kv_len,
                 max_abs_tol=3e-2 * max(1.0, float(np.abs(h_ref).max())))
    check_logits(lg, l_ref, "7B layer kv=%d logits" % kv_len)
    check_kv(k_gpu, om.kv(0, 0), "7B layer kv=%d K" % kv_len)
    check_kv(v_gpu, om.kv(0, 1), "7B layer kv=%d V" % kv_len)
    om.close()


@pytest.mark.parametrize("flags", [2, 4, 18], ids=["multikernel", "persistent", "fused-attn-oproj"])
def test_one_7b_layer_long_decode_to_kv_1000(torch_cuda, oracle32, flags):
    """Decode-path attention at the long end of the regime: prompt 500, then
    500 teacher-forced decode steps (KV grows to 1000) on one 7B-shaped layer;
    hidden state compared at a sample of steps including the last."""
    import torch
    from paper_2604_23467_amd import binding
    n_prompt, n_steps = 500, 500
    cfg = wl.llama7b_cfg(n_layers=1, vocab=1024, max_seq=n_prompt + n_steps + 1)
    w_t = wl.make_weights_torch(cfg, seed=1, device="cuda:0", emb_std=1.0)
    w_np = wl.weights_to_numpy(w_t)
    toks = wl.make_tokens(n_prompt + n_steps, cfg["vocab"], seed=8)
    om = oracle32.model(cfg, w_np)
    om.prefill(toks[:n_prompt])
    check_at = {0, 1, 63, 64, 255, 256, 498, 499}
    with binding.Session(cfg, w_t, flags=flags) as s:
        s.ll_prefill(toks[:n_prompt])
        for i in range(n_steps):
            t_in = int(toks[n_prompt + i])
            s.ll_dbg_force_next_token(t_in)
            s.ll_decode_step()
            _, l_ref, h_ref = om.step(t_in)
            if i in check_at:
                check_logits(s.ll_dbg_get_hidden(), h_ref, "long decode step %d hidden" % i,
                             max_abs_tol=3e-2 * max(1.0, float(np.abs(h_ref).max())))
                check_logits(s.ll_dbg_get_logits(), l_ref, "long decode step %d logits" % i)
        assert s.ll_position() == 1000
    om.close()


# ------------------------------------------------------------ configs 3 and 4: full 7B-shaped model
@pytest.fixture(scope="module")
def full_7b(torch_cuda):
    """32 layers, vocab 32000, fp16 N(0,0.02) weights seed 0: drawn on the GPU once for the module,
    the same bits on the host for the oracle."""
    cfg = wl.llama7b_cfg(max_seq=1024)
    w_t = wl.make_weights_torch(cfg, seed=0, device="cuda:0")
    w_np = wl.weights_to_numpy(w_t)
    yield cfg, w_t, w_np
    del w_t
    torch_cuda.cuda.empty_cache()


def test_full_7b_prompt10_100_steps_graph_and_eager(full_7b, oracle32):
    """Config 3: 10-token prompt seed 0, prefill + all 100 greedy decode steps, teacher-forced,
    as graph replays and as eager launches (one oracle run serves both); the persistent kernel
    follows the same trace for its first 6 steps."""
    from paper_2604_23467_amd import binding
    cfg, w_t, w_np = full_7b
    prompt = wl.make_tokens(10, cfg["vocab"], seed=0)
    om = oracle32.model(cfg, w_np)
    trace = oracle_trace(om, prompt, 100)
    for flags, label, n in ((binding.LL_FLAG_MULTIKERNEL, "7B graph", 100), (binding.LL_FLAG_EAGER, "7B eager", 100),
                            (binding.LL_FLAG_PERSISTENT, "7B persistent", 6)):
        with binding.Session(cfg, w_t, flags=flags) as s:
            stats = run_teacher_forced(s, om, prompt, n, label, trace=trace)
            assert gated_steps(stats) > 0
            assert s.ll_position() == 10 + n
            for which in range(2):
                check_kv(s.ll_dbg_get_kv(31, which, 10 + n), om.kv(31, which, 10 + n), "%s layer 31 %s" % (label, "KV"[which]))
            # full-size LM head, sampled rows recomputed one by one from the GPU's own hidden state
            h = s.ll_dbg_get_hidden().astype(np.float64)
            lg = s.ll_dbg_get_logits()
        a = h / np.sqrt(np.mean(h * h) + float(np.float32(cfg["rms_eps"])))
        rows = np.random.default_rng(0).integers(0, cfg["vocab"], size=64)
        ref = w_np["lm_head"][rows].astype(np.float64) @ a
        assert np.abs(lg[rows] - ref).max() < 2e-3
        print("%s: %d steps, %d token-gated, worst max-abs %.2e rel-L2 %.2e" % (
            label, n, gated_steps(stats), max(x[0] for x in stats), max(x[1] for x in stats)))
    om.close()


def test_full_7b_prompt500_prefill_and_16_steps(full_7b, oracle32):
    """Config 4, the workload the headline latency is measured on: 500-token prompt seed 0 through
    the 512-row MFMA prefill at full depth (logits, hidden state and the first token at the end of
    the prompt), then the first 16 decode steps teacher-forced, then the K and V rows of the first
    and the last layer.  The remaining 484 steps of the config run the same kernels at longer KV
    lengths, which the one-layer test up to KV 1000 covers."""
    from paper_2604_23467_amd import binding
    cfg, w_t, w_np = full_7b
    prompt = wl.make_tokens(500, cfg["vocab"], seed=0)
    om = oracle32.model(cfg, w_np)
    with binding.Session(cfg, w_t) as s:
        stats = run_teacher_forced(s, om, prompt, 16, "7B prompt 500")
        assert gated_steps(stats) > 0
        assert s.ll_position() == 516 and om.pos == 516
        for layer in (0, 31):
            for which in range(2):
                check_kv(s.ll_dbg_get_kv(layer, which, 516), om.kv(layer, which),
                         "7B prompt 500 layer %d %s" % (layer, "KV"[which]), rel_tol=LOGIT_REL_L2 if layer else 3e-3)
    om.close()
    print("7B prompt 500: prefill max-abs %.2e rel-L2 %.2e; 16 steps worst max-abs %.2e rel-L2 %.2e" % (
        stats[0][0], stats[0][1], max(x[0] for x in stats[1:]), max(x[1] for x in stats[1:])))


@pytest.mark.parametrize("n_prompt", [1044, 1100])
def test_one_7b_layer_long_context_instance(torch_cuda, oracle32, n_prompt):
    """Long-context instance (max_seq > 2048) at head_dim 128: the prompt goes through a 1024-row
    chunk and then a 20-row (short-prompt kernels at a position offset) or a 76-row tail (MFMA GEMM
    bucket, four key groups per query block at an offset); the decode steps run the attention with
    four workgroups per head plus the merge kernel in front of the O projection."""
    from paper_2604_23467_amd import binding
    cfg = wl.llama7b_cfg(n_layers=1, vocab=1024, max_seq=2304)
    w_t = wl.make_weights_torch(cfg, seed=3, device="cuda:0", emb_std=1.0)
    w_np = wl.weights_to_numpy(w_t)
    prompt = wl.make_tokens(n_prompt, cfg["vocab"], seed=n_prompt)
    om = oracle32.model(cfg, w_np)
    with binding.Session(cfg, w_t) as s:
        run_teacher_forced(s, om, prompt, 4, "7B layer long context")
        for which in range(2):
            check_kv(s.ll_dbg_get_kv(0, which, n_prompt + 4), om.kv(0, which), "long context %s" % "KV"[which])
    om.close()


# ------------------------------------------------------------ greedy selection: planted ties
@pytest.mark.parametrize("flags", [0, 1, 4], ids=["graph", "eager", "persistent"])
def test_greedy_ties_resolve_to_the_lowest_index(torch_cuda, flags):
    """Index work, checked exactly.  (1) A zero LM head makes every logit 0: token 0.  (2) Copies of one
    row planted at several vocabulary positions give bit-identical maximal logits in rows that belong to
    different waves and workgroups of the LM-head kernel (and, at vocab 9000, to two passes of one wave):
    the lowest planted index must come back, from the prefill and from a decode step."""
    import torch
    for vocab, planted in ((1024, (901, 10, 333)), (9000, (8801, 8392, 201))):
        cfg = wl.custom_cfg(1, 2, 64, 136, vocab, 24)
        w = wl.weights_astype(wl.make_weights_numpy(cfg, seed=71), np.float16)
        prompt = wl.make_tokens(6, vocab, seed=3)
        zero = dict(w, lm_head=np.zeros_like(w["lm_head"]))
        with _session(cfg, zero, flags) as s:
            assert s.ll_prefill(prompt) == 0 and s.ll_decode_step() == 0
            assert not s.ll_dbg_get_logits().any()
        # a row aligned with the final hidden state wins by a wide margin; the hidden states of the prefill
        # and of the step after it differ, so the planted row is built from their sum
        with _session(cfg, w, flags) as s:
            s.ll_prefill(prompt)
            h = s.ll_dbg_get_hidden().astype(np.float64)
            s.ll_dbg_force_next_token(7)
            s.ll_decode_step()
            h2 = s.ll_dbg_get_hidden().astype(np.float64)
        v = h / np.linalg.norm(h) + h2 / np.linalg.norm(h2)
        tied = dict(w, lm_head=w["lm_head"].copy())
        for r in planted:
            tied["lm_head"][r] = (v / np.linalg.norm(v)).astype(np.float16)
        with _session(cfg, tied, flags) as s:
            for what, tok in (("prefill", s.ll_prefill(prompt)), ("step", None)):
                if tok is None:
                    s.ll_dbg_force_next_token(7)
                    tok = s.ll_decode_step()
                lg = s.ll_dbg_get_logits()
                vals = lg[list(planted)]
                assert (vals == vals[0]).all(), "planted rows did not give identical logits: %r" % (vals,)
                assert vals[0] == lg.max() and (lg == lg.max()).sum() == len(planted)
                assert tok == min(planted), "%s vocab %d: token %d, lowest planted index %d" % (what, vocab, tok, min(planted))


def test_timing_hooks_leave_a_usable_context(torch_cuda, oracle32):
    cfg = wl.tiny_cfg(max_seq=64)
    w = wl.make_weights_numpy(cfg, seed=0)
    prompt = wl.make_tokens(10, cfg["vocab"], seed=0)
    om = oracle32.model(cfg, w)
    with _session(cfg, w) as s:
        s.ll_prefill(prompt)
        for name in ("qkv", "attn", "oproj", "gateup", "down", "lmhead"):
            assert s.ll_dbg_time_kernel_class(name, 2) > 0.0
        assert s.ll_position() == 10
        prof = s.ll_dbg_profile_decode(2)
        assert prof["gateup"][1] == cfg["n_layers"] and prof["oproj"][1] == cfg["n_layers"] and s.ll_position() == 12
        assert s.ll_dbg_time_decode(3) > 0.0 and s.ll_position() == 15
        s.ll_reset()                                   # required after the class timing hook
        run_teacher_forced(s, om, prompt, 3, "after-hooks")
    om.close()
    from paper_2604_23467_amd import binding
    with _session(cfg, w, binding.LL_FLAG_FUSED_ATTN_OPROJ) as s:
        s.ll_prefill(prompt)
        assert s.ll_dbg_time_kernel_class("attn", 2) > 0.0
        with pytest.raises(binding.LLError) as e:           # no launch of its own: it runs inside the attention launch
            s.ll_dbg_time_kernel_class("oproj", 2)
        assert e.value.code == binding.LL_E_STATE
        assert s.ll_dbg_profile_decode(1)["oproj"][1] == 0
    with _session(cfg, w, binding.LL_FLAG_PERSISTENT) as s:
        s.ll_prefill(prompt)
        t = s.ll_dbg_trace_decode()
        assert t.shape == (5 * cfg["n_layers"] + 1, 8) and s.ll_position() == 11
        assert (np.diff(t[:, 4]) > 0).all()            # barrier-passed stamps are ordered
    with _session(cfg, w, binding.LL_FLAG_MULTIKERNEL) as s:
        s.ll_prefill(prompt)
        with pytest.raises(binding.LLError):
            s.ll_dbg_trace_decode()


def test_stream_copy_calibration_kernel(torch_cuda):
    import torch
    from paper_2604_23467_amd import binding
    a = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda:0")
    b = torch.zeros_like(a)
    binding.ll_dbg_stream_copy(b, a)
    assert torch.equal(a, b)
