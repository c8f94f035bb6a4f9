"""Shared helpers of the GPU parity tests: run the HIP path (through the C ABI
binding) and the CPU oracle on the same seeded inputs and compare.

Acceptance (fp16 GPU path against the fp32 oracle):
  logits   max-abs error <= 3e-2 and relative L2 error <= 1e-2
  tokens   identical wherever the oracle's top-2 logit margin exceeds 0.1; and, on every greedy
           step, bit-exact against the lowest index among the maxima of the GPU's OWN logits
           (index work: no tolerance)
  K/V rows relative L2 error of the whole cache < 3e-3 and, element by element,
           |gpu - ref| <= 2e-2 * rms(ref row) + 2^-10 * |ref|
           (the logits' max-abs bound of 3e-2 on values of rms ~1.3 is 2.3e-2 of their rms: the same
           bound relative to the row; half an fp16 ulp of the stored value is 2^-11 |v|.  One wrong
           element of one row, e.g. a zero or a neighbour's value, fails it).  The last layers of the
           32-layer model are held to the logits' own relative bound instead (rel-L2 <= 1e-2, the
           element bound widened in proportion): their K/V rows are, like the logits, a linear image
           of a residual stream that has collected 32 layers of fp16 operand rounding.
Parity runs are teacher-forced: every step feeds the oracle's token to both
sides, so one low-margin disagreement cannot derail the comparison.
"""
import numpy as np

LOGIT_MAX_ABS = 3e-2
LOGIT_REL_L2 = 1e-2
TOKEN_MARGIN = 0.1
KV_REL_L2 = 3e-3
KV_ROW_REL = 2e-2
KV_ELEM_REL = 2.0 ** -10


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def max_abs(a, b):
    return float(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)).max())


def top2_margin(logits):
    part = np.partition(np.asarray(logits, dtype=np.float64), -2)[-2:]
    return float(part[1] - part[0])


def check_logits(gpu, ref, what, max_abs_tol=LOGIT_MAX_ABS, rel_tol=LOGIT_REL_L2):
    assert np.isfinite(gpu).all(), "%s: non-finite GPU output" % what
    ma, rl = max_abs(gpu, ref), rel_l2(gpu, ref)
    assert ma <= max_abs_tol, "%s: max-abs %.3e > %.1e (rel-L2 %.3e)" % (what, ma, max_abs_tol, rl)
    assert rl <= rel_tol, "%s: rel-L2 %.3e > %.1e (max-abs %.3e)" % (what, rl, rel_tol, ma)
    return ma, rl


def check_token(gpu_tok, ref_tok, ref_logits, what):
    margin = top2_margin(ref_logits)
    if margin > TOKEN_MARGIN:
        assert gpu_tok == ref_tok, "%s: token %d != oracle %d at margin %.3f" % (what, gpu_tok, ref_tok, margin)
    return margin


def check_greedy_token(gpu_tok, gpu_logits, what):
    """Greedy selection is index work: the returned id must be the lowest index among the maxima of
    the logits the GPU itself produced, exactly."""
    want = int(np.flatnonzero(gpu_logits == gpu_logits.max())[0])
    assert gpu_tok == want, "%s: token %d is not the lowest-index argmax %d of the GPU's own logits" % (
        what, gpu_tok, want)


def check_kv(gpu, ref, what, rel_tol=KV_REL_L2):
    """Cached K or V rows [n_pos, d_model] against the oracle's, row by row and element by element."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, "%s: shape %s != %s" % (what, gpu.shape, ref.shape)
    assert np.isfinite(gpu).all(), "%s: non-finite cache rows" % what
    rl = rel_l2(gpu, ref)
    assert rl < rel_tol, "%s: rel-L2 %.3e >= %.1e" % (what, rl, rel_tol)
    row_rms = np.sqrt(np.mean(ref * ref, axis=1, keepdims=True))
    bound = KV_ROW_REL * (rel_tol / KV_REL_L2) * row_rms + KV_ELEM_REL * np.abs(ref)
    excess = np.abs(gpu - ref) - bound
    if (excess > 0).any():
        p, e = np.unravel_index(int(np.argmax(excess)), excess.shape)
        raise AssertionError("%s: position %d element %d: gpu %.6f ref %.6f, bound %.3e" % (
            what, p, e, gpu[p, e], ref[p, e], bound[p, e]))
    return rl


def oracle_trace(omodel, prompt, n_steps):
    """The oracle's own greedy run: [(token, logits, hidden)] for the prefill and n_steps steps."""
    out = [omodel.prefill(prompt)]
    for _ in range(n_steps):
        out.append(omodel.step(out[-1][0]))
    return out


def run_teacher_forced(sess, omodel, prompt, n_steps, label="", trace=None, greedy=True):
    """Prefill + n_steps decode steps on both sides, the oracle's tokens fed to
    both.  Asserts parity at every step; returns per-step (max_abs, rel_l2, margin).
    `trace` (from oracle_trace on the same prompt) replaces the live oracle run, so that one
    oracle pass can serve several GPU modes."""
    stats = []
    nxt = iter(trace) if trace is not None else None
    t_ref, l_ref, h_ref = next(nxt) if nxt else omodel.prefill(prompt)
    t_gpu = sess.ll_prefill(prompt)
    lg = sess.ll_dbg_get_logits()
    ma, rl = check_logits(lg, l_ref, "%s prefill(%d) logits" % (label, len(prompt)))
    hg = sess.ll_dbg_get_hidden()
    check_logits(hg, h_ref, "%s prefill(%d) hidden" % (label, len(prompt)),
                 max_abs_tol=LOGIT_MAX_ABS * max(1.0, float(np.abs(h_ref).max())))
    mg = check_token(t_gpu, t_ref, l_ref, "%s prefill(%d)" % (label, len(prompt)))
    if greedy:
        check_greedy_token(t_gpu, lg, "%s prefill(%d)" % (label, len(prompt)))
    stats.append((ma, rl, mg))
    for i in range(n_steps):
        if t_gpu != t_ref:
            sess.ll_dbg_force_next_token(t_ref)
        t_in = t_ref
        t_ref, l_ref, h_ref = next(nxt) if nxt else omodel.step(t_in)
        t_gpu = sess.ll_decode_step()
        lg = sess.ll_dbg_get_logits()
        ma, rl = check_logits(lg, l_ref, "%s step %d logits" % (label, i))
        mg = check_token(t_gpu, t_ref, l_ref, "%s step %d" % (label, i))
        if greedy:
            check_greedy_token(t_gpu, lg, "%s step %d" % (label, i))
        stats.append((ma, rl, mg))
    return stats


def gated_steps(stats):
    """Number of steps whose oracle margin made the token comparison binding."""
    return sum(1 for s in stats if s[2] > TOKEN_MARGIN)
