"""Shared helpers of the GPU parity tests: run the HIP path (through the C ABI
binding) and the CPU oracle on the same seeded inputs and compare.

Acceptance (fp16 GPU path against the fp32 oracle):
  logits   max-abs error <= 3e-2 and relative L2 error <= 1e-2
  tokens   identical wherever the oracle's top-2 logit margin exceeds 0.1
Parity runs are teacher-forced: every step feeds the oracle's token to both
sides, so one low-margin disagreement cannot derail the comparison.
"""
import numpy as np

LOGIT_MAX_ABS = 3e-2
LOGIT_REL_L2 = 1e-2
TOKEN_MARGIN = 0.1


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


def run_teacher_forced(sess, omodel, prompt, n_steps, label=""):
    """Prefill + n_steps decode steps on both sides, the oracle's tokens fed to
    both.  Asserts parity at every step; returns per-step (max_abs, rel_l2, margin)."""
    stats = []
    t_ref, l_ref, h_ref = omodel.prefill(prompt)
    t_gpu = sess.ll_prefill(prompt)
    lg = sess.ll_dbg_get_logits()
    ma, rl = check_logits(lg, l_ref, "%s prefill(%d) logits" % (label, len(prompt)))
    hg = sess.ll_dbg_get_hidden()
    check_logits(hg, h_ref, "%s prefill(%d) hidden" % (label, len(prompt)),
                 max_abs_tol=LOGIT_MAX_ABS * max(1.0, float(np.abs(h_ref).max())))
    mg = check_token(t_gpu, t_ref, l_ref, "%s prefill(%d)" % (label, len(prompt)))
    stats.append((ma, rl, mg))
    for i in range(n_steps):
        if t_gpu != t_ref:
            sess.ll_dbg_force_next_token(t_ref)
        t_in = t_ref
        t_ref, l_ref, h_ref = omodel.step(t_in)
        t_gpu = sess.ll_decode_step()
        lg = sess.ll_dbg_get_logits()
        ma, rl = check_logits(lg, l_ref, "%s step %d logits" % (label, i))
        mg = check_token(t_gpu, t_ref, l_ref, "%s step %d" % (label, i))
        stats.append((ma, rl, mg))
    return stats
