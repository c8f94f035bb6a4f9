"""Seeded synthetic inputs: model shapes, random weights, random prompts.

This module only draws numbers.  It holds none of the decoder's arithmetic, so
both the HIP path and the CPU oracle may be fed from it without sharing any of
the method's code.  The paper evaluates LLaMA-2 7B at batch 1 with prompts of
10-500 tokens and up to 500 generated tokens (Sec. IV-E); its trained weights
and prompts are not available, so weights are i.i.d. N(0, 0.02^2) and token
ids are uniform, which leaves every shape, byte count and kernel unchanged.
"""
import numpy as np

CFG_KEYS = ("n_layers", "d_model", "n_heads", "head_dim", "ffn_hidden", "vocab", "max_seq",
            "rope_theta", "rms_eps")
LAYER_KEYS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")
WEIGHT_STD = 0.02


def tiny_cfg(max_seq=64):
    """2-layer toy decoder: d=256, 4 heads x 64, FFN 688, vocab 1024."""
    return dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, ffn_hidden=688, vocab=1024,
                max_seq=max_seq, rope_theta=10000.0, rms_eps=1e-5)


def llama7b_cfg(n_layers=32, vocab=32000, max_seq=1024):
    """LLaMA-2-7B shape: d=4096, 32 heads x 128, FFN 11008, vocab 32000."""
    return dict(n_layers=n_layers, d_model=4096, n_heads=32, head_dim=128, ffn_hidden=11008,
                vocab=vocab, max_seq=max_seq, rope_theta=10000.0, rms_eps=1e-5)


def custom_cfg(n_layers, n_heads, head_dim, ffn_hidden, vocab, max_seq, rope_theta=10000.0,
               rms_eps=1e-5):
    return dict(n_layers=n_layers, d_model=n_heads * head_dim, n_heads=n_heads, head_dim=head_dim,
                ffn_hidden=ffn_hidden, vocab=vocab, max_seq=max_seq, rope_theta=rope_theta,
                rms_eps=rms_eps)


def weight_shapes(cfg):
    """(top-level shapes, per-layer shapes); every linear map is [out, in]."""
    d, F, V = cfg["d_model"], cfg["ffn_hidden"], cfg["vocab"]
    top = dict(tok_emb=(V, d), final_norm=(d,), lm_head=(V, d))
    layer = dict(attn_norm=(d,), wq=(d, d), wk=(d, d), wv=(d, d), wo=(d, d), ffn_norm=(d,),
                 w_gate=(F, d), w_up=(F, d), w_down=(d, F))
    return top, layer


def make_weights_numpy(cfg, seed=0, dtype=np.float32, gain_jitter=0.0, emb_std=WEIGHT_STD):
    """numpy weights, N(0, 0.02^2); RMSNorm gains 1.0 (+ optional N(0, jitter^2))."""
    rng = np.random.default_rng(seed)
    top, layer = weight_shapes(cfg)

    def draw(name, shape):
        if name.endswith("norm"):
            g = np.ones(shape, dtype=np.float64)
            if gain_jitter:
                g = g + gain_jitter * rng.standard_normal(shape)
            return g.astype(dtype)
        std = emb_std if name == "tok_emb" else WEIGHT_STD
        return (std * rng.standard_normal(shape)).astype(dtype)

    w = {k: draw(k, s) for k, s in top.items()}
    w["layers"] = [{k: draw(k, layer[k]) for k in LAYER_KEYS} for _ in range(cfg["n_layers"])]
    return w


def make_weights_torch(cfg, seed=0, device="cuda", emb_std=WEIGHT_STD):
    """fp16 torch weights drawn on `device` (one seeded generator per tensor).

    Used for the 7B shapes, where drawing 6.7e9 normals on the host would take
    minutes.  The same tensors, copied to the host, feed the oracle.
    """
    import torch
    top, layer = weight_shapes(cfg)
    counter = [0]

    def draw(name, shape):
        counter[0] += 1
        if name.endswith("norm"):
            return torch.ones(shape, dtype=torch.float16, device=device)
        g = torch.Generator(device=device)
        g.manual_seed(seed * 1000003 + counter[0])
        std = emb_std if name == "tok_emb" else WEIGHT_STD
        t = torch.empty(shape, dtype=torch.float32, device=device)
        t.normal_(0.0, std, generator=g)
        return t.to(torch.float16)

    w = {k: draw(k, s) for k, s in top.items()}
    w["layers"] = [{k: draw(k, layer[k]) for k in LAYER_KEYS} for _ in range(cfg["n_layers"])]
    return w


def weights_to_numpy(w):
    """torch weight dict -> numpy dict on the host (same bits)."""
    conv = lambda t: t.detach().cpu().numpy()
    out = {k: conv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: conv(v) for k, v in L.items()} for L in w["layers"]]
    return out


def weights_to_torch(w, device="cuda", dtype=None):
    """numpy weight dict -> torch dict on `device` (optionally cast, e.g. to fp16)."""
    import torch
    def conv(a):
        t = torch.from_numpy(np.ascontiguousarray(a))
        if dtype is not None:
            t = t.to(dtype)
        return t.to(device).contiguous()
    out = {k: conv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: conv(v) for k, v in L.items()} for L in w["layers"]]
    return out


def weights_astype(w, dtype):
    """numpy weight dict cast to another numpy dtype (e.g. fp32 -> fp16 -> fp32)."""
    out = {k: np.asarray(v).astype(dtype) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: np.asarray(v).astype(dtype) for k, v in L.items()} for L in w["layers"]]
    return out


def make_tokens(n, vocab, seed=0):
    """n token ids uniform in [0, vocab)."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def sweep_token_seed(prompt_len, rep):
    """Seed of repetition `rep` of the latency sweep at one prompt length."""
    return 1000 * prompt_len + rep
