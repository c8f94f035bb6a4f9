"""Thin ctypes binding of ``libll.so`` (declarations: ``include/ll.h``).

Argument marshalling only: every step of the decode / prefill path runs in the
HIP kernels behind the C ABI.  PyTorch appears here solely as the owner of
device memory (weights, workspace) and of the HIP stream.  There is no CPU
fallback: a missing library raises.
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libll.so")

LL_OK = 0
LL_E_NOT_INIT, LL_E_BAD_CONFIG, LL_E_BAD_ARG, LL_E_CAPACITY = -1, -2, -3, -4
LL_E_WORKSPACE, LL_E_STATE, LL_E_HIP, LL_E_ALREADY_INIT = -5, -6, -7, -8
LL_FLAG_EAGER = 1
LL_FLAG_MULTIKERNEL = 2
LL_FLAG_PERSISTENT = 4
LL_FLAG_PER_LENGTH_GRAPHS = 8
LL_FLAG_FUSED_ATTN_OPROJ = 16
LL_FLAG_LEAN_WORKSPACE = 32
LL_MODE_PERSISTENT_GRAPH, LL_MODE_MULTIKERNEL_GRAPH, LL_MODE_EAGER, LL_MODE_PER_LENGTH_GRAPHS = 0, 1, 2, 3
KERNEL_CLASSES = ("embed", "qkv", "attn", "oproj", "gateup", "down", "lmhead", "sample")
LAYER_KEYS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")

EXPORTS = ("ll_workspace_bytes", "ll_init", "ll_prefill", "ll_prefill_static", "ll_decode_step", "ll_decode_n", "ll_reset",
           "ll_set_sampling", "ll_shutdown", "ll_max_prompt", "ll_position", "ll_decode_mode", "ll_last_error", "ll_dbg_get_logits",
           "ll_batch_pool_bytes", "ll_batch_open", "ll_batch_add", "ll_batch_step", "ll_batch_remove", "ll_batch_close",
           "ll_batch_dbg_get_logits", "ll_batch_dbg_force_next_token", "ll_batch_dbg_time_steps",
           "ll_dbg_get_hidden", "ll_dbg_graph_stats", "ll_dbg_gemm_plan", "ll_dbg_gemm_slice_count", "ll_dbg_force_next_token", "ll_dbg_get_kv", "ll_dbg_profile_decode",
           "ll_dbg_time_decode", "ll_dbg_time_kernel_class", "ll_dbg_stream_copy", "ll_dbg_stream_read", "ll_dbg_poison_scratch", "ll_dbg_trace_decode")


class LLConfig(C.Structure):
    _fields_ = [(k, C.c_int32) for k in
                ("n_layers", "d_model", "n_heads", "head_dim", "ffn_hidden", "vocab", "max_seq")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float), ("flags", C.c_int32)]


class LLLayerWeights(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in LAYER_KEYS]


class LLWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("layers", C.POINTER(LLLayerWeights)),
                ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class LLError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("ll error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load():
    """Loads libll.so (built beforehand by ``paper_2604_23467_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("HIP library %s is missing: run `python -m paper_2604_23467_amd.build` "
                           "(there is no CPU fallback)" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    L.ll_workspace_bytes.restype = C.c_size_t
    L.ll_workspace_bytes.argtypes = [C.POINTER(LLConfig)]
    L.ll_init.restype = C.c_int
    L.ll_init.argtypes = [C.POINTER(LLConfig), C.POINTER(LLWeights), C.c_void_p, C.c_size_t, C.c_void_p]
    L.ll_prefill.restype = C.c_int32
    L.ll_prefill.argtypes = [C.POINTER(C.c_int32), C.c_int32]
    L.ll_prefill_static.restype = C.c_int32
    L.ll_prefill_static.argtypes = [C.POINTER(C.c_int32), C.c_int32]
    L.ll_decode_step.restype = C.c_int32
    L.ll_decode_step.argtypes = []
    L.ll_decode_n.restype = C.c_int32
    L.ll_decode_n.argtypes = [C.c_int32, C.POINTER(C.c_int32)]
    for name in ("ll_reset", "ll_shutdown", "ll_dbg_poison_scratch"):
        getattr(L, name).restype = C.c_int
        getattr(L, name).argtypes = []
    for name in ("ll_max_prompt", "ll_position", "ll_decode_mode"):
        getattr(L, name).restype = C.c_int32
        getattr(L, name).argtypes = []
    L.ll_set_sampling.restype = C.c_int
    L.ll_set_sampling.argtypes = [C.c_float, C.c_int32, C.c_float, C.c_uint64]
    L.ll_last_error.restype = C.c_char_p
    L.ll_last_error.argtypes = []
    L.ll_dbg_get_logits.restype = C.c_int
    L.ll_dbg_get_logits.argtypes = [C.POINTER(C.c_float)]
    L.ll_batch_pool_bytes.restype = C.c_size_t
    L.ll_batch_pool_bytes.argtypes = [C.c_int32, C.c_int32]
    L.ll_batch_open.restype = C.c_int
    L.ll_batch_open.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t]
    L.ll_batch_add.restype = C.c_int32
    L.ll_batch_add.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32)]
    L.ll_batch_step.restype = C.c_int
    L.ll_batch_step.argtypes = [C.POINTER(C.c_int32)]
    L.ll_batch_remove.restype = C.c_int
    L.ll_batch_remove.argtypes = [C.c_int32]
    L.ll_batch_close.restype = C.c_int
    L.ll_batch_close.argtypes = []
    L.ll_batch_dbg_get_logits.restype = C.c_int
    L.ll_batch_dbg_get_logits.argtypes = [C.c_int32, C.POINTER(C.c_float)]
    L.ll_batch_dbg_force_next_token.restype = C.c_int
    L.ll_batch_dbg_force_next_token.argtypes = [C.c_int32, C.c_int32]
    L.ll_batch_dbg_time_steps.restype = C.c_int
    L.ll_batch_dbg_time_steps.argtypes = [C.c_int32, C.POINTER(C.c_float)]
    L.ll_dbg_gemm_plan.restype = C.c_int
    L.ll_dbg_gemm_plan.argtypes = [C.c_int32] * 4 + [C.POINTER(C.c_int32)]
    L.ll_dbg_gemm_slice_count.restype = C.c_int
    L.ll_dbg_gemm_slice_count.argtypes = [C.c_int32] * 5
    L.ll_dbg_graph_stats.restype = C.c_int
    L.ll_dbg_graph_stats.argtypes = [C.POINTER(C.c_int64)]
    L.ll_dbg_get_hidden.restype = C.c_int
    L.ll_dbg_get_hidden.argtypes = [C.POINTER(C.c_float)]
    L.ll_dbg_force_next_token.restype = C.c_int
    L.ll_dbg_force_next_token.argtypes = [C.c_int32]
    L.ll_dbg_get_kv.restype = C.c_int
    L.ll_dbg_get_kv.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float)]
    L.ll_dbg_profile_decode.restype = C.c_int
    L.ll_dbg_profile_decode.argtypes = [C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    L.ll_dbg_time_kernel_class.restype = C.c_int
    L.ll_dbg_time_kernel_class.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_float)]
    L.ll_dbg_trace_decode.restype = C.c_int
    L.ll_dbg_trace_decode.argtypes = [C.POINTER(C.c_uint64), C.c_int32]
    L.ll_dbg_stream_copy.restype = C.c_int
    L.ll_dbg_stream_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
    L.ll_dbg_stream_read.restype = C.c_int
    L.ll_dbg_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.POINTER(C.c_float)]
    L.ll_dbg_time_decode.restype = C.c_int
    L.ll_dbg_time_decode.argtypes = [C.c_int32, C.POINTER(C.c_float)]
    _lib = L
    return L


def _check(rc):
    if rc < 0:
        raise LLError(rc, load().ll_last_error().decode())
    return rc


def make_config(cfg, flags=0):
    return LLConfig(**{k: int(cfg[k]) for k in ("n_layers", "d_model", "n_heads", "head_dim",
                                                  "ffn_hidden", "vocab", "max_seq")},
                    rope_theta=float(cfg["rope_theta"]), rms_eps=float(cfg["rms_eps"]), flags=flags)


def ll_workspace_bytes(cfg, flags=0):
    c = make_config(cfg, flags)
    return int(load().ll_workspace_bytes(C.byref(c)))


def ll_dbg_stream_copy(dst, src):
    """Copies one contiguous CUDA tensor into another of the same byte size."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    return _check(load().ll_dbg_stream_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()),
                                            C.c_size_t(nbytes)))


def ll_dbg_stream_read(src, reps=4):
    """GB/s of a read-only streaming pass over one contiguous CUDA tensor."""
    import torch
    sink = torch.zeros(4096, dtype=torch.int32, device=src.device)
    out = C.c_float(0.0)
    _check(load().ll_dbg_stream_read(C.c_void_p(src.data_ptr()), C.c_size_t(src.numel() * src.element_size()),
                                     reps, C.c_void_p(sink.data_ptr()), C.byref(out)))
    return float(out.value)


def ll_set_sampling_raw(temperature, top_k, top_p, seed):
    """ll_set_sampling on whatever instance the library holds (an error without one)."""
    return _check(load().ll_set_sampling(C.c_float(temperature), C.c_int32(top_k), C.c_float(top_p),
                                         C.c_uint64(seed)))


def ll_dbg_gemm_plan(N, K, nmat, rows):
    """Work distribution of the prefill projection GEMM (host arithmetic, no GPU needed)."""
    out = (C.c_int32 * 6)()
    _check(load().ll_dbg_gemm_plan(N, K, nmat, rows, out))
    return dict(zip(("row_tile", "row_tiles", "runs", "quota", "tile_slabs", "max_slices"), out))


def ll_dbg_gemm_slice_count(N, K, nmat, rows, col):
    return _check(load().ll_dbg_gemm_slice_count(N, K, nmat, rows, col))


def ll_last_error():
    return load().ll_last_error().decode()


class Session:
    """Owns the torch tensors the library points into, for the life of one ll_init()."""

    def __init__(self, cfg, weights, flags=0, stream=None, device="cuda:0"):
        """``weights``: dict of fp16 torch tensors on ``device`` (see workloads.weight_shapes)."""
        import torch
        self.torch = torch
        self.cfg = dict(cfg)
        self.lib = load()
        self.device = torch.device(device)
        self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        self._weights = weights
        for name, t in self._iter_weights(weights):
            if t.dtype != torch.float16 or not t.is_contiguous() or t.device.type != "cuda":
                raise ValueError("weight %s must be a contiguous fp16 CUDA tensor" % name)
        self._layers = (LLLayerWeights * cfg["n_layers"])()
        for i, Lw in enumerate(weights["layers"]):
            for k in LAYER_KEYS:
                setattr(self._layers[i], k, Lw[k].data_ptr())
        self._w = LLWeights(tok_emb=weights["tok_emb"].data_ptr(),
                            layers=C.cast(self._layers, C.POINTER(LLLayerWeights)),
                            final_norm=weights["final_norm"].data_ptr(),
                            lm_head=weights["lm_head"].data_ptr())
        self._cfg = make_config(cfg, flags)
        nbytes = int(self.lib.ll_workspace_bytes(C.byref(self._cfg)))
        if nbytes == 0:
            raise LLError(LL_E_BAD_CONFIG, "ll_workspace_bytes rejected the configuration")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        torch.cuda.synchronize(self.device)
        _check(self.lib.ll_init(C.byref(self._cfg), C.byref(self._w), C.c_void_p(self._ws_ptr),
                                C.c_size_t(nbytes), C.c_void_p(self.stream.cuda_stream)))
        self.open = True

    @staticmethod
    def _iter_weights(w):
        for k, v in w.items():
            if k == "layers":
                for i, Lw in enumerate(v):
                    for kk, vv in Lw.items():
                        yield "layers[%d].%s" % (i, kk), vv
            else:
                yield k, v

    # ---- the four calls ------------------------------------------------
    def ll_prefill(self, tokens):
        arr = np.ascontiguousarray(tokens, dtype=np.int32)
        return _check(self.lib.ll_prefill(arr.ctypes.data_as(C.POINTER(C.c_int32)), arr.shape[0]))

    def ll_prefill_static(self, tokens):
        arr = np.ascontiguousarray(tokens, dtype=np.int32)
        return _check(self.lib.ll_prefill_static(arr.ctypes.data_as(C.POINTER(C.c_int32)), arr.shape[0]))

    def ll_decode_step(self):
        return _check(self.lib.ll_decode_step())

    def ll_decode_n(self, k):
        out = np.empty(k, dtype=np.int32)
        _check(self.lib.ll_decode_n(k, out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out

    def ll_reset(self):
        return _check(self.lib.ll_reset())

    def ll_set_sampling(self, temperature, top_k=0, top_p=1.0, seed=0):
        return ll_set_sampling_raw(temperature, top_k, top_p, seed)

    def ll_shutdown(self):
        if self.open:
            self.open = False
            rc = _check(self.lib.ll_shutdown())
            self.workspace = None          # the library is done with it
            self.pool = None
            return rc
        return 0

    close = ll_shutdown

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def ll_max_prompt(self):
        return _check(self.lib.ll_max_prompt())

    def ll_decode_mode(self):
        return _check(self.lib.ll_decode_mode())

    def ll_position(self):
        return _check(self.lib.ll_position())

    # ---- hooks ---------------------------------------------------------
    def ll_dbg_get_logits(self):
        out = np.empty(self.cfg["vocab"], dtype=np.float32)
        _check(self.lib.ll_dbg_get_logits(out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    # ---- batched decoding over a paged KV cache ----
    def ll_batch_open(self, max_batch, page_tokens, n_pages):
        nbytes = int(self.lib.ll_batch_pool_bytes(page_tokens, n_pages))
        if nbytes == 0:
            raise LLError(LL_E_BAD_ARG, "ll_batch_pool_bytes rejected the arguments")
        self.pool = self.torch.empty(nbytes + 256, dtype=self.torch.uint8, device=self.device)
        ptr = (self.pool.data_ptr() + 255) // 256 * 256
        self.max_batch = max_batch
        return _check(self.lib.ll_batch_open(max_batch, page_tokens, n_pages, C.c_void_p(ptr), C.c_size_t(nbytes)))

    def ll_batch_add(self, tokens):
        arr = (C.c_int32 * len(tokens))(*[int(t) for t in tokens])
        first = C.c_int32(-1)
        slot = _check(self.lib.ll_batch_add(arr, len(tokens), C.byref(first)))
        return slot, int(first.value)

    def ll_batch_step(self):
        out = (C.c_int32 * self.max_batch)()
        _check(self.lib.ll_batch_step(out))
        return list(out)

    def ll_batch_remove(self, slot):
        return _check(self.lib.ll_batch_remove(slot))

    def ll_batch_close(self):
        rc = _check(self.lib.ll_batch_close())
        self.pool = None
        return rc

    def ll_batch_dbg_get_logits(self, slot):
        out = np.empty(self.cfg["vocab"], dtype=np.float32)
        _check(self.lib.ll_batch_dbg_get_logits(slot, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def ll_batch_dbg_force_next_token(self, slot, tok):
        return _check(self.lib.ll_batch_dbg_force_next_token(slot, int(tok)))

    def ll_batch_dbg_time_steps(self, k):
        ms = C.c_float(0)
        _check(self.lib.ll_batch_dbg_time_steps(k, C.byref(ms)))
        return float(ms.value)

    def ll_dbg_graph_stats(self):
        out = (C.c_int64 * 4)()
        _check(self.lib.ll_dbg_graph_stats(out))
        return dict(buffered_replays=out[0], blocking_captures=out[1], overlapped_captures=out[2],
                    capture_ms=out[3] / 1e6)

    def ll_dbg_get_hidden(self):
        out = np.empty(self.cfg["d_model"], dtype=np.float32)
        _check(self.lib.ll_dbg_get_hidden(out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def ll_dbg_poison_scratch(self):
        return _check(self.lib.ll_dbg_poison_scratch())

    def ll_dbg_force_next_token(self, tok):
        return _check(self.lib.ll_dbg_force_next_token(int(tok)))

    def ll_dbg_get_kv(self, layer, which, n_pos):
        out = np.empty((n_pos, self.cfg["d_model"]), dtype=np.float32)
        _check(self.lib.ll_dbg_get_kv(layer, which, n_pos, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def ll_dbg_profile_decode(self, steps):
        us = np.zeros(len(KERNEL_CLASSES), dtype=np.float32)
        n = np.zeros(len(KERNEL_CLASSES), dtype=np.int32)
        _check(self.lib.ll_dbg_profile_decode(steps, us.ctypes.data_as(C.POINTER(C.c_float)),
                                              n.ctypes.data_as(C.POINTER(C.c_int32))))
        return {k: (float(us[i]), int(n[i])) for i, k in enumerate(KERNEL_CLASSES)}

    def ll_dbg_time_kernel_class(self, name, reps):
        us = C.c_float(0.0)
        _check(self.lib.ll_dbg_time_kernel_class(KERNEL_CLASSES.index(name), reps, C.byref(us)))
        return float(us.value)

    def ll_dbg_trace_decode(self):
        """[phases][5] timestamps in microseconds relative to the first one."""
        n = 5 * self.cfg["n_layers"] + 1
        buf = np.zeros((n, 8), dtype=np.uint64)
        _check(self.lib.ll_dbg_trace_decode(buf.ctypes.data_as(C.POINTER(C.c_uint64)), n))
        return (buf.astype(np.int64) - np.int64(buf[0, 0])) / 100.0

    def ll_dbg_time_decode(self, k):
        ms = C.c_float(0.0)
        _check(self.lib.ll_dbg_time_decode(k, C.byref(ms)))
        return float(ms.value)
