"""ctypes binding of ``oracle.c`` (the fp32 oracle, and its fp64 twin).

TEST INFRASTRUCTURE ONLY: see ``oracle.c``.  ``build()`` compiles the C file
with gcc into ``liboracle_f32.so`` / ``liboracle_f64.so`` next to this file;
``Oracle(precision)`` loads one of them (compiling it first if it is absent).

Weights are passed as a dict of numpy arrays (see ``full_recompute.py`` for the
keys), all float32 or all float16; they are used in place, never copied.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")

_LAYER_KEYS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class OracleConfig(C.Structure):
    _fields_ = [(k, C.c_int32) for k in
                ("n_layers", "d_model", "n_heads", "head_dim", "ffn_hidden", "vocab", "max_seq")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class OracleLayer(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in _LAYER_KEYS]


class OracleWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("layers", C.POINTER(OracleLayer)),
                ("final_norm", C.c_void_p), ("lm_head", C.c_void_p), ("dtype", C.c_int32)]


def lib_path(precision):
    return os.path.join(_HERE, "liboracle_%s.so" % precision)


def build(force=False):
    """Compile both precisions of the oracle with gcc."""
    for precision, flag in (("f32", []), ("f64", ["-DORACLE_F64"])):
        out = lib_path(precision)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra"] + flag + \
              ["-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)


def _ptr(a):
    return C.c_void_p(a.ctypes.data)


class Oracle:
    """One loaded oracle library; ``real`` is its numpy dtype."""

    def __init__(self, precision="f32"):
        assert precision in ("f32", "f64")
        build()
        self.lib = C.CDLL(lib_path(precision))
        self.real = np.float32 if precision == "f32" else np.float64
        L = self.lib
        assert L.oracle_real_bytes() == np.dtype(self.real).itemsize
        L.oracle_half_to_float.restype = C.c_float
        L.oracle_half_to_float.argtypes = [C.c_uint16]
        L.oracle_rmsnorm.restype = None
        L.oracle_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_float, C.c_void_p]
        L.oracle_matvec.restype = None
        L.oracle_matvec.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.oracle_rope.restype = None
        L.oracle_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float]
        L.oracle_attention_head.restype = None
        L.oracle_attention_head.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                            C.c_int, C.c_void_p, C.c_void_p]
        L.oracle_swiglu.restype = None
        L.oracle_swiglu.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.oracle_argmax.restype = C.c_int
        L.oracle_argmax.argtypes = [C.c_void_p, C.c_int]
        L.oracle_model_new.restype = C.c_void_p
        L.oracle_model_new.argtypes = [C.POINTER(OracleConfig), C.POINTER(OracleWeights)]
        L.oracle_model_free.restype = None
        L.oracle_model_free.argtypes = [C.c_void_p]
        L.oracle_model_reset.restype = None
        L.oracle_model_reset.argtypes = [C.c_void_p]
        L.oracle_model_pos.restype = C.c_int
        L.oracle_model_pos.argtypes = [C.c_void_p]
        L.oracle_model_kv.restype = C.c_void_p
        L.oracle_model_kv.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.oracle_model_step.restype = C.c_int
        L.oracle_model_step.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]

    # ---- helpers -------------------------------------------------------
    def _r(self, a):
        return np.ascontiguousarray(a, dtype=self.real)

    @staticmethod
    def _w(a):
        """Weight array -> (contiguous array, dtype code)."""
        a = np.ascontiguousarray(a)
        if a.dtype == np.float16:
            return a, 1
        if a.dtype == np.float32:
            return a, 0
        raise TypeError("weights must be float32 or float16, got %s" % a.dtype)

    # ---- operators -----------------------------------------------------
    def half_to_float(self, bits):
        return float(self.lib.oracle_half_to_float(int(bits)))

    def rmsnorm(self, x, g, eps):
        x = self._r(x)
        g, dt = self._w(g)
        out = np.empty_like(x)
        self.lib.oracle_rmsnorm(_ptr(x), _ptr(g), dt, x.shape[0], eps, _ptr(out))
        return out

    def matvec(self, W, x):
        W, dt = self._w(W)
        x = self._r(x)
        assert W.ndim == 2 and W.shape[1] == x.shape[0]
        y = np.empty(W.shape[0], dtype=self.real)
        self.lib.oracle_matvec(_ptr(W), dt, W.shape[0], W.shape[1], _ptr(x), _ptr(y))
        return y

    def rope(self, vec, n_heads, head_dim, pos, theta):
        v = self._r(vec).copy()
        assert v.shape[0] == n_heads * head_dim
        self.lib.oracle_rope(_ptr(v), n_heads, head_dim, pos, theta)
        return v

    def attention_head(self, q, K, V):
        """q [dh], K/V [n_keys, dh] -> (o [dh], softmax weights [n_keys])."""
        q, K, V = self._r(q), self._r(K), self._r(V)
        n_keys, dh = K.shape
        o = np.empty(dh, dtype=self.real)
        w = np.empty(n_keys, dtype=self.real)
        self.lib.oracle_attention_head(_ptr(q), _ptr(K), _ptr(V), n_keys, dh, dh, _ptr(o), _ptr(w))
        return o, w

    def swiglu(self, g, u):
        g, u = self._r(g), self._r(u)
        m = np.empty_like(g)
        self.lib.oracle_swiglu(_ptr(g), _ptr(u), g.shape[0], _ptr(m))
        return m

    def argmax(self, v):
        v = self._r(v)
        return int(self.lib.oracle_argmax(_ptr(v), v.shape[0]))

    def model(self, cfg, weights):
        return OracleModel(self, cfg, weights)


class OracleModel:
    """Token-by-token decoder with a KV cache (``oracle_model_*`` in oracle.c)."""

    def __init__(self, oracle, cfg, weights):
        self.o = oracle
        self.cfg = dict(cfg)
        self._keep = []
        dts = set()

        def w(a):
            arr, dt = Oracle._w(a)
            self._keep.append(arr)
            dts.add(dt)
            return arr.ctypes.data

        n_layers = cfg["n_layers"]
        assert len(weights["layers"]) == n_layers
        self._layers = (OracleLayer * n_layers)()
        for i, L in enumerate(weights["layers"]):
            for k in _LAYER_KEYS:
                setattr(self._layers[i], k, w(L[k]))
        ow = OracleWeights()
        ow.tok_emb = w(weights["tok_emb"])
        ow.final_norm = w(weights["final_norm"])
        ow.lm_head = w(weights["lm_head"])
        ow.layers = C.cast(self._layers, C.POINTER(OracleLayer))
        assert len(dts) == 1, "all weights must share one dtype"
        ow.dtype = dts.pop()
        oc = OracleConfig(**{k: cfg[k] for k in ("n_layers", "d_model", "n_heads", "head_dim",
                                                 "ffn_hidden", "vocab", "max_seq")},
                          rope_theta=cfg["rope_theta"], rms_eps=cfg["rms_eps"])
        self._h = oracle.lib.oracle_model_new(C.byref(oc), C.byref(ow))
        if not self._h:
            raise ValueError("oracle_model_new rejected the configuration")

    def close(self):
        if self._h:
            self.o.lib.oracle_model_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self):
        self.o.lib.oracle_model_reset(self._h)

    @property
    def pos(self):
        return int(self.o.lib.oracle_model_pos(self._h))

    def step(self, token):
        """Feed one token at the next position -> (greedy next token, logits, hidden)."""
        logits = np.empty(self.cfg["vocab"], dtype=self.o.real)
        hidden = np.empty(self.cfg["d_model"], dtype=self.o.real)
        t = self.o.lib.oracle_model_step(self._h, int(token), _ptr(logits), _ptr(hidden))
        if t < 0:
            raise ValueError("oracle_model_step: bad token or cache full")
        return int(t), logits, hidden

    def prefill(self, tokens):
        """Feed the prompt token by token; result of the last call."""
        out = None
        for t in tokens:
            out = self.step(t)
        return out

    def kv(self, layer, which, n_pos=None):
        """Cached keys (which=0) or values (which=1) of one layer, [n_pos, d_model] copy."""
        n_pos = self.pos if n_pos is None else n_pos
        d = self.cfg["d_model"]
        p = self.o.lib.oracle_model_kv(self._h, layer, which)
        buf = (C.c_char * (n_pos * d * np.dtype(self.o.real).itemsize)).from_address(p)
        return np.frombuffer(buf, dtype=self.o.real).reshape(n_pos, d).copy()
