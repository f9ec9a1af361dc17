"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE, not product).

Only tests/, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It neither imports nor is imported by
the HIP library's package.

The arithmetic lives in ``edgefm_oracle.c`` (plain C, fp64); this file only
marshals numpy arrays.  ``build()`` compiles the C file with gcc.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "edgefm_oracle.c")
_LIBS = {"f64": os.path.join(_DIR, "liboracle_f64.so"), "f32": os.path.join(_DIR, "liboracle_f32.so")}


def build(force: bool = False) -> None:
    """Compile the oracle: the fp64 library (the oracle proper) and an fp32 build of the same source
    (used by one test that measures the sensitivity to evaluation precision)."""
    for kind, path in _LIBS.items():
        if not force and os.path.exists(path) and os.path.getmtime(path) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", path, _SRC, "-lm"]
        if kind == "f32":
            cmd.insert(1, "-DORACLE_REAL=float")
        subprocess.run(cmd, check=True)


class _Config(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim",
                                           "intermediate", "vocab", "max_seq_len")] + \
               [("rms_eps", C.c_double), ("rope_theta", C.c_double)] + \
               [(n, C.c_uint32) for n in ("weight_dtype", "kv_dtype", "tie_embeddings", "qkv_bias", "kv_round")]


_PP = C.POINTER(C.c_void_p)


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, _PP) for n in ("attn_norm", "wqkv", "bqkv", "wo", "mlp_norm", "w_gate_up", "w_down")]


_loaded = {}


def _lib(kind: str = "f64"):
    if kind not in _loaded:
        build()
        lib = C.CDLL(_LIBS[kind])
        lib.oracle_create.restype = C.c_void_p
        lib.oracle_create.argtypes = [C.POINTER(_Config), C.POINTER(_Weights)]
        lib.oracle_destroy.argtypes = [C.c_void_p]
        lib.oracle_kv_len.restype = C.c_uint32
        lib.oracle_kv_len.argtypes = [C.c_void_p]
        lib.oracle_kv_reset.argtypes = [C.c_void_p, C.c_uint32]
        lib.oracle_kv_set_len.argtypes = [C.c_void_p, C.c_uint32]
        lib.oracle_kv_read.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        lib.oracle_kv_write.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
        lib.oracle_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32,
                                       C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        lib.oracle_round_kv.restype = C.c_double
        lib.oracle_round_kv.argtypes = [C.c_double, C.c_uint32]
        lib.oracle_upcast.restype = C.c_double
        lib.oracle_upcast.argtypes = [C.c_uint16, C.c_uint32]
        lib.oracle_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_double, C.c_void_p]
        lib.oracle_matvec.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32,
                                      C.c_void_p, C.c_void_p]
        lib.oracle_rope.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_double, C.c_void_p]
        lib.oracle_attend.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_size_t,
                                      C.c_void_p, C.c_void_p]
        lib.oracle_swiglu.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]
        lib.oracle_argmax.restype = C.c_int32
        lib.oracle_argmax.argtypes = [C.c_void_p, C.c_uint32]
        lib.oracle_real_bytes.restype = C.c_int
        lib.oracle_num_threads.restype = C.c_int
        _loaded[kind] = lib
    return _loaded[kind]


def num_threads() -> int:
    """Threads the oracle's OpenMP loops use on this host."""
    return _lib().oracle_num_threads()


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16
    return a


class Ops:
    """The oracle's operators, one call each, on numpy arrays (used by the pin tests)."""

    def __init__(self, kind: str = "f64"):
        self.lib = _lib(kind)
        self.real = np.float64 if kind == "f64" else np.float32
        assert self.lib.oracle_real_bytes() == np.dtype(self.real).itemsize

    def _r(self, a):
        return np.ascontiguousarray(a, dtype=self.real)

    def round_kv(self, x: float, dtype: int) -> float:
        return self.lib.oracle_round_kv(float(x), dtype)

    def upcast(self, bits: int, dtype: int) -> float:
        return self.lib.oracle_upcast(int(bits), dtype)

    def rmsnorm(self, x, gain_bits, dtype, eps):
        x = self._r(x); g = _u16(gain_bits); y = np.empty_like(x)
        self.lib.oracle_rmsnorm(_p(x), _p(g), dtype, x.size, eps, _p(y))
        return y

    def matvec(self, W_bits, bias_bits, dtype, a):
        W = _u16(W_bits); a = self._r(a); b = None if bias_bits is None else _u16(bias_bits)
        y = np.empty(W.shape[0], dtype=self.real)
        self.lib.oracle_matvec(_p(W), _p(b), dtype, W.shape[0], W.shape[1], _p(a), _p(y))
        return y

    def rope(self, x, pos, theta):
        x = self._r(x); y = np.empty_like(x)
        self.lib.oracle_rope(_p(x), x.size, pos, theta, _p(y))
        return y

    def attend(self, q, K, V):
        q = self._r(q); K = self._r(K); V = self._r(V)
        n, d = K.shape
        o = np.empty(d, dtype=self.real); probs = np.empty(n, dtype=self.real)
        self.lib.oracle_attend(_p(q), _p(K), _p(V), n, d, d, _p(o), _p(probs))
        return o, probs

    def swiglu(self, gate, up):
        gate = self._r(gate); up = self._r(up); h = np.empty_like(gate)
        self.lib.oracle_swiglu(_p(gate), _p(up), gate.size, _p(h))
        return h

    def argmax(self, x):
        x = self._r(x)
        return self.lib.oracle_argmax(_p(x), x.size)


class OracleModel:
    """One decoder instance with its own KV cache: the paper's Eq. 3 (prefill) and Eq. 4 (decode step)."""

    def __init__(self, shape, weights: dict, max_seq_len: int | None = None, kv_round: bool = True,
                 n_layers: int | None = None, kind: str = "f64"):
        self.lib = _lib(kind)
        self.real = np.float64 if kind == "f64" else np.float32
        self.shape = shape
        L = len(weights["layers"]) if n_layers is None else n_layers
        self.n_layers = L
        self.max_seq_len = shape.max_seq_len if max_seq_len is None else max_seq_len
        cfg = _Config(L, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.intermediate,
                      shape.vocab, self.max_seq_len, shape.rms_eps, shape.rope_theta, shape.weight_dtype,
                      shape.kv_dtype, int(shape.tie_embeddings), int(shape.qkv_bias), int(kv_round))
        self._keep = [weights]  # the C side borrows the arrays

        def table(key):
            arr = (C.c_void_p * L)()
            for l in range(L):
                t = weights["layers"][l][key]
                arr[l] = None if t is None else _u16(t).ctypes.data
            self._keep.append(arr)
            return C.cast(arr, _PP)

        for l in range(L):
            for k, t in weights["layers"][l].items():
                assert t is None or (t.flags["C_CONTIGUOUS"] and t.dtype == np.uint16), k
        w = _Weights(_u16(weights["embed"]).ctypes.data,
                     None if weights["lm_head"] is None else _u16(weights["lm_head"]).ctypes.data,
                     _u16(weights["final_norm"]).ctypes.data,
                     table("attn_norm"), table("wqkv"), table("bqkv"), table("wo"), table("mlp_norm"),
                     table("w_gate_up"), table("w_down"))
        self.h = self.lib.oracle_create(C.byref(cfg), C.byref(w))
        if not self.h:
            raise ValueError("oracle_create rejected the configuration")

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.oracle_destroy(self.h)
            self.h = None

    @property
    def kv_len(self) -> int:
        return self.lib.oracle_kv_len(self.h)

    def kv_reset(self, keep_len: int = 0) -> None:
        if self.lib.oracle_kv_reset(self.h, keep_len):
            raise ValueError("keep_len exceeds kv_len")

    def kv_read(self, layer: int, pos: int):
        n = self.shape.kv_dim
        k = np.empty(n, dtype=self.real); v = np.empty(n, dtype=self.real)
        if self.lib.oracle_kv_read(self.h, layer, pos, _p(k), _p(v)):
            raise IndexError((layer, pos))
        return k, v

    def kv_inject(self, rows_per_layer) -> None:
        """rows_per_layer[l] = (k_bits, v_bits), each [n_pos, n_kv*d]; positions 0..n_pos-1 become valid."""
        n_pos = None
        for l, (k, v) in enumerate(rows_per_layer):
            k = _u16(k); v = _u16(v)
            n_pos = k.shape[0]
            if self.lib.oracle_kv_write(self.h, l, n_pos, _p(k), _p(v)):
                raise ValueError("kv_write")
        self.lib.oracle_kv_set_len(self.h, n_pos)

    def forward(self, tokens=None, embeds=None, logits: str = "last", want_hidden: bool = True):
        """Append the embedding rows, then the tokens, to the context.

        Returns dict(hidden [n,H] final-norm outputs, logits ([V] or [n,V]), next (argmax))."""
        tokens = np.zeros(0, np.int32) if tokens is None else np.ascontiguousarray(tokens, dtype=np.int32)
        n_emb = 0 if embeds is None else embeds.shape[0]
        emb = None if embeds is None else _u16(embeds)
        n = n_emb + tokens.size
        H, V = self.shape.hidden, self.shape.vocab
        hidden = np.empty((n, H), dtype=self.real) if want_hidden else None
        mode = {"none": 0, "last": 1, "all": 2}[logits]
        lg = None if mode == 0 else np.empty(V if mode == 1 else (n, V), dtype=self.real)
        nxt = None if mode == 0 else np.empty(1 if mode == 1 else n, dtype=np.int32)
        rc = self.lib.oracle_forward(self.h, _p(emb), n_emb, _p(tokens), tokens.size, _p(hidden), mode,
                                     _p(lg), _p(nxt))
        if rc:
            raise ValueError({-1: "bad argument", -2: "context overflow", -3: "bad token id"}.get(rc, rc))
        return {"hidden": hidden, "logits": lg, "next": nxt}

    def prefill(self, tokens=None, embeds=None, **kw):
        return self.forward(tokens, embeds, **kw)

    def decode_step(self, token: int, **kw):
        return self.forward(np.array([token], dtype=np.int32), None, **kw)


def restricted_argmax(logits, subset):
    """Greedy choice under vocabulary pruning: the candidate with the largest logit, the lowest token id on
    ties.  `subset` holds ascending token ids.  Returns (token id, logits of the candidates in subset order).
    The paper names vocabulary pruning (Section 3.2) without defining it; this is the definition the library
    documents: the forward pass is unchanged and only the output distribution is restricted."""
    logits = np.asarray(logits)
    subset = np.asarray(subset, dtype=np.int64)
    cand = logits[subset]
    best = None
    for tok, val in zip(subset.tolist(), cand.tolist()):  # plain scan: first maximum wins
        if best is None or val > best[1]:
            best = (tok, val)
    return best[0], cand
