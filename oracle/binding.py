"""ctypes wrapper around sd_oracle.c (test infrastructure; argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sd_oracle.c")
_LIB = os.path.join(_HERE, "libsd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over output rows).  SD_ORACLE_LIB names a library to load
    instead: the test that plants mistakes points it at deliberately broken copies it has built."""
    override = os.environ.get("SD_ORACLE_LIB")
    if override:
        return override
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("d_model", C.c_int), ("n_heads", C.c_int), ("head_dim", C.c_int),
                ("d_ffn", C.c_int), ("vocab", C.c_int), ("dtype", C.c_int),
                ("rope_base", C.c_double), ("rms_eps", C.c_double)]


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        vp, ip, fp, dp = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_double)
        pp = C.POINTER(C.c_void_p)
        lib.orc_model_new.restype = vp
        lib.orc_model_new.argtypes = [C.POINTER(_Cfg), vp, vp, vp] + [pp] * 9
        lib.orc_model_free.argtypes = [vp]
        lib.orc_seq_new.restype = vp
        lib.orc_seq_new.argtypes = [vp, C.c_int]
        lib.orc_seq_free.argtypes = [vp]
        lib.orc_seq_len.argtypes = [vp]
        lib.orc_model_set_lora.argtypes = [vp, C.c_int, C.c_int, C.c_double] + [pp] * 8
        lib.orc_seq_set_adapter.argtypes = [vp, vp, C.c_int]
        lib.orc_seq_truncate.argtypes = [vp, C.c_int]
        lib.orc_seq_set_kv.argtypes = [vp, vp, C.c_int, vp, vp, C.c_int]
        lib.orc_forward.argtypes = [vp, vp, vp, C.c_int, vp, C.c_int]
        lib.orc_accept.argtypes = [C.c_int, C.c_int, C.c_double, vp, vp, vp, vp, vp, vp, vp]
        lib.orc_accept.restype = None
        lib.orc_draft.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_double, vp, vp, vp, vp]
        lib.orc_verify.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_double, vp, vp, vp, vp, vp, vp, vp]
        lib.orc_rmsnorm.argtypes = [vp, vp, C.c_int, C.c_double, vp]
        lib.orc_rmsnorm.restype = None
        lib.orc_rope.argtypes = [vp, C.c_int, C.c_int, C.c_double]
        lib.orc_rope.restype = None
        lib.orc_softmax_T.argtypes = [vp, C.c_int, C.c_double, vp]
        lib.orc_softmax_T.restype = None
        lib.orc_argmax.argtypes = [vp, C.c_int, vp]
        lib.orc_sample_cdf.argtypes = [vp, C.c_int, C.c_double, vp]
        lib.orc_route.argtypes = [vp, vp, C.c_int, C.c_int, vp, C.c_int, vp]
        lib.orc_route.restype = None
        lib.orc_next_weights.argtypes = [C.c_int, C.c_int, C.c_double, vp, vp, C.c_int, vp]
        lib.orc_next_weights.restype = None
        lib.orc_cdf_distance.argtypes = [vp, C.c_int, C.c_double, C.c_int]
        lib.orc_cdf_distance.restype = C.c_double
        lib.orc_round_bf16.argtypes = [C.c_float]
        lib.orc_round_bf16.restype = C.c_float
        _lib = lib
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


class OracleModel:
    """Borrowed weights (numpy arrays from datagen.make_weights) behind an orc_model."""

    def __init__(self, shape, weights: Dict[str, object]):
        lib = _load()
        self.shape = shape
        self._keep = weights
        cfg = _Cfg(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                   shape.dtype, shape.rope_base, shape.rms_eps)
        L = shape.n_layers

        def arr(name):
            lst = weights[name]
            for a in lst:
                assert a.flags["C_CONTIGUOUS"]
            return (C.c_void_p * L)(*[a.ctypes.data for a in lst])

        self._arrs = [arr(n) for n in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm_attn", "norm_ffn")]
        self.h = lib.orc_model_new(C.byref(cfg), _p(weights["embed"]), _p(weights["lm_head"]),
                                   _p(weights["final_norm"]), *self._arrs)

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.orc_model_free(self.h)
            self.h = None

    def set_lora(self, lora: Dict[str, object], scale: float) -> None:
        """Attach adapters from datagen.make_lora (arrays are borrowed): y = W x + scale * B_a (A_a x) on
        the q, k, v, o projections for sequences that choose adapter a."""
        L = self.shape.n_layers
        self._lora_keep = lora
        arrs = []
        for pnm in ("q", "k", "v", "o"):
            for ab in ("a_", "b_"):
                lst = lora.get(ab + pnm)
                if lst is None:
                    arrs.append(None)
                    continue
                for a in lst:
                    assert a.flags["C_CONTIGUOUS"]
                arrs.append((C.c_void_p * L)(*[a.ctypes.data for a in lst]))
        self._lora_arrs = arrs
        if _load().orc_model_set_lora(self.h, lora["n_adapters"], lora["rank"], float(scale), *arrs) != 0:
            raise ValueError("oracle set_lora failed")

    def new_seq(self, cap: int, adapter: int = -1) -> "OracleSeq":
        s = OracleSeq(self, cap)
        if adapter >= 0:
            s.set_adapter(adapter)
        return s


class OracleSeq:
    """One sequence's KV cache for one model."""

    def __init__(self, model: OracleModel, cap: int):
        self.model = model
        self.h = _load().orc_seq_new(model.h, cap)

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.orc_seq_free(self.h)
            self.h = None

    @property
    def len(self) -> int:
        return _load().orc_seq_len(self.h)

    def truncate(self, n: int) -> None:
        if _load().orc_seq_truncate(self.h, n) != 0:
            raise ValueError("truncate beyond length")

    def set_adapter(self, adapter: int) -> None:
        if _load().orc_seq_set_adapter(self.model.h, self.h, adapter) != 0:
            raise ValueError("adapter out of range")

    def set_kv(self, layer: int, k: np.ndarray, v: np.ndarray) -> None:
        k, v = np.ascontiguousarray(k), np.ascontiguousarray(v)
        if _load().orc_seq_set_kv(self.model.h, self.h, layer, _p(k), _p(v), k.shape[0]) != 0:
            raise ValueError("set_kv out of range")

    def forward(self, tokens: Sequence[int], logits_from: int = 0) -> np.ndarray:
        """Feed tokens, return fp32 logits of rows >= logits_from."""
        t = _i32(tokens)
        n = t.shape[0]
        V = self.model.shape.vocab
        out = np.empty((max(n - logits_from, 0), V), dtype=np.float32)
        rc = _load().orc_forward(self.model.h, self.h, _p(t), n, _p(out) if out.size else None, logits_from)
        if rc != 0:
            raise ValueError("oracle forward failed (capacity or token id)")
        return out

    def draft(self, ctx: Sequence[int], gamma: int, T: float, u: np.ndarray):
        """-> (cand[gamma], q[gamma][V] or None when greedy, margins[gamma])"""
        ctx = _i32(ctx)
        V = self.model.shape.vocab
        u = _f32(u)
        cand = np.empty(gamma, dtype=np.int32)
        q = np.zeros((gamma, V), dtype=np.float32) if T > 0 else None
        mg = np.empty(gamma, dtype=np.float64)
        rc = _load().orc_draft(self.model.h, self.h, _p(ctx), ctx.shape[0], gamma, float(T), _p(u), _p(cand),
                               _p(q), _p(mg))
        if rc != 0:
            raise ValueError("oracle draft failed")
        return cand, q, mg

    def verify(self, ctx: Sequence[int], gamma: int, T: float, cand, q, u, want_logits: bool = False):
        """-> (n_acc, next_token, margins[gamma+1], logits or None).  Does not commit:
        call truncate(len(ctx) + n_acc) afterwards."""
        ctx = _i32(ctx)
        V = self.model.shape.vocab
        cand = _i32(cand if gamma else np.zeros(0))
        u = _f32(u)
        qq = _f32(q) if (q is not None and T > 0 and gamma > 0) else None
        na, nx = C.c_int32(0), C.c_int32(0)
        mg = np.empty(gamma + 1, dtype=np.float64)
        lg = np.empty((gamma + 1, V), dtype=np.float32) if want_logits else None
        rc = _load().orc_verify(self.model.h, self.h, _p(ctx), ctx.shape[0], gamma, float(T), _p(cand), _p(qq),
                                _p(u), C.byref(na), C.byref(nx), _p(lg), _p(mg))
        if rc != 0:
            raise ValueError("oracle verify failed")
        return int(na.value), int(nx.value), mg, lg


def accept(logits: np.ndarray, q: Optional[np.ndarray], cand, u, T: float):
    """The acceptance rule alone -> (n_acc, next_token, margins[gamma+1])."""
    logits = _f32(logits)
    gamma = logits.shape[0] - 1
    V = logits.shape[1]
    cand = _i32(cand)
    u = _f32(u)
    qq = _f32(q) if (q is not None and gamma > 0) else None
    na, nx = C.c_int32(0), C.c_int32(0)
    mg = np.empty(gamma + 1, dtype=np.float64)
    _load().orc_accept(V, gamma, float(T), _p(logits), _p(qq), _p(cand), _p(u), C.byref(na), C.byref(nx), _p(mg))
    return int(na.value), int(nx.value), mg


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = _f32(g)
    out = np.empty_like(x)
    _load().orc_rmsnorm(_p(x), _p(g), x.shape[0], float(eps), _p(out))
    return out


def rope(x: np.ndarray, pos: int, base: float) -> np.ndarray:
    x = np.array(x, dtype=np.float64, order="C")
    _load().orc_rope(_p(x), x.shape[0], int(pos), float(base))
    return x


def softmax_T(logits: np.ndarray, T: float) -> np.ndarray:
    logits = _f32(logits)
    p = np.empty_like(logits)
    _load().orc_softmax_T(_p(logits), logits.shape[0], float(T), _p(p))
    return p


def argmax(x: np.ndarray):
    x = _f32(x)
    gap = C.c_double(0)
    k = _load().orc_argmax(_p(x), x.shape[0], C.byref(gap))
    return int(k), gap.value


def sample_cdf(w: np.ndarray, u: float):
    w = np.ascontiguousarray(w, dtype=np.float64)
    mg = C.c_double(0)
    k = _load().orc_sample_cdf(_p(w), w.shape[0], float(u), C.byref(mg))
    return int(k), mg.value


def route(W: np.ndarray, b: Optional[np.ndarray], emb: np.ndarray) -> np.ndarray:
    W, emb = _f32(W), _f32(emb)
    bb = _f32(b) if b is not None else None
    out = np.empty(emb.shape[0], dtype=np.int32)
    _load().orc_route(_p(W), _p(bb), W.shape[0], W.shape[1], _p(emb), emb.shape[0], _p(out))
    return out


def round_bf16(x: float) -> float:
    return float(_load().orc_round_bf16(float(x)))


def next_weights(logits: np.ndarray, q: Optional[np.ndarray], n_acc: int, T: float) -> np.ndarray:
    """Weights the next token is drawn from after n_acc accepted candidates (T > 0)."""
    logits = _f32(logits)
    gamma, V = logits.shape[0] - 1, logits.shape[1]
    qq = _f32(q) if (q is not None and gamma > 0) else None
    w = np.empty(V, dtype=np.float64)
    _load().orc_next_weights(V, gamma, float(T), _p(logits), _p(qq), int(n_acc), _p(w))
    return w


def cdf_distance(w: np.ndarray, u: float, k: int) -> float:
    """Distance of u from token k's inverse-CDF interval, as a fraction of the mass."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    return float(_load().orc_cdf_distance(_p(w), w.shape[0], float(u), int(k)))
