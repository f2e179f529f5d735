"""Thin Python binding of libsd (include/sd.h): argument marshalling only.

PyTorch is used for device memory and streams; every step of the draft/verify
path runs in the HIP kernels of libsd.so.  There is no fallback: if the library
is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsd.so")
_lib = None

SD_OK, SD_EINVAL, SD_ECAP, SD_EHIP, SD_ESTATE = 0, -1, -2, -3, -4
SD_FP32, SD_BF16 = 0, 1

EXPORTS = ["sd_load_model", "sd_free_model", "sd_ctx_create", "sd_ctx_free", "sd_ctx_attach", "sd_ctx_set_tokens",
           "sd_prefill", "sd_draft", "sd_verify", "sd_commit", "sd_route", "sd_ctx_sync", "sd_ctx_get_tokens",
           "sd_ctx_set_kv", "sd_ctx_truncate", "sd_debug_read", "sd_debug_layout_index", "sd_last_logits", "sd_set_option", "sd_profile_read", "sd_last_error",
           "sd_eq1_speedup", "sd_choose_gamma", "sd_alpha_hat", "sd_model_set_lora", "sd_ctx_set_adapters",
           "sd_classifier_create", "sd_classifier_destroy", "sd_route_classifier", "sd_accept",
           "sd_accept_static", "sd_debug_stream_read", "sd_debug_gemm_plan",
           "sd_policy_set", "sd_policy_choose", "sd_policy_read"]


class SdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libsd error {code}: {msg}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("dtype", C.c_int32), ("rope_base", C.c_float),
                ("rms_eps", C.c_float), ("max_rows", C.c_int32), ("max_pos", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown",
                                                     "norm_attn", "norm_ffn")]


class _LoraW(C.Structure):
    _fields_ = [("n_adapters", C.c_int32), ("rank", C.c_int32), ("scale", C.c_float)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("a_q", "b_q", "a_k", "b_k", "a_v", "b_v", "a_o", "b_o")]


CLASSIFIER_WEIGHTS = ("emb", "w_in", "conv_w", "conv_b", "w_x", "w_dt", "b_dt", "a_log", "d", "w_out", "w_fc", "b_fc")


class _ClsShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("vocab", "d_model", "d_inner", "d_state", "dt_rank", "d_conv", "n_classes")]


class _ClsWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in CLASSIFIER_WEIGHTS]


def lib():
    """Load libsd.so (built in-tree by paper_2505_08600_amd.build); never falls back."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_08600_amd.build` "
                              "(there is no CPU fallback for the draft/verify path)")
        L = C.CDLL(LIB_PATH)
        vp, i32 = C.c_void_p, C.c_int32
        L.sd_load_model.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(vp)]
        L.sd_free_model.argtypes = [vp]
        L.sd_ctx_create.argtypes = [i32, vp, C.POINTER(vp)]
        L.sd_ctx_free.argtypes = [vp]
        L.sd_ctx_attach.argtypes = [vp, vp]
        L.sd_ctx_set_tokens.argtypes = [vp, vp, vp, vp, i32]
        L.sd_prefill.argtypes = [vp, vp, vp, i32, i32, vp]
        L.sd_draft.argtypes = [vp, vp, vp, i32, i32, C.c_float, vp, vp, vp, vp]
        L.sd_verify.argtypes = [vp, vp, vp, i32, i32, C.c_float, vp, vp, vp, vp, vp, i32, vp]
        L.sd_commit.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp]
        L.sd_accept.argtypes = [vp, i32, i32, i32, C.c_float, vp, vp, vp, vp, vp, vp, vp]
        L.sd_policy_set.argtypes = [vp, vp]
        L.sd_policy_choose.argtypes = [vp, vp, i32, C.c_double, i32, C.c_double, vp, vp]
        L.sd_policy_read.argtypes = [vp, vp, vp, vp]
        L.sd_debug_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.sd_accept_static.argtypes = [vp, i32, i32, i32, C.c_float, vp, vp, vp, vp, vp, vp]
        L.sd_route.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp]
        L.sd_ctx_sync.argtypes = [vp, vp, vp, vp]
        L.sd_ctx_get_tokens.argtypes = [vp, i32, vp, i32, C.POINTER(i32)]
        L.sd_ctx_set_kv.argtypes = [vp, vp, i32, i32, vp, vp, i32]
        L.sd_ctx_truncate.argtypes = [vp, vp, i32, i32]
        L.sd_debug_read.argtypes = [vp, C.c_char_p, vp, i32]
        L.sd_debug_gemm_plan.argtypes = [i32, i32, i32, i32, i32, C.POINTER(C.c_int32)]
        L.sd_debug_layout_index.argtypes = [i32, C.c_int64, C.c_int64, C.c_int64, C.c_int64]
        L.sd_debug_layout_index.restype = C.c_int64
        L.sd_last_logits.argtypes = [vp, vp, i32, C.POINTER(i32)]
        L.sd_set_option.argtypes = [C.c_char_p, i32]
        L.sd_profile_read.argtypes = [i32, C.POINTER(C.c_char_p), C.POINTER(i32), C.POINTER(C.c_float)]
        L.sd_last_error.restype = C.c_char_p
        L.sd_model_set_lora.argtypes = [vp, C.POINTER(_LoraW)]
        L.sd_ctx_set_adapters.argtypes = [vp, vp, vp]
        L.sd_classifier_create.argtypes = [C.POINTER(_ClsShape), C.POINTER(_ClsWeights), C.POINTER(vp)]
        L.sd_classifier_destroy.argtypes = [vp]
        L.sd_classifier_destroy.restype = None
        L.sd_route_classifier.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
        L.sd_eq1_speedup.argtypes = [C.c_double, i32, C.c_double]
        L.sd_eq1_speedup.restype = C.c_double
        L.sd_choose_gamma.argtypes = [C.c_double, C.c_double, i32, C.POINTER(C.c_double)]
        L.sd_choose_gamma.restype = i32
        L.sd_alpha_hat.argtypes = [vp, i32, i32]
        L.sd_alpha_hat.restype = C.c_double
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != SD_OK:
        raise SdError(rc, lib().sd_last_error().decode())


def _dp(t: Optional[torch.Tensor]):
    """Device pointer of a contiguous tensor (None -> NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _np_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def set_option(name: str, value: int) -> None:
    _check(lib().sd_set_option(name.encode(), int(value)))


def profile_read() -> Dict[str, tuple]:
    """{kernel class: (launches, total ms)} gathered under set_option("profile", 1)."""
    out = {}
    i = 0
    while True:
        name, cnt, ms = C.c_char_p(), C.c_int32(), C.c_float()
        if lib().sd_profile_read(i, C.byref(name), C.byref(cnt), C.byref(ms)) != SD_OK:
            break
        out[name.value.decode()] = (cnt.value, ms.value)
        i += 1
    return out


def to_device(a: np.ndarray, device="cuda") -> torch.Tensor:
    """Upload a numpy array; uint16 bf16 bit patterns travel as int16."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


class Model:
    """sd_load_model / sd_free_model.  The library copies the weights at load, so the staging
    tensors are released right after."""

    def __init__(self, shape, weights: Dict[str, object], max_rows: int, max_pos: int, device="cuda"):
        self.shape = shape
        self.device = device
        self.t: Dict[str, object] = {}
        for k, v in weights.items():
            self.t[k] = [to_device(a, device) for a in v] if isinstance(v, list) else to_device(v, device)
        L = shape.n_layers
        self._arrs = {}
        w = _Weights()
        w.embed, w.lm_head, w.final_norm = (self.t[n].data_ptr() for n in ("embed", "lm_head", "final_norm"))
        for n in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "norm_attn", "norm_ffn"):
            arr = (C.c_void_p * L)(*[t.data_ptr() for t in self.t[n]])
            self._arrs[n] = arr
            setattr(w, n, C.cast(arr, C.POINTER(C.c_void_p)))
        cfg = _Config(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                      shape.dtype, shape.rope_base, shape.rms_eps, max_rows, max_pos)
        self.max_rows = max_rows
        h = C.c_void_p()
        with torch.cuda.device(device):
            _check(lib().sd_load_model(C.byref(cfg), C.byref(w), C.byref(h)))
        self.h = h
        self.t.clear()
        self._arrs.clear()

    def set_lora(self, lora: Dict[str, object], scale: float) -> None:
        """sd_model_set_lora: adapters from datagen.make_lora (host numpy arrays; the library copies them)."""
        L = self.shape.n_layers
        w = _LoraW()
        w.n_adapters, w.rank, w.scale = lora["n_adapters"], lora["rank"], float(scale)
        keep = []
        for pnm in ("q", "k", "v", "o"):
            for ab in ("a_", "b_"):
                lst = lora.get(ab + pnm)
                if lst is None:
                    continue
                arrs = [np.ascontiguousarray(a) for a in lst]
                ptrs = (C.c_void_p * L)(*[a.ctypes.data for a in arrs])
                keep.append((arrs, ptrs))
                setattr(w, ab + pnm, C.cast(ptrs, C.POINTER(C.c_void_p)))
        with torch.cuda.device(self.device):
            _check(lib().sd_model_set_lora(self.h, C.byref(w)))

    def close(self):
        if getattr(self, "h", None):
            lib().sd_free_model(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def debug_read(self, name: str, rows: int) -> np.ndarray:
        """Host copy (fp32) of a workspace buffer of the last forward: x, qkv, q, o, a, act; or, with
        rows = number of sequences, the last plan's seq_order / seq_len as one column."""
        width = {"x": self.shape.d_model, "qkv": 3 * self.shape.d_model, "act": self.shape.d_ffn,
                 "seq_order": 1, "seq_len": 1}.get(name, self.shape.d_model)
        out = np.empty((rows, width), np.float32)
        _check(lib().sd_debug_read(self.h, name.encode(), out.ctypes.data_as(C.c_void_p), rows))
        return out

    def last_logits(self) -> torch.Tensor:
        """Copy of the fp32 logits [rows][vocab] of the last forward (synchronises)."""
        out = torch.empty((self.max_rows, self.shape.vocab), dtype=torch.float32, device=self.device)
        rows = C.c_int32()
        _check(lib().sd_last_logits(self.h, _dp(out), self.max_rows, C.byref(rows)))
        return out[:rows.value]


class Context:
    """sd_ctx_*: B sequences with per-sequence capacities."""

    def __init__(self, caps: Sequence[int]):
        self.caps = _np_i32(caps)
        self.B = len(self.caps)
        h = C.c_void_p()
        _check(lib().sd_ctx_create(self.B, self.caps.ctypes.data_as(C.c_void_p), C.byref(h)))
        self.h = h
        self._models: List[Model] = []

    def close(self):
        if getattr(self, "h", None):
            lib().sd_ctx_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def attach(self, m: Model) -> None:
        _check(lib().sd_ctx_attach(self.h, m.h))
        self._models.append(m)

    def set_tokens(self, seqs: Sequence[Sequence[int]], seq_ids: Optional[Sequence[int]] = None) -> None:
        lens = _np_i32([len(s) for s in seqs])
        flat = _np_i32(np.concatenate([np.asarray(s, dtype=np.int32) for s in seqs]))
        ids = _np_i32(seq_ids) if seq_ids is not None else None
        _check(lib().sd_ctx_set_tokens(self.h, flat.ctypes.data_as(C.c_void_p), lens.ctypes.data_as(C.c_void_p),
                                       ids.ctypes.data_as(C.c_void_p) if ids is not None else None, len(seqs)))

    def sync(self, m: Optional[Model] = None):
        """-> (n_tokens[B], kv_len[B] or None); raises SdError(SD_ESTATE) on a device flag."""
        nt = np.zeros(self.B, np.int32)
        kv = np.zeros(self.B, np.int32) if m is not None else None
        _check(lib().sd_ctx_sync(self.h, m.h if m is not None else None, nt.ctypes.data_as(C.c_void_p),
                                 kv.ctypes.data_as(C.c_void_p) if kv is not None else None))
        return nt, kv

    def get_tokens(self, seq: int) -> np.ndarray:
        out = np.zeros(int(self.caps[seq]) + 64, np.int32)
        n = C.c_int32()
        _check(lib().sd_ctx_get_tokens(self.h, seq, out.ctypes.data_as(C.c_void_p), out.shape[0], C.byref(n)))
        return out[:n.value].copy()

    def set_adapters(self, m: Model, adapter_ids: Sequence[int]) -> None:
        """sd_ctx_set_adapters: the low-rank adapter of every sequence for model m (-1: none)."""
        a = _np_i32(adapter_ids)
        assert len(a) == self.B
        _check(lib().sd_ctx_set_adapters(self.h, m.h, a.ctypes.data_as(C.c_void_p)))

    def policy_set(self, gammas: Optional[Sequence[int]]) -> None:
        """sd_policy_set: candidate count per sequence (None: off)."""
        if gammas is None:
            _check(lib().sd_policy_set(self.h, None))
            return
        g = _np_i32(gammas)
        assert len(g) == self.B
        _check(lib().sd_policy_set(self.h, g.ctypes.data_as(C.c_void_p)))

    def policy_choose(self, seq_ids: Optional[torch.Tensor], n_seq: int, c_ratio: float, gamma_max: int, alpha0: float,
                      gammas_out: Optional[torch.Tensor] = None) -> None:
        """sd_policy_choose: counts from Equation 1 and the running acceptance estimate, on the device."""
        _check(lib().sd_policy_choose(self.h, _dp(seq_ids), n_seq, c_ratio, gamma_max, alpha0, _dp(gammas_out), _stream()))

    def policy_read(self):
        """-> (per-sequence counts on?, gammas[B], accepted[B], examined[B])"""
        g, a, e = (np.zeros(self.B, np.int32) for _ in range(3))
        rc = lib().sd_policy_read(self.h, g.ctypes.data_as(C.c_void_p), a.ctypes.data_as(C.c_void_p),
                                  e.ctypes.data_as(C.c_void_p))
        if rc < 0:
            _check(rc)
        return bool(rc), g, a, e

    def truncate(self, m: Model, seq: int, length: int) -> None:
        _check(lib().sd_ctx_truncate(self.h, m.h, seq, length))

    def set_kv(self, m: Model, layer: int, seq: int, k, v) -> None:
        """k, v: [len][n_heads][head_dim] numpy arrays (host) or contiguous torch tensors (device)."""
        if isinstance(k, torch.Tensor):
            assert k.is_contiguous() and v.is_contiguous()
            _check(lib().sd_ctx_set_kv(self.h, m.h, layer, seq, _dp(k), _dp(v), k.shape[0]))
            return
        k, v = np.ascontiguousarray(k), np.ascontiguousarray(v)
        _check(lib().sd_ctx_set_kv(self.h, m.h, layer, seq, k.ctypes.data_as(C.c_void_p),
                                   v.ctypes.data_as(C.c_void_p), k.shape[0]))


def gemm_plan(mode: int, m: int, n: int, k: int, n_per_seg: Optional[int] = None):
    """sd_debug_gemm_plan -> (weight rows per block, rows per block, column tiles, row blocks, K splits, blocks on the
    busiest die), or None when the row-blocked kernel does not take the shape."""
    plan = (C.c_int32 * 6)()
    if lib().sd_debug_gemm_plan(mode, m, n, k, n if n_per_seg is None else n_per_seg, plan) != SD_OK:
        return None
    return tuple(int(x) for x in plan)


def layout_index(kind: int, a: int, b: int, c: int, d: int = 0) -> int:
    """sd_debug_layout_index: 0 tiled weight (n, k, K), 1 step-major activation (m, k, K, rows), 2 value cache / 3 key cache (t, dim, head_dim)."""
    return int(lib().sd_debug_layout_index(kind, a, b, c, d))


def sd_prefill(m: Model, ctx: Context, seq_ids: Optional[torch.Tensor], n_seq: int, max_new: int) -> None:
    _check(lib().sd_prefill(m.h, ctx.h, _dp(seq_ids), n_seq, max_new, _stream()))


def sd_draft(draft: Model, ctx: Context, seq_ids: Optional[torch.Tensor], n_seq: int, gamma: int,
             temperature: float, uniforms: Optional[torch.Tensor], cand: torch.Tensor,
             q: Optional[torch.Tensor]) -> None:
    _check(lib().sd_draft(draft.h, ctx.h, _dp(seq_ids), n_seq, gamma, temperature, _dp(uniforms), _dp(cand), _dp(q),
                          _stream()))


def sd_verify(target: Model, ctx: Context, seq_ids: Optional[torch.Tensor], n_seq: int, gamma: int,
              temperature: float, cand: Optional[torch.Tensor], q: Optional[torch.Tensor],
              uniforms: Optional[torch.Tensor], n_accepted: torch.Tensor, next_token: torch.Tensor,
              commit: bool = True) -> None:
    _check(lib().sd_verify(target.h, ctx.h, _dp(seq_ids), n_seq, gamma, temperature, _dp(cand), _dp(q),
                           _dp(uniforms), _dp(n_accepted), _dp(next_token), int(commit), _stream()))


def sd_accept(logits: torch.Tensor, gamma: int, temperature: float, cand: Optional[torch.Tensor],
              q: Optional[torch.Tensor], uniforms: Optional[torch.Tensor], n_accepted: torch.Tensor,
              next_token: torch.Tensor, workspace: torch.Tensor) -> None:
    """sd_accept: logits [n_seq][gamma+1][vocab]; workspace fp32 [3 * n_seq * (gamma+1)]."""
    n_seq, rows, vocab = logits.shape
    assert rows == gamma + 1 and workspace.numel() >= 3 * n_seq * rows and workspace.dtype == torch.float32
    _check(lib().sd_accept(_dp(logits), n_seq, gamma, vocab, temperature, _dp(cand), _dp(q), _dp(uniforms),
                           _dp(n_accepted), _dp(next_token), _dp(workspace), _stream()))


def sd_accept_static(logits: torch.Tensor, gamma: int, temperature: float, cand: Optional[torch.Tensor],
                     q: Optional[torch.Tensor], uniforms: Optional[torch.Tensor], n_accepted: torch.Tensor,
                     next_token: torch.Tensor) -> None:
    """sd_accept_static: sd_accept without a workspace argument and without any allocation."""
    n_seq, rows, vocab = logits.shape
    assert rows == gamma + 1
    _check(lib().sd_accept_static(_dp(logits), n_seq, gamma, vocab, temperature, _dp(cand), _dp(q), _dp(uniforms),
                                  _dp(n_accepted), _dp(next_token), _stream()))


def stream_read(buf: torch.Tensor, scratch: torch.Tensor) -> None:
    """sd_debug_stream_read: one plain read of the whole buffer on the current stream."""
    _check(lib().sd_debug_stream_read(_dp(buf), buf.numel() * buf.element_size(), _dp(scratch), _stream()))


def sd_commit(ctx: Context, seq_ids: Optional[torch.Tensor], n_seq: int, gamma: int, cand: Optional[torch.Tensor],
              n_accepted: torch.Tensor, next_token: torch.Tensor) -> None:
    _check(lib().sd_commit(ctx.h, _dp(seq_ids), n_seq, gamma, _dp(cand), _dp(n_accepted), _dp(next_token),
                           _stream()))


def eq1_speedup(alpha: float, gamma: int, c: float) -> float:
    """sd_eq1_speedup: Equation 1 (host only)."""
    return float(lib().sd_eq1_speedup(alpha, gamma, c))


def choose_gamma(alpha: float, c: float, gamma_max: int = 15):
    """sd_choose_gamma: (gamma maximising Equation 1, that maximum)."""
    v = C.c_double()
    g = lib().sd_choose_gamma(alpha, c, gamma_max, C.byref(v))
    if g < 0:
        raise SdError(SD_EINVAL, lib().sd_last_error().decode())
    return int(g), float(v.value)


def alpha_hat(n_accepted: Sequence[int], gamma: int) -> float:
    """sd_alpha_hat: accepted over examined candidates (host only)."""
    a = _np_i32(n_accepted)
    return float(lib().sd_alpha_hat(a.ctypes.data_as(C.c_void_p), len(a), gamma))


class Classifier:
    """sd_classifier: the prompt classifier of Sections 2.4 and 3.3.3 on one device."""

    def __init__(self, shape, weights: Dict[str, np.ndarray], device: int = 0):
        self.shape, self.device = shape, device
        s = _ClsShape(*[getattr(shape, n) for n, _ in _ClsShape._fields_])
        arrs = {n: np.ascontiguousarray(weights[n], dtype=np.float32) for n in CLASSIFIER_WEIGHTS}
        w = _ClsWeights(*[arrs[n].ctypes.data for n in CLASSIFIER_WEIGHTS])
        h = C.c_void_p()
        with torch.cuda.device(device):
            _check(lib().sd_classifier_create(C.byref(s), C.byref(w), C.byref(h)))
        self.h = h

    def route(self, tokens: torch.Tensor, lens: torch.Tensor, draft_id: torch.Tensor,
              logits: Optional[torch.Tensor] = None) -> None:
        """sd_route_classifier on the current stream; tokens int32 [n][max_len], lens int32 [n]."""
        with torch.cuda.device(self.device):
            _check(lib().sd_route_classifier(self.h, _dp(tokens), _dp(lens), tokens.shape[0], tokens.shape[1],
                                             _dp(logits), _dp(draft_id), _stream()))

    def close(self):
        if getattr(self, "h", None):
            lib().sd_classifier_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def sd_route(W: torch.Tensor, b: Optional[torch.Tensor], prompt_emb: torch.Tensor, draft_id: torch.Tensor) -> None:
    _check(lib().sd_route(_dp(W), _dp(b), W.shape[0], W.shape[1], _dp(prompt_emb), prompt_emb.shape[0],
                          _dp(draft_id), _stream()))
