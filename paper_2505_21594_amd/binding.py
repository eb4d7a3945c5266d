"""Thin ctypes binding over libeeverify.so: argument marshalling only.

Every step of the verification pass runs in the library's HIP kernels; this
module never computes anything itself and has no CPU fallback: if the shared
library is missing or does not load, importing the names below raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

EE_MAX_M = 16
EE_MAX_EXITS = 40
EE_MAX_BATCH = 16
EE_MAX_ROWS = 48

EE_OK, EE_NOT_READY, EE_DONE = 0, 1, 2
EE_EINVAL, EE_ESTATE, EE_ECAPACITY, EE_EIO, EE_EFORMAT, EE_EDEVICE = -1, -2, -3, -4, -5, -6

HOLD_LAST = 1
KEEP_LOGITS = 1
NO_AUTOCOMMIT = 2
SAMPLING = 4
TIME_LAUNCHES = 16
OPT_ATT_SPLITS, OPT_SCATTER_PAGES, OPT_HEAD_BATCH = 1, 2, 3
LAUNCH_NAMES = ("qkv", "o", "gu", "dn", "head", "adapter_down", "adapter_up", "embed", "att", "sample")

EXPORTS = [
    "ee_last_error", "ee_model_load", "ee_model_load_ex", "ee_model_free", "ee_model_info",
    "ee_session_create", "ee_session_free", "ee_prefill", "ee_prefill_embeds", "ee_verify",
    "ee_verify_batch", "ee_verify_static", "ee_verify_sampled", "ee_wait_exit", "ee_query_exit", "ee_wait_final", "ee_query_final",
    "ee_pass_time_ms", "ee_kv_truncate", "ee_set_pending", "ee_kv_len", "ee_pending",
    "ee_verify_sampled_batch", "ee_debug_logits", "ee_debug_mfma_layout", "ee_debug_div_small", "ee_tune_k_split", "ee_device_synchronize", "ee_session_option",
    "ee_launch_times", "ee_debug_copy", "ee_exit_pop", "ee_exit_order", "ee_latency_model",
]


class EEError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"[{code}] {msg}")
        self.code = code


class ModelConfigC(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("d_ffn", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("n_exits", ctypes.c_int32), ("exit_layers", ctypes.c_int32 * EE_MAX_EXITS),
                ("rope_base", ctypes.c_float), ("rms_eps", ctypes.c_float),
                ("n_adapters", ctypes.c_int32), ("adapter_width", ctypes.c_int32),
                ("max_rows", ctypes.c_int32), ("n_workgroups", ctypes.c_int32)]


class SamplingC(ctypes.Structure):
    _fields_ = [("draft_probs", ctypes.POINTER(ctypes.c_float)), ("u", ctypes.POINTER(ctypes.c_float)),
                ("v", ctypes.POINTER(ctypes.c_float)), ("temperature", ctypes.c_float)]


class VerifyResultC(ctypes.Structure):
    _fields_ = [("gamma", ctypes.c_int32), ("n_exits", ctypes.c_int32),
                ("accept_len", ctypes.c_int32), ("next_token", ctypes.c_int32),
                ("final_tokens", ctypes.c_int32 * EE_MAX_M),
                ("exit_accept_len", ctypes.c_int32 * EE_MAX_EXITS),
                ("exit_tokens", (ctypes.c_int32 * EE_MAX_M) * EE_MAX_EXITS),
                ("device_status", ctypes.c_int32), ("reserved", ctypes.c_int32 * 15),
                ("final_conf", ctypes.c_float * EE_MAX_M), ("exit_conf", (ctypes.c_float * EE_MAX_M) * EE_MAX_EXITS)]


class LatencyParamsC(ctypes.Structure):
    _fields_ = [("T_p", ctypes.c_double), ("T_q", ctypes.c_double), ("T_c", ctypes.c_double), ("T_r", ctypes.c_double),
                ("tau", ctypes.c_double), ("r", ctypes.c_double), ("gamma", ctypes.c_int32), ("n", ctypes.c_int32)]


class LatencyC(ctypes.Structure):
    _fields_ = [(k, ctypes.c_double) for k in ("ar_ms", "sd_ms", "fsd_ms", "ar_ms_per_token", "sd_ms_per_token", "fsd_ms_per_token",
                                                "speedup_ar_to_sd", "speedup_sd_to_fsd", "c", "projected_sd_to_fsd")]


_lib = None


def lib_path() -> str:
    return _build.LIB_PATH


def load_library():
    """Load libeeverify.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        _build.build()
    lib = ctypes.CDLL(path)
    P = ctypes.POINTER
    vp, i32p, ci = ctypes.c_void_p, P(ctypes.c_int32), ctypes.c_int
    lib.ee_last_error.restype = ctypes.c_char_p
    lib.ee_last_error.argtypes = []
    lib.ee_model_load.argtypes = [ctypes.c_char_p, ci, P(vp)]
    lib.ee_model_load_ex.argtypes = [ctypes.c_char_p, ci, ci, P(vp)]
    lib.ee_model_free.argtypes = [vp]
    lib.ee_model_info.argtypes = [vp, P(ModelConfigC)]
    lib.ee_session_create.argtypes = [vp, ci, ci, ctypes.c_uint, P(vp)]
    lib.ee_session_free.argtypes = [vp]
    lib.ee_prefill.argtypes = [vp, i32p, ci, ctypes.c_uint, i32p]
    lib.ee_prefill_embeds.argtypes = [vp, vp, ci, i32p, ci, ctypes.c_uint, i32p]
    lib.ee_verify.argtypes = [vp, i32p, ci, i32p, ci, P(P(VerifyResultC))]
    lib.ee_verify_static.argtypes = [vp, i32p, ci, i32p, ci, P(P(VerifyResultC))]
    lib.ee_verify_sampled.argtypes = [vp, i32p, ci, i32p, ci, P(SamplingC), P(P(VerifyResultC))]
    lib.ee_verify_batch.argtypes = [P(vp), ci, P(i32p), ci, i32p, ci, P(P(VerifyResultC))]
    lib.ee_verify_sampled_batch.argtypes = [P(vp), ci, P(i32p), ci, i32p, ci, P(SamplingC), P(P(VerifyResultC))]
    lib.ee_wait_exit.argtypes = [vp, ci]
    lib.ee_query_exit.argtypes = [vp, ci]
    lib.ee_wait_final.argtypes = [vp]
    lib.ee_query_final.argtypes = [vp]
    lib.ee_pass_time_ms.argtypes = [vp, ci, P(ctypes.c_float)]
    lib.ee_kv_truncate.argtypes = [vp, ci]
    lib.ee_set_pending.argtypes = [vp, ctypes.c_int32]
    lib.ee_kv_len.argtypes = [vp, P(ci)]
    lib.ee_pending.argtypes = [vp, i32p]
    lib.ee_debug_logits.argtypes = [vp, ci, vp]
    lib.ee_debug_mfma_layout.argtypes = [ci]
    lib.ee_tune_k_split.argtypes = [ctypes.c_uint, ci]
    lib.ee_debug_div_small.argtypes = [ci, ctypes.POINTER(ctypes.c_int32), ci, ctypes.POINTER(ctypes.c_longlong)]
    lib.ee_device_synchronize.argtypes = [ci]
    lib.ee_session_option.argtypes = [vp, ci, ci]
    lib.ee_exit_pop.argtypes = [vp, ci, P(ci), P(ctypes.c_float)]
    lib.ee_exit_order.argtypes = [vp, P(ci), P(ctypes.c_float)]
    lib.ee_latency_model.argtypes = [P(LatencyParamsC), P(LatencyC)]
    lib.ee_debug_copy.argtypes = [ci, ctypes.c_size_t, ci]
    lib.ee_launch_times.argtypes = [vp, i32p, P(ctypes.c_float), ci, P(ci)]
    for name in EXPORTS:
        if name != "ee_last_error":
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(rc: int) -> int:
    if rc < 0:
        raise EEError(rc, load_library().ee_last_error().decode(errors="replace"))
    return rc


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32).reshape(-1))


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if a.size else None


def ee_device_synchronize(device: int = 0) -> None:
    _check(load_library().ee_device_synchronize(device))


def ee_verify_sampled_batch(sessions: List[Session], drafts: List[Sequence[int]], draft_probs, u, v, temperatures,
                            exit_layers: Sequence[int] = ()) -> None:
    """ee_verify_batch with each session's draft distributions [gamma][vocab], uniform numbers
    u [gamma], v [gamma+1] and temperature (lists, one entry per session)."""
    lib = load_library()
    n = len(sessions)
    hs = (ctypes.c_void_p * n)(*[s._h for s in sessions])
    ds = [_i32(d) for d in drafts]
    gamma = ds[0].size
    assert all(d.size == gamma for d in ds)
    dp = (ctypes.POINTER(ctypes.c_int32) * n)(*[_p(d) for d in ds])
    fp = ctypes.POINTER(ctypes.c_float)
    keep = []
    sms = (SamplingC * n)()
    for i in range(n):
        pr = np.ascontiguousarray(draft_probs[i], dtype=np.float32)
        uu = np.ascontiguousarray(u[i], dtype=np.float32)
        vv = np.ascontiguousarray(v[i], dtype=np.float32)
        if pr.shape != (gamma, sessions[i].model.vocab) or uu.size != gamma or vv.size != gamma + 1:
            raise ValueError("draft_probs [gamma][vocab], u [gamma], v [gamma+1] expected for every session")
        keep += [pr, uu, vv]
        sms[i] = SamplingC(pr.ctypes.data_as(fp), uu.ctypes.data_as(fp), vv.ctypes.data_as(fp), float(temperatures[i]))
    ex = _i32(exit_layers)
    outs = (ctypes.POINTER(VerifyResultC) * n)()
    _check(lib.ee_verify_sampled_batch(hs, n, dp, gamma, _p(ex), ex.size, sms, outs))
    for i, s in enumerate(sessions):
        s._res, s._n_exits, s._gamma = outs[i], ex.size, gamma


def ee_debug_mfma_layout(device: int = 0) -> None:
    _check(load_library().ee_debug_mfma_layout(device))


def ee_tune_k_split(kind_mask: int, log2_splits: int) -> None:
    _check(load_library().ee_tune_k_split(kind_mask, log2_splits))


def ee_debug_div_small(divisors, device: int = 0) -> int:
    d = np.ascontiguousarray(divisors, dtype=np.int32)
    bad = ctypes.c_longlong(-1)
    _check(load_library().ee_debug_div_small(device, d.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), int(d.size), ctypes.byref(bad)))
    return int(bad.value)


@dataclass
class VerifyOutput:
    gamma: int
    accept_len: int
    next_token: int
    final_tokens: np.ndarray
    exit_accept_len: np.ndarray
    exit_tokens: np.ndarray
    final_conf: np.ndarray = None   # [gamma+1] float32
    exit_conf: np.ndarray = None    # [n_exits][gamma+1] float32


class Model:
    """ee_model_load / ee_model_free / ee_model_info."""

    def __init__(self, path: str, device: int = 0, max_rows: int = 16):
        self._l = load_library()
        h = ctypes.c_void_p()
        _check(self._l.ee_model_load_ex(path.encode(), device, max_rows, ctypes.byref(h)))
        self._h = h
        c = ModelConfigC()
        _check(self._l.ee_model_info(h, ctypes.byref(c)))
        self.config = c
        self.n_layers, self.d_model, self.n_heads, self.head_dim = c.n_layers, c.d_model, c.n_heads, c.head_dim
        self.d_ffn, self.vocab, self.max_rows, self.n_workgroups = c.d_ffn, c.vocab, c.max_rows, c.n_workgroups
        self.exit_layers = [c.exit_layers[i] for i in range(c.n_exits)]

    def free(self):
        if self._h:
            self._l.ee_model_free(self._h)
            self._h = None

    def session(self, max_ctx: int, max_gamma: int = 8, flags: int = 0) -> "Session":
        return Session(self, max_ctx, max_gamma, flags)


class Session:
    """ee_session_create and the per-session calls, same names as the C ABI."""

    def __init__(self, model: Model, max_ctx: int, max_gamma: int = 8, flags: int = 0):
        self.model = model
        self._l = model._l
        h = ctypes.c_void_p()
        _check(self._l.ee_session_create(model._h, max_ctx, max_gamma, flags, ctypes.byref(h)))
        self._h = h
        self._res = None
        self._n_exits = 0
        self._gamma = 0

    def free(self):
        if self._h:
            self._l.ee_session_free(self._h)
            self._h = None

    def ee_prefill(self, tokens: Sequence[int], flags: int = 0, emb: Optional[np.ndarray] = None) -> Optional[int]:
        t = _i32(tokens)
        first = ctypes.c_int32(-1)
        if emb is None:
            _check(self._l.ee_prefill(self._h, _p(t), t.size, flags, ctypes.byref(first)))
        else:
            e = np.ascontiguousarray(emb, dtype=np.uint16)
            _check(self._l.ee_prefill_embeds(self._h, e.ctypes.data, e.shape[0], _p(t), t.size, flags,
                                             ctypes.byref(first)))
        return None if flags & HOLD_LAST else int(first.value)

    def ee_verify(self, draft_tokens: Sequence[int], exit_layers: Sequence[int] = ()) -> None:
        """Asynchronous; results via ee_wait_exit / ee_wait_final + exit_result / final_result."""
        d, ex = _i32(draft_tokens), _i32(exit_layers)
        res = ctypes.POINTER(VerifyResultC)()
        _check(self._l.ee_verify(self._h, _p(d), d.size, _p(ex), ex.size, ctypes.byref(res)))
        self._res, self._n_exits, self._gamma = res, ex.size, d.size

    def ee_verify_static(self, draft_tokens: Sequence[int], exit_layers: Sequence[int] = ()) -> None:
        """ee_verify on the library's static scratch array (allocates nothing)."""
        d, ex = _i32(draft_tokens), _i32(exit_layers)
        res = ctypes.POINTER(VerifyResultC)()
        _check(self._l.ee_verify_static(self._h, _p(d), d.size, _p(ex), ex.size, ctypes.byref(res)))
        self._res, self._n_exits, self._gamma = res, ex.size, d.size

    def ee_verify_sampled(self, draft_tokens: Sequence[int], draft_probs, u, v, temperature: float = 1.0,
                          exit_layers: Sequence[int] = ()) -> None:
        """ee_verify with the draft model's distributions [gamma][vocab] and the caller's uniform numbers."""
        d, ex = _i32(draft_tokens), _i32(exit_layers)
        pr = np.ascontiguousarray(draft_probs, dtype=np.float32)
        uu = np.ascontiguousarray(u, dtype=np.float32)
        vv = np.ascontiguousarray(v, dtype=np.float32)
        if pr.ndim != 2 or pr.shape[0] != d.size or pr.shape[1] != self.model.vocab or uu.size != d.size or vv.size != d.size + 1:
            raise ValueError("draft_probs [gamma][vocab], u [gamma], v [gamma+1] expected")
        fp = ctypes.POINTER(ctypes.c_float)
        sm = SamplingC(pr.ctypes.data_as(fp), uu.ctypes.data_as(fp), vv.ctypes.data_as(fp), float(temperature))
        res = ctypes.POINTER(VerifyResultC)()
        _check(self._l.ee_verify_sampled(self._h, _p(d), d.size, _p(ex), ex.size, ctypes.byref(sm), ctypes.byref(res)))
        self._res, self._n_exits, self._gamma = res, ex.size, d.size

    def ee_wait_exit(self, exit_idx: int) -> None:
        _check(self._l.ee_wait_exit(self._h, exit_idx))

    def ee_query_exit(self, exit_idx: int) -> bool:
        return _check(self._l.ee_query_exit(self._h, exit_idx)) == EE_OK

    def ee_wait_final(self) -> None:
        _check(self._l.ee_wait_final(self._h))

    def ee_query_final(self) -> bool:
        return _check(self._l.ee_query_final(self._h)) == EE_OK

    def ee_pass_time_ms(self, exit_idx: int) -> float:
        ms = ctypes.c_float()
        _check(self._l.ee_pass_time_ms(self._h, exit_idx, ctypes.byref(ms)))
        return float(ms.value)

    def ee_kv_truncate(self, new_len: int) -> None:
        _check(self._l.ee_kv_truncate(self._h, new_len))

    def ee_set_pending(self, token: int) -> None:
        _check(self._l.ee_set_pending(self._h, token))

    def ee_kv_len(self) -> int:
        v = ctypes.c_int()
        _check(self._l.ee_kv_len(self._h, ctypes.byref(v)))
        return int(v.value)

    def ee_pending(self) -> int:
        v = ctypes.c_int32()
        _check(self._l.ee_pending(self._h, ctypes.byref(v)))
        return int(v.value)

    def ee_debug_logits(self, head_idx: int) -> np.ndarray:
        out = np.empty((self._gamma + 1, self.model.vocab), dtype=np.float32)
        _check(self._l.ee_debug_logits(self._h, head_idx, out.ctypes.data))
        return out

    def ee_exit_pop(self, wait: bool = True):
        """(status, exit index, score): status EE_OK, EE_NOT_READY or EE_DONE."""
        idx, sc = ctypes.c_int(-1), ctypes.c_float(0.0)
        rc = _check(self._l.ee_exit_pop(self._h, 1 if wait else 0, ctypes.byref(idx), ctypes.byref(sc)))
        return rc, int(idx.value), float(sc.value)

    def ee_exit_order(self):
        """([exit index], [score]) in the order the sender's queue releases them."""
        n = self._n_exits
        order, sc = (ctypes.c_int * max(n, 1))(), (ctypes.c_float * max(n, 1))()
        _check(self._l.ee_exit_order(self._h, order, sc))
        return [int(order[i]) for i in range(n)], [float(sc[i]) for i in range(n)]

    def ee_session_option(self, option: int, value: int) -> None:
        _check(self._l.ee_session_option(self._h, option, value))

    def ee_launch_times(self):
        """[(launch code, milliseconds)] of every launch of the last verify pass."""
        cap = 4096
        codes, ms, n = (ctypes.c_int32 * cap)(), (ctypes.c_float * cap)(), ctypes.c_int()
        _check(self._l.ee_launch_times(self._h, codes, ms, cap, ctypes.byref(n)))
        return [(int(codes[i]), float(ms[i])) for i in range(n.value)]

    # plain reads of the pinned result block (no computation)
    def exit_result(self, exit_idx: int):
        r, M = self._res.contents, self._gamma + 1
        return np.array(r.exit_tokens[exit_idx][:M], dtype=np.int32), int(r.exit_accept_len[exit_idx])

    def exit_conf(self, exit_idx: int) -> np.ndarray:
        r, M = self._res.contents, self._gamma + 1
        return np.array(r.exit_conf[exit_idx][:M], dtype=np.float32)

    def final_result(self) -> VerifyOutput:
        r, M, E = self._res.contents, self._gamma + 1, self._n_exits
        return VerifyOutput(
            gamma=self._gamma, accept_len=int(r.accept_len), next_token=int(r.next_token),
            final_tokens=np.array(r.final_tokens[:M], dtype=np.int32),
            exit_accept_len=np.array(r.exit_accept_len[:E], dtype=np.int32),
            exit_tokens=np.array([list(r.exit_tokens[e][:M]) for e in range(E)], dtype=np.int32).reshape(E, M),
            final_conf=np.array(r.final_conf[:M], dtype=np.float32),
            exit_conf=np.array([list(r.exit_conf[e][:M]) for e in range(E)], dtype=np.float32).reshape(E, M))

    def verify_sync(self, draft_tokens: Sequence[int], exit_layers: Sequence[int] = ()) -> VerifyOutput:
        self.ee_verify(draft_tokens, exit_layers)
        self.ee_wait_final()
        return self.final_result()


def ee_latency_model(T_p: float, T_q: float, T_c: float, tau: float, gamma: int = 4, n: int = 200, r: float = 1.0,
                     T_r: float = 0.0) -> dict:
    """The paper's AR / SD / FSD latency formulas and Eq. 9 (times in ms); plain marshalling."""
    p = LatencyParamsC(T_p, T_q, T_c, T_r, tau, r, gamma, n)
    out = LatencyC()
    _check(load_library().ee_latency_model(ctypes.byref(p), ctypes.byref(out)))
    return {k: getattr(out, k) for k, _ in LatencyC._fields_}


def ee_debug_copy(device: int, nbytes: int, reps: int) -> None:
    _check(load_library().ee_debug_copy(device, nbytes, reps))


def ee_verify_batch(sessions: List[Session], drafts: List[Sequence[int]], exit_layers: Sequence[int] = ()) -> None:
    """One pass for several sessions; wait on any of them, read each one's result."""
    lib = load_library()
    n = len(sessions)
    hs = (ctypes.c_void_p * n)(*[s._h for s in sessions])
    ds = [_i32(d) for d in drafts]
    gamma = ds[0].size
    assert all(d.size == gamma for d in ds)
    dp = (ctypes.POINTER(ctypes.c_int32) * n)(*[_p(d) for d in ds])
    ex = _i32(exit_layers)
    outs = (ctypes.POINTER(VerifyResultC) * n)()
    _check(lib.ee_verify_batch(hs, n, dp, gamma, _p(ex), ex.size, outs))
    for i, s in enumerate(sessions):
        s._res, s._n_exits, s._gamma = outs[i], ex.size, gamma
