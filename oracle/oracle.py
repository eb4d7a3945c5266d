"""ctypes wrapper over the CPU oracle (oracle/ee_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg; never by the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
EO_MAX_EXITS = 40
EO_MAX_M = 64
HOLD_LAST = 1

EO_OK, EO_EINVAL, EO_ESTATE, EO_ECAPACITY, EO_EIO, EO_EFORMAT = 0, -1, -2, -3, -4, -5


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: oracle status {code}")
        self.code = code


class _Config(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("d_model", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("d_ffn", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("n_exits", ctypes.c_int32), ("rope_base", ctypes.c_float),
                ("rms_eps", ctypes.c_float), ("exit_layers", ctypes.c_int32 * EO_MAX_EXITS)]


class _Result(ctypes.Structure):
    _fields_ = [("gamma", ctypes.c_int32), ("n_exits", ctypes.c_int32),
                ("accept_len", ctypes.c_int32), ("next_token", ctypes.c_int32),
                ("final_tokens", ctypes.c_int32 * EO_MAX_M),
                ("exit_accept_len", ctypes.c_int32 * EO_MAX_EXITS),
                ("exit_tokens", (ctypes.c_int32 * EO_MAX_M) * EO_MAX_EXITS),
                ("final_conf", ctypes.c_double * EO_MAX_M),
                ("exit_conf", (ctypes.c_double * EO_MAX_M) * EO_MAX_EXITS)]


class _Trace(ctypes.Structure):
    _fields_ = [("h", ctypes.c_void_p), ("q", ctypes.c_void_p), ("k", ctypes.c_void_p),
                ("v", ctypes.c_void_p), ("attn", ctypes.c_void_p)]


def build(force: bool = False) -> None:
    """Compile the float (liboracle32.so) and double (liboracle64.so) builds."""
    src = os.path.join(_HERE, "ee_oracle.c")
    hdr = os.path.join(_HERE, "ee_oracle.h")
    newest = max(os.path.getmtime(src), os.path.getmtime(hdr))
    for name, extra in (("liboracle32.so", []), ("liboracle64.so", ["-DEO_REAL=double"])):
        out = os.path.join(_HERE, name)
        if force or not os.path.exists(out) or os.path.getmtime(out) < newest:
            subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ftree-vectorize", "-Wall", "-Wextra",
                                   "-shared", "-fPIC", *extra, "-o", out, src, "-lm"])


_libs = {}


def _lib(real: str):
    if real not in _libs:
        # EE_ORACLE_LIBDIR: load prebuilt libraries from another folder (the mutation
        # tests point it at deliberately broken builds of the oracle).
        libdir = os.environ.get("EE_ORACLE_LIBDIR")
        if not libdir:
            build()
            libdir = _HERE
        lib = ctypes.CDLL(os.path.join(libdir, {"f32": "liboracle32.so", "f64": "liboracle64.so"}[real]))
        P = ctypes.POINTER
        vp, i32p = ctypes.c_void_p, P(ctypes.c_int32)
        lib.eo_model_open.argtypes = [ctypes.c_char_p, P(vp)]
        lib.eo_model_close.argtypes = [vp]
        lib.eo_model_close.restype = None
        lib.eo_model_config.argtypes = [vp, P(_Config)]
        lib.eo_session_new.argtypes = [vp, ctypes.c_int, P(vp)]
        lib.eo_session_free.argtypes = [vp]
        lib.eo_session_free.restype = None
        lib.eo_prefill.argtypes = [vp, i32p, ctypes.c_int, ctypes.c_uint, i32p]
        lib.eo_prefill_embeds.argtypes = [vp, vp, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_uint, i32p]
        lib.eo_verify.argtypes = [vp, i32p, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_int,
                                  P(_Result), vp, P(_Trace)]
        lib.eo_kv_truncate.argtypes = [vp, ctypes.c_int]
        lib.eo_set_pending.argtypes = [vp, ctypes.c_int32]
        lib.eo_commit_rows.argtypes = [vp, ctypes.c_int, ctypes.c_int32]
        lib.eo_kv_len.argtypes = [vp]
        lib.eo_pending.argtypes = [vp, i32p]
        lib.eo_full_logits.argtypes = [vp, vp, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_int, vp]
        lib.eo_ar_decode.argtypes = [vp, vp, ctypes.c_int, i32p, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, i32p]
        assert lib.eo_sizeof_real() == {"f32": 4, "f64": 8}[real]
        _libs[real] = lib
    return _libs[real]


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32).reshape(-1))


def _ptr(a: Optional[np.ndarray]):
    if a is None or a.size == 0:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _check(rc: int, what: str):
    if rc != EO_OK:
        raise OracleError(rc, what)


@dataclass
class VerifyResult:
    gamma: int
    accept_len: int
    next_token: int
    final_tokens: np.ndarray            # [gamma+1]
    exit_accept_len: np.ndarray         # [n_exits]
    exit_tokens: np.ndarray             # [n_exits][gamma+1]
    final_conf: np.ndarray = None       # [gamma+1] max softmax probability per row, final head
    exit_conf: np.ndarray = None        # [n_exits][gamma+1] the same for every exit head
    logits: Optional[np.ndarray] = None  # [n_exits+1][gamma+1][V] float64 (final head last)
    trace: Optional[dict] = None


class Model:
    def __init__(self, path: str, real: str = "f32"):
        self.real = real
        self._l = _lib(real)
        h = ctypes.c_void_p()
        _check(self._l.eo_model_open(path.encode(), ctypes.byref(h)), "eo_model_open")
        self._h = h
        c = _Config()
        _check(self._l.eo_model_config(h, ctypes.byref(c)), "eo_model_config")
        self.n_layers, self.d_model, self.n_heads = c.n_layers, c.d_model, c.n_heads
        self.head_dim, self.d_ffn, self.vocab = c.head_dim, c.d_ffn, c.vocab
        self.exit_layers = [c.exit_layers[i] for i in range(c.n_exits)]
        self.rope_base, self.rms_eps = c.rope_base, c.rms_eps

    def close(self):
        if self._h:
            self._l.eo_model_close(self._h)
            self._h = None

    def session(self, max_ctx: int) -> "Session":
        return Session(self, max_ctx)

    def full_logits(self, tokens: Sequence[int], exit_layer: int = 0,
                    emb: Optional[np.ndarray] = None) -> np.ndarray:
        t = _i32(tokens)
        n_emb = 0 if emb is None else emb.shape[0]
        e = None if emb is None else np.ascontiguousarray(emb, dtype=np.uint16)
        out = np.empty((n_emb + t.size, self.vocab), dtype=np.float64)
        _check(self._l.eo_full_logits(self._h, None if e is None else e.ctypes.data, n_emb,
                                      _ptr(t), t.size, exit_layer, out.ctypes.data), "eo_full_logits")
        return out

    def ar_decode(self, tokens: Sequence[int], n_new: int, exit_layer: int = 0,
                  emb: Optional[np.ndarray] = None) -> np.ndarray:
        t = _i32(tokens)
        n_emb = 0 if emb is None else emb.shape[0]
        e = None if emb is None else np.ascontiguousarray(emb, dtype=np.uint16)
        out = np.empty(n_new, dtype=np.int32)
        _check(self._l.eo_ar_decode(self._h, None if e is None else e.ctypes.data, n_emb,
                                    _ptr(t), t.size, exit_layer, n_new, _ptr(out)), "eo_ar_decode")
        return out


class Session:
    def __init__(self, model: Model, max_ctx: int):
        self.model = model
        self._l = model._l
        h = ctypes.c_void_p()
        _check(self._l.eo_session_new(model._h, max_ctx, ctypes.byref(h)), "eo_session_new")
        self._h = h

    def close(self):
        if self._h:
            self._l.eo_session_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, tokens: Sequence[int], flags: int = 0, emb: Optional[np.ndarray] = None) -> Optional[int]:
        t = _i32(tokens)
        first = ctypes.c_int32(-1)
        if emb is None:
            rc = self._l.eo_prefill(self._h, _ptr(t), t.size, flags, ctypes.byref(first))
        else:
            e = np.ascontiguousarray(emb, dtype=np.uint16)
            rc = self._l.eo_prefill_embeds(self._h, e.ctypes.data, e.shape[0], _ptr(t), t.size, flags,
                                           ctypes.byref(first))
        _check(rc, "eo_prefill")
        return None if (flags & HOLD_LAST) else int(first.value)

    def verify(self, drafts: Sequence[int], exit_layers: Sequence[int] = (), commit: bool = True,
               want_logits: bool = False, want_trace: bool = False) -> VerifyResult:
        d = _i32(drafts)
        ex = _i32(exit_layers)
        gamma, M = d.size, d.size + 1
        res = _Result()
        m = self.model
        logits = np.empty((ex.size + 1, M, m.vocab), dtype=np.float64) if want_logits else None
        tr, trace = None, None
        if want_trace:
            L, dm = m.n_layers, m.d_model
            trace = {"h": np.zeros((L + 1, M, dm)), "q": np.zeros((L, M, dm)), "k": np.zeros((L, M, dm)),
                     "v": np.zeros((L, M, dm)), "attn": np.zeros((L, M, dm))}
            tr = _Trace(*(trace[k].ctypes.data for k in ("h", "q", "k", "v", "attn")))
        rc = self._l.eo_verify(self._h, _ptr(d), gamma, _ptr(ex), ex.size, int(commit), ctypes.byref(res),
                               None if logits is None else logits.ctypes.data,
                               None if tr is None else ctypes.byref(tr))
        _check(rc, "eo_verify")
        return VerifyResult(
            gamma=gamma, accept_len=res.accept_len, next_token=res.next_token,
            final_tokens=np.array(res.final_tokens[:M], dtype=np.int32),
            exit_accept_len=np.array(res.exit_accept_len[:ex.size], dtype=np.int32),
            exit_tokens=np.array([list(res.exit_tokens[e][:M]) for e in range(ex.size)],
                                 dtype=np.int32).reshape(ex.size, M),
            final_conf=np.array(res.final_conf[:M], dtype=np.float64),
            exit_conf=np.array([list(res.exit_conf[e][:M]) for e in range(ex.size)],
                               dtype=np.float64).reshape(ex.size, M),
            logits=logits, trace=trace)

    def kv_truncate(self, new_len: int):
        _check(self._l.eo_kv_truncate(self._h, new_len), "eo_kv_truncate")

    def commit_rows(self, delta: int, token: int):
        """Commit of the last verify(commit=False) pass with an accept decision taken outside."""
        _check(self._l.eo_commit_rows(self._h, delta, token), "eo_commit_rows")

    def set_pending(self, token: int):
        _check(self._l.eo_set_pending(self._h, token), "eo_set_pending")

    @property
    def kv_len(self) -> int:
        return int(self._l.eo_kv_len(self._h))

    @property
    def pending(self) -> int:
        t = ctypes.c_int32()
        _check(self._l.eo_pending(self._h, ctypes.byref(t)), "eo_pending")
        return int(t.value)


def top2_margin(logits: np.ndarray) -> np.ndarray:
    """Gap between the largest and second-largest logit along the last axis."""
    part = np.partition(logits, logits.shape[-1] - 2, axis=-1)
    return part[..., -1] - part[..., -2]
