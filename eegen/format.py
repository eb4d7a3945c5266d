"""Model-file layout and seeded writer for synthetic Llama-style decoders.

The file is the only thing the CPU oracle and the GPU library have in common:
each has its own reader.  Layout (little endian):

  bytes 0..255   header
      0   char[8]  magic "EEVMODL1"
      8   u32      version (1)
      12  u32      n_layers  L
      16  u32      d_model   d
      20  u32      n_heads   H
      24  u32      head_dim  hd   (H*hd == d)
      28  u32      d_ffn     F
      32  u32      vocab     V
      36  u32      n_exits        (number of exit heads stored)
      40  f32      rope_base
      44  f32      rms_eps
      48  u32[40]  exit_layers    (1-based "after layer e", strictly increasing; unused entries 0)
      208 u32      n_adapters     (bottleneck adapters per exit head; 0 = exit heads without adapters)
      212 u32      adapter_width  (width of one bottleneck)
  then bf16 tensors, each starting on a 256-byte boundary, row-major, in this order:
      emb[V][d]
      for l in 1..L: g_attn[d] wq[d][d] wk[d][d] wv[d][d] wo[d][d]
                     g_ffn[d]  wg[F][d] wu[F][d] wd[d][F]
      g_final[d]  w_lm[V][d]
      g_exit[e][d] for every stored exit, in header order
      with adapters (A = n_adapters * adapter_width), for every stored exit in header order:
          ad_down[A][d]  ad_bdown[A]  ad_up[d][A]  ad_bup[n_adapters][d]

All matrices are [out_features][in_features].  This module contains no part of
the decoding method's arithmetic, only sizes, offsets and random fills.
"""
from __future__ import annotations

import ctypes
import os
import struct
import subprocess
from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

MAGIC = b"EEVMODL1"
VERSION = 1
HEADER_BYTES = 256
ALIGN = 256
MAX_EXITS = 40

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libeegen.so")


@dataclass(frozen=True)
class ModelConfig:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    exit_layers: Tuple[int, ...] = ()
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    n_adapters: int = 0        # bottleneck adapters per exit head (0: none)
    adapter_width: int = 0     # width of one bottleneck

    def __post_init__(self):
        assert (self.n_adapters == 0) == (self.adapter_width == 0)
        assert self.n_heads * self.head_dim == self.d_model
        assert len(self.exit_layers) <= MAX_EXITS
        assert all(1 <= e < self.n_layers for e in self.exit_layers)
        assert list(self.exit_layers) == sorted(set(self.exit_layers))


def build_lib(force: bool = False) -> str:
    """Compile the bulk filler (gcc, OpenMP) next to this file."""
    src = os.path.join(_HERE, "fill.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src, "-lm"]
        )
    return _LIB_PATH


_lib = None


def _get_lib():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_lib())
        lib.eeg_fill_normal_bf16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                             ctypes.c_uint64, ctypes.c_double]
        lib.eeg_fill_normal_bf16.restype = None
        lib.eeg_fill_uniform_bf16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint64,
                                              ctypes.c_uint64, ctypes.c_double, ctypes.c_double]
        lib.eeg_fill_uniform_bf16.restype = None
        lib.eeg_fill_const_bf16.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_double]
        lib.eeg_fill_const_bf16.restype = None
        _lib = lib
    return _lib


def _align(x: int) -> int:
    return (x + ALIGN - 1) // ALIGN * ALIGN


def tensor_table(cfg: ModelConfig) -> Tuple[Dict[str, Tuple[int, Tuple[int, ...]]], int]:
    """name -> (byte offset, shape); also returns the total file size."""
    d, F, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    names: List[Tuple[str, Tuple[int, ...]]] = [("emb", (V, d))]
    for l in range(1, cfg.n_layers + 1):
        names += [
            (f"l{l}.g_attn", (d,)), (f"l{l}.wq", (d, d)), (f"l{l}.wk", (d, d)),
            (f"l{l}.wv", (d, d)), (f"l{l}.wo", (d, d)), (f"l{l}.g_ffn", (d,)),
            (f"l{l}.wg", (F, d)), (f"l{l}.wu", (F, d)), (f"l{l}.wd", (d, F)),
        ]
    names += [("g_final", (d,)), ("w_lm", (V, d))]
    for e in cfg.exit_layers:
        names.append((f"g_exit{e}", (d,)))
    A = cfg.n_adapters * cfg.adapter_width
    if A:
        for e in cfg.exit_layers:
            names += [(f"ad_down{e}", (A, d)), (f"ad_bdown{e}", (A,)), (f"ad_up{e}", (d, A)),
                      (f"ad_bup{e}", (cfg.n_adapters, d))]
    table = {}
    off = HEADER_BYTES
    for name, shape in names:
        off = _align(off)
        table[name] = (off, shape)
        off += 2 * int(np.prod(shape))
    return table, _align(off)


def pack_header(cfg: ModelConfig) -> bytes:
    ex = list(cfg.exit_layers) + [0] * (MAX_EXITS - len(cfg.exit_layers))
    h = MAGIC + struct.pack("<8I2f40I2I", VERSION, cfg.n_layers, cfg.d_model, cfg.n_heads,
                            cfg.head_dim, cfg.d_ffn, cfg.vocab, len(cfg.exit_layers),
                            cfg.rope_base, cfg.rms_eps, *ex, cfg.n_adapters, cfg.adapter_width)
    return h + b"\0" * (HEADER_BYTES - len(h))


def read_header(path: str) -> ModelConfig:
    with open(path, "rb") as f:
        h = f.read(HEADER_BYTES)
    assert h[:8] == MAGIC, "bad magic"
    vals = struct.unpack("<8I2f40I2I", h[8:8 + 32 + 8 + 160 + 8])
    ver, L, d, H, hd, F, V, ne = vals[:8]
    assert ver == VERSION
    base, eps = vals[8:10]
    ex = vals[10:10 + ne]
    return ModelConfig(L, d, H, hd, F, V, tuple(ex), base, eps, vals[50], vals[51])


def _stream_id(name: str) -> int:
    # stable 64-bit id per tensor name (FNV-1a)
    h = 0xCBF29CE484222325
    for c in name.encode():
        h = ((h ^ c) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def write_model(path: str, cfg: ModelConfig, seed: int, gains: str = "ones", std: float = 0.02,
                zero: Sequence[str] = ()) -> None:
    """Create a model file: matrices and adapter biases ~ N(0, std^2) rounded to bf16; gain
    vectors all 1.0 (gains="ones") or U[0.5,1.5) (gains="uniform").  Tensors whose per-layer
    short name (e.g. "wo", "wd") is in `zero`, or whose name starts with an entry of `zero` that
    ends in "*" (e.g. "ad_up*"), are left all-zero."""
    assert gains in ("ones", "uniform")
    lib = _get_lib()
    table, total = tensor_table(cfg)
    with open(path, "wb") as f:
        f.truncate(total)
    mm = np.memmap(path, dtype=np.uint8, mode="r+")
    mm[:HEADER_BYTES] = np.frombuffer(pack_header(cfg), dtype=np.uint8)
    base = mm.ctypes.data
    for name, (off, shape) in table.items():
        n = int(np.prod(shape))
        short = name.split(".")[-1]
        ptr = ctypes.c_void_p(base + off)
        if short in zero or any(z.endswith("*") and short.startswith(z[:-1]) for z in zero):
            continue  # file is zero-filled by truncate
        if len(shape) == 1 and not short.startswith("ad_b"):
            if gains == "ones":
                lib.eeg_fill_const_bf16(ptr, n, 1.0)
            else:
                lib.eeg_fill_uniform_bf16(ptr, n, seed, _stream_id(name), 0.5, 1.5)
        else:
            lib.eeg_fill_normal_bf16(ptr, n, seed, _stream_id(name), std)
    mm.flush()
    del mm


def adapter_parameters(cfg: ModelConfig, n_heads_with_adapters: int) -> int:
    """Weights and biases of the adapters of n exit heads."""
    d, w = cfg.d_model, cfg.adapter_width
    return n_heads_with_adapters * cfg.n_adapters * (2 * d * w + w + d)


def open_tensors(path: str, mode: str = "r") -> Dict[str, np.ndarray]:
    """Memory-map every tensor as a uint16 (raw bf16) array; mode "r+" allows
    tests to patch weights in place."""
    cfg = read_header(path)
    table, _ = tensor_table(cfg)
    mm = np.memmap(path, dtype=np.uint8, mode=mode)
    out = {}
    for name, (off, shape) in table.items():
        n = int(np.prod(shape))
        out[name] = mm[off:off + 2 * n].view(np.uint16).reshape(shape)
    return out


def bf16_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16(a: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + 0x7FFF + ((u >> 16) & 1)
    return (r >> 16).astype(np.uint16)
