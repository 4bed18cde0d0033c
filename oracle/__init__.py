"""CPU oracle of the NestedKV prefill compression pass.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg, never by the product package.  The arithmetic
lives in ``nkv_oracle.c`` (plain C, fp64); this file compiles it with gcc and
marshals numpy arrays.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nkv_oracle.c")
_LIB = os.path.join(_HERE, "libnkv_oracle.so")

PIN = np.float32(3.0e38)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over heads) and return the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Params(C.Structure):
    _fields_ = [("window", C.c_int32), ("block_div", C.c_int32), ("block_min", C.c_int32),
                ("block_max", C.c_int32), ("n_sink", C.c_int32), ("gate_mode", C.c_int32),
                ("surprise_mode", C.c_int32), ("std_ddof", C.c_int32), ("scale_mask", C.c_int32), ("pad_", C.c_int32),
                ("top_frac", C.c_double),
                ("prior", C.c_double * 3), ("beta", C.c_double), ("tau", C.c_double), ("kappa", C.c_double)]


class _Debug(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("mu_s", "mu_e", "mu_c", "a_raw", "a_tilde", "delta", "w",
                                          "surprise", "alpha", "blend", "win")]


@dataclass
class Params:
    window: int = 64
    block_div: int = 32
    block_min: int = 128
    block_max: int = 256
    n_sink: int = 4
    gate_mode: int = 0
    surprise_mode: int = 0
    std_ddof: int = 0
    scale_mask: int = 7       # bits 0..2: stable, episodic, current take part
    top_frac: float = 0.10
    prior: Tuple[float, float, float] = (0.4, 0.4, 0.2)
    beta: float = 3.0
    tau: float = 0.60
    kappa: float = 10.0
    safeguard: float = 0.20   # used by budgets only

    def _c(self) -> _Params:
        p = _Params()
        for n in ("window", "block_div", "block_min", "block_max", "n_sink", "gate_mode", "surprise_mode",
                  "std_ddof", "scale_mask", "top_frac", "beta", "tau", "kappa"):
            setattr(p, n, getattr(self, n))
        p.prior = (C.c_double * 3)(*self.prior)
        return p


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.nkvo_block_size.restype = C.c_int64
        L.nkvo_block_size.argtypes = [C.c_int64, C.POINTER(_Params)]
        L.nkvo_k0.restype = C.c_int64
        L.nkvo_k0.argtypes = [C.c_int64, C.c_double]
        L.nkvo_m_safe.restype = C.c_int64
        L.nkvo_m_safe.argtypes = [C.c_int64, C.c_double]
        L.nkvo_m_p.restype = C.c_int64
        L.nkvo_m_p.argtypes = [C.c_int64, C.c_double]
        L.nkvo_score_layer.restype = C.c_int
        L.nkvo_score_layer.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int, C.POINTER(_Params),
                                       C.c_void_p, C.POINTER(_Debug)]
        L.nkvo_budget_layer.restype = C.c_int
        L.nkvo_budget_layer.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p]
        L.nkvo_select_head.restype = C.c_int
        L.nkvo_select_head.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p]
        L.nkvo_gather_rows.restype = C.c_int
        L.nkvo_gather_rows.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p]
        _lib = L
    return _lib


def block_size(N: int, params: Optional[Params] = None) -> int:
    p = (params or Params())._c()
    return int(lib().nkvo_block_size(int(N), C.byref(p)))


def k0(N: int, r: float) -> int:
    return int(lib().nkvo_k0(int(N), float(r)))


def m_safe(k0_: int, safeguard: float = 0.20) -> int:
    return int(lib().nkvo_m_safe(int(k0_), float(safeguard)))


def m_p(N: int, top_frac: float = 0.10) -> int:
    return int(lib().nkvo_m_p(int(N), float(top_frac)))


_DEBUG_SHAPES = {
    "mu_s": lambda H, N, d, nb: (H, d), "mu_e": lambda H, N, d, nb: (H, nb, d),
    "mu_c": lambda H, N, d, nb: (H, N, d), "a_raw": lambda H, N, d, nb: (3, H, N),
    "a_tilde": lambda H, N, d, nb: (3, H, N), "delta": lambda H, N, d, nb: (H, 3),
    "w": lambda H, N, d, nb: (H, 3), "surprise": lambda H, N, d, nb: (H, N),
    "alpha": lambda H, N, d, nb: (H, N), "blend": lambda H, N, d, nb: (H, N), "win": lambda H, N, d, nb: (H, N),
}


def score_layer(keys: np.ndarray, params: Optional[Params] = None,
                debug: Sequence[str] = ()) -> Tuple[np.ndarray, Dict[str, np.ndarray]]:
    """keys [H, N, d] (float32 holding the stored values exactly) -> scores [H, N] float32.

    ``debug`` names intermediates to return (see ``nkvo_debug`` in the C source).
    """
    params = params or Params()
    keys = np.ascontiguousarray(keys, dtype=np.float32)
    H, N, d = keys.shape
    scores = np.empty((H, N), dtype=np.float32)
    p = params._c()
    dbg = _Debug()
    out: Dict[str, np.ndarray] = {}
    nb = (N + block_size(N, params) - 1) // block_size(N, params)
    for name in debug:
        arr = np.zeros(_DEBUG_SHAPES[name](H, N, d, nb), dtype=np.float64)
        out[name] = arr
        setattr(dbg, name, arr.ctypes.data)
    rc = lib().nkvo_score_layer(keys.ctypes.data, H, N, d, C.byref(p), scores.ctypes.data, C.byref(dbg))
    if rc != 0:
        raise RuntimeError(f"nkvo_score_layer failed: {rc}")
    return scores, out


def budget_layer(scores: np.ndarray, r: float, safeguard: float = 0.20) -> np.ndarray:
    """scores [H, N] float32 -> B [H] int32 with sum(B) == H * k0."""
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    H, N = scores.shape
    kk = k0(N, r)
    ms = m_safe(kk, safeguard)
    B = np.empty(H, dtype=np.int32)
    rc = lib().nkvo_budget_layer(scores.ctypes.data, H, N, kk, ms, B.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"nkvo_budget_layer failed: {rc}")
    return B


def select_head(scores: np.ndarray, B: int) -> np.ndarray:
    """scores [N] float32, budget B -> kept token indices, ascending, int32 [B]."""
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    kept = np.empty(max(int(B), 0), dtype=np.int32)
    rc = lib().nkvo_select_head(scores.ctypes.data, scores.shape[0], int(B), kept.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"nkvo_select_head failed: {rc}")
    return kept


def gather_rows(rows: np.ndarray, kept: np.ndarray) -> np.ndarray:
    """rows [N, ...] of any dtype (viewed as bytes), kept int32 [B] -> bitwise copies rows[kept]."""
    rows = np.ascontiguousarray(rows)
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    out = np.empty((kept.shape[0],) + rows.shape[1:], dtype=rows.dtype)
    row_bytes = rows.strides[0]
    rc = lib().nkvo_gather_rows(rows.ctypes.data, row_bytes, kept.ctypes.data, kept.shape[0], out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"nkvo_gather_rows failed: {rc}")
    return out


@dataclass
class Compressed:
    """Result of the whole pass, laid out like the library's output."""
    scores: np.ndarray        # [L, H, T] float32
    k_per_head: np.ndarray    # [P, L, H] int32
    head_off: np.ndarray      # [P*L*H + 1] int64, row offsets of every (prompt, layer, head)
    kept_idx: np.ndarray      # [rows] int32, prompt-local token indices, ascending per head
    packed_k: np.ndarray      # [rows, d]   (dtype of the input)
    packed_v: np.ndarray      # [rows, dv]


def compress(keys_f32: np.ndarray, keys_raw: np.ndarray, values_raw: np.ndarray, cu_seqlens: Sequence[int],
             r_per_prompt: Sequence[float], params: Optional[Params] = None,
             scores: Optional[np.ndarray] = None, k_per_head: Optional[np.ndarray] = None) -> Compressed:
    """The whole pass over keys[L, H, T, d]: score, budget, select, compact.

    ``keys_f32`` are the stored key values widened to float32; ``keys_raw`` / ``values_raw`` are arrays of
    the stored element type (or an integer view of it), copied bitwise into the packed outputs.  Passing
    ``scores`` and/or ``k_per_head`` skips the corresponding stage (stage-wise parity tests).
    """
    params = params or Params()
    L, H, T, d = keys_f32.shape
    P = len(cu_seqlens) - 1
    if scores is None:
        scores = np.empty((L, H, T), dtype=np.float32)
        for p in range(P):
            lo, hi = cu_seqlens[p], cu_seqlens[p + 1]
            for l in range(L):
                scores[l, :, lo:hi] = score_layer(keys_f32[l, :, lo:hi], params)[0]
    if k_per_head is None:
        k_per_head = np.empty((P, L, H), dtype=np.int32)
        for p in range(P):
            lo, hi = cu_seqlens[p], cu_seqlens[p + 1]
            for l in range(L):
                k_per_head[p, l] = budget_layer(scores[l, :, lo:hi], r_per_prompt[p], params.safeguard)
    head_off = np.zeros(P * L * H + 1, dtype=np.int64)
    head_off[1:] = np.cumsum(k_per_head.reshape(-1).astype(np.int64))
    rows = int(head_off[-1])
    kept_idx = np.empty(rows, dtype=np.int32)
    packed_k = np.empty((rows,) + keys_raw.shape[3:], dtype=keys_raw.dtype)
    packed_v = np.empty((rows,) + values_raw.shape[3:], dtype=values_raw.dtype)
    u = 0
    for p in range(P):
        lo, hi = cu_seqlens[p], cu_seqlens[p + 1]
        for l in range(L):
            for h in range(H):
                o, e = int(head_off[u]), int(head_off[u + 1])
                kept = select_head(scores[l, h, lo:hi], e - o)
                kept_idx[o:e] = kept
                packed_k[o:e] = gather_rows(keys_raw[l, h, lo:hi], kept)
                packed_v[o:e] = gather_rows(values_raw[l, h, lo:hi], kept)
                u += 1
    return Compressed(scores, k_per_head, head_off, kept_idx, packed_k, packed_v)
