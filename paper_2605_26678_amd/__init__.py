"""Python binding of libnkv, the MI355X (gfx950) NestedKV prefill compression pass.

Argument marshalling only: every step of the pass runs in the HIP kernels behind the C ABI declared in
``include/nkv.h``; the functions here have the same names as the C entry points.  torch is used to own
device memory and streams.  There is no fallback: if ``libnkv.so`` has not been built
(``python -m paper_2605_26678_amd.build``) importing the library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

from . import build as _build

NKV_OK = 0
NKV_EINVAL, NKV_ESHAPE, NKV_EWORKSPACE, NKV_EHIP, NKV_EUNSUPPORTED, NKV_ESCRATCH = -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_BYTES = 32 << 20
DTYPE_F32, DTYPE_BF16, DTYPE_F16, DTYPE_F8_E4M3 = 0, 1, 2, 3
FLAG_GENERIC_KERNELS = 1
FLAG_TWO_PASS_STABLE = 2
FLAG_DEFER_STABLE = 4
FLAG_NO_UNIT_SUMS = 8
FLAG_BUDGET_PER_HEAD = 16
FLAG_STATS_PER_HEAD = 32
FLAG_VECTOR_SCAN = 128
FLAG_SELECT_PER_HEAD = 64
FLAG_COMPACT_IN_PLACE = 256
PIN = 3.0e38

EXPORTS = ("nkv_params_default", "nkv_block_size", "nkv_k0", "nkv_m_safe", "nkv_m_p", "nkv_packed_rows",
           "nkv_workspace_bytes", "nkv_score", "nkv_score_raw", "nkv_budget", "nkv_budget_noalloc", "nkv_select_compact",
           "nkv_decode_workspace_bytes", "nkv_decode_attention", "nkv_copy_probe", "nkv_strerror", "nkv_version")
KERNELS = ("scan", "finalize", "budget", "select", "gather", "decode")
PASS_KERNELS = KERNELS[:5]          # the kernels of the compression pass itself


class nkv_params(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("window", C.c_int32), ("block_div", C.c_int32),
                ("block_min", C.c_int32), ("block_max", C.c_int32), ("n_sink", C.c_int32),
                ("gate_mode", C.c_int32), ("surprise_mode", C.c_int32), ("flags", C.c_uint32),
                ("scale_mask", C.c_int32), ("top_frac", C.c_double), ("prior", C.c_double * 3),
                ("beta", C.c_double), ("tau", C.c_double), ("kappa", C.c_double), ("safeguard", C.c_double),
                ("near_tol", C.c_double), ("prof_start", C.c_void_p * 6), ("prof_stop", C.c_void_p * 6),
                ("scan_counters", C.c_void_p)]


class nkv_shape(C.Structure):
    _fields_ = [("L", C.c_int32), ("H", C.c_int32), ("d", C.c_int32), ("dv", C.c_int32), ("dtype", C.c_int32),
                ("n_prompts", C.c_int32), ("cu_seqlens", C.POINTER(C.c_int32)),
                ("key_strides", C.POINTER(C.c_int64)), ("value_strides", C.POINTER(C.c_int64)),
                ("key_layer_offsets", C.POINTER(C.c_int64)), ("value_layer_offsets", C.POINTER(C.c_int64))]


class NkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        path = _build.library_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it with `python -m paper_2605_26678_amd.build`")
        L = C.CDLL(path)
        vp, i64, f64 = C.c_void_p, C.c_int64, C.c_double
        L.nkv_params_default.argtypes = [C.POINTER(nkv_params)]
        L.nkv_block_size.argtypes = [i64, C.POINTER(nkv_params)]
        L.nkv_block_size.restype = i64
        L.nkv_k0.argtypes = [i64, f64]
        L.nkv_k0.restype = i64
        L.nkv_m_safe.argtypes = [i64, f64]
        L.nkv_m_safe.restype = i64
        L.nkv_m_p.argtypes = [i64, f64]
        L.nkv_m_p.restype = i64
        L.nkv_packed_rows.argtypes = [C.POINTER(nkv_shape), C.POINTER(f64), C.POINTER(i64)]
        L.nkv_workspace_bytes.argtypes = [C.POINTER(nkv_shape), C.POINTER(nkv_params), C.POINTER(C.c_size_t)]
        L.nkv_score.argtypes = [vp, C.POINTER(nkv_shape), C.POINTER(nkv_params), vp, vp, C.c_size_t, vp]
        L.nkv_score_raw.argtypes = [vp, C.POINTER(nkv_shape), C.POINTER(nkv_params), vp, vp, C.c_size_t, vp]
        L.nkv_budget.argtypes = [vp, C.POINTER(nkv_shape), C.POINTER(nkv_params), C.POINTER(f64), vp, vp,
                                 C.c_size_t, vp]
        L.nkv_budget_noalloc.argtypes = [vp, C.POINTER(nkv_shape), C.POINTER(nkv_params), C.POINTER(f64), vp, vp]
        L.nkv_select_compact.argtypes = [vp, vp, vp, vp, C.POINTER(nkv_shape), C.POINTER(nkv_params), vp, vp, vp,
                                         vp, i64, vp, vp, C.c_size_t, vp]
        L.nkv_decode_workspace_bytes.argtypes = [C.POINTER(nkv_shape), C.c_int32, i64, C.POINTER(C.c_size_t)]
        L.nkv_decode_attention.argtypes = [vp, vp, vp, vp, i64, C.POINTER(nkv_shape), C.POINTER(nkv_params),
                                           C.c_int32, f64, vp, vp, vp, C.c_size_t, vp]
        L.nkv_copy_probe.argtypes = [vp, vp, C.c_size_t, vp]
        L.nkv_strerror.argtypes = [C.c_int]
        L.nkv_strerror.restype = C.c_char_p
        L.nkv_version.restype = C.c_int
        for name in EXPORTS:
            getattr(L, name)
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().nkv_strerror(int(status)).decode()


def params_default(**overrides) -> nkv_params:
    p = nkv_params()
    rc = lib().nkv_params_default(C.byref(p))
    if rc:
        raise NkvError(rc, "nkv_params_default")
    for k, v in overrides.items():
        if k == "prior":
            p.prior = (C.c_double * 3)(*v)
        else:
            if not hasattr(p, k):
                raise AttributeError(k)
            setattr(p, k, v)
    return p


def block_size(N: int, params: Optional[nkv_params] = None) -> int:
    p = params or params_default()
    return int(lib().nkv_block_size(int(N), C.byref(p)))


def k0(N: int, r: float) -> int:
    return int(lib().nkv_k0(int(N), float(r)))


def m_safe(k0_: int, safeguard: float = 0.20) -> int:
    return int(lib().nkv_m_safe(int(k0_), float(safeguard)))


def m_p(N: int, top_frac: float = 0.10) -> int:
    return int(lib().nkv_m_p(int(N), float(top_frac)))


class Shape:
    """Host-side description of keys[L][H][T][d] / values[L][H][T][dv] holding one or more prompts.
    ``key_strides`` / ``value_strides``: None for the dense layout, else (layer, head, prompt) strides in
    elements as ``nkv_shape`` in nkv.h defines them.  ``key_layers`` / ``value_layers``: None, or one tensor
    (or device address) per layer when every layer has a tensor of its own; the calls are then handed layer
    0's tensor."""

    def __init__(self, L: int, H: int, d: int, dv: int, dtype: int, cu_seqlens: Sequence[int],
                 key_strides: Optional[Sequence[int]] = None, value_strides: Optional[Sequence[int]] = None,
                 key_layers: Optional[Sequence] = None, value_layers: Optional[Sequence] = None):
        self.cu = (C.c_int32 * len(cu_seqlens))(*[int(x) for x in cu_seqlens])
        self.ks = None if key_strides is None else (C.c_int64 * 3)(*[int(x) for x in key_strides])
        self.vs = None if value_strides is None else (C.c_int64 * 3)(*[int(x) for x in value_strides])
        esize = {DTYPE_F32: 4, DTYPE_BF16: 2, DTYPE_F16: 2, DTYPE_F8_E4M3: 1}.get(int(dtype), 1)

        def offsets(layers):
            if layers is None:
                return None
            addr = [int(t) if isinstance(t, int) else int(t.data_ptr()) for t in layers]
            if len(addr) != int(L) or any((a - addr[0]) % esize for a in addr):
                raise ValueError("one tensor per layer, element-aligned")
            return (C.c_int64 * len(addr))(*[(a - addr[0]) // esize for a in addr])

        self.klo, self.vlo = offsets(key_layers), offsets(value_layers)
        self.c = nkv_shape(int(L), int(H), int(d), int(dv), int(dtype), len(cu_seqlens) - 1, self.cu,
                           self.ks, self.vs, self.klo, self.vlo)
        self.L, self.H, self.d, self.dv, self.dtype = int(L), int(H), int(d), int(dv), int(dtype)
        self.n_prompts = len(cu_seqlens) - 1
        self.T = int(cu_seqlens[-1])
        self.cu_seqlens = [int(x) for x in cu_seqlens]

    @property
    def n_units(self) -> int:
        return self.n_prompts * self.L * self.H


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


def packed_rows(shape: Shape, r_per_prompt: Sequence[float]) -> int:
    r = (C.c_double * shape.n_prompts)(*[float(x) for x in r_per_prompt])
    out = C.c_int64(0)
    rc = lib().nkv_packed_rows(C.byref(shape.c), r, C.byref(out))
    if rc:
        raise NkvError(rc, "nkv_packed_rows")
    return int(out.value)


def workspace_bytes(shape: Shape, params: Optional[nkv_params] = None) -> int:
    p = params or params_default()
    out = C.c_size_t(0)
    rc = lib().nkv_workspace_bytes(C.byref(shape.c), C.byref(p), C.byref(out))
    if rc:
        raise NkvError(rc, "nkv_workspace_bytes")
    return int(out.value)


def score(keys, shape: Shape, params: nkv_params, scores, ws, stream=None) -> None:
    """keys [L,H,T,d] (device) -> scores [L,H,T] fp32 (device), enqueued on ``stream``."""
    rc = lib().nkv_score(_ptr(keys), C.byref(shape.c), C.byref(params), _ptr(scores), _ptr(ws),
                         0 if ws is None else ws.numel() * ws.element_size(), _stream(stream))
    if rc:
        raise NkvError(rc, "nkv_score")


def score_raw(keys, shape: Shape, params: nkv_params, a_raw, ws, stream=None) -> None:
    """keys -> a_raw [3,L,H,T] fp32: the per-scale anomalies before normalisation."""
    rc = lib().nkv_score_raw(_ptr(keys), C.byref(shape.c), C.byref(params), _ptr(a_raw), _ptr(ws),
                             0 if ws is None else ws.numel() * ws.element_size(), _stream(stream))
    if rc:
        raise NkvError(rc, "nkv_score_raw")


def budget(scores, shape: Shape, params: nkv_params, r_per_prompt: Sequence[float], k_per_head, ws=None,
           stream=None) -> None:
    """scores [L,H,T] -> k_per_head [P,L,H] int32."""
    r = (C.c_double * shape.n_prompts)(*[float(x) for x in r_per_prompt])
    rc = lib().nkv_budget(_ptr(scores), C.byref(shape.c), C.byref(params), r, _ptr(k_per_head), _ptr(ws),
                          0 if ws is None else ws.numel() * ws.element_size(), _stream(stream))
    if rc:
        raise NkvError(rc, "nkv_budget")


def budget_noalloc(scores, shape: Shape, params: nkv_params, r_per_prompt: Sequence[float], k_per_head,
                   stream=None) -> None:
    """``budget`` on the library's own static scratch array (no workspace argument, nothing allocated)."""
    r = (C.c_double * shape.n_prompts)(*[float(x) for x in r_per_prompt])
    rc = lib().nkv_budget_noalloc(_ptr(scores), C.byref(shape.c), C.byref(params), r, _ptr(k_per_head),
                                  _stream(stream))
    if rc:
        raise NkvError(rc, "nkv_budget_noalloc")


def select_compact(keys, values, scores, k_per_head, shape: Shape, params: nkv_params, packed_k, packed_v,
                   kept_idx, head_off, row_capacity: int, near_threshold_count=None, ws=None, stream=None) -> None:
    """Top-B_h selection, ordered compaction and K/V gather; see ``nkv_select_compact`` in nkv.h."""
    rc = lib().nkv_select_compact(_ptr(keys), _ptr(values), _ptr(scores), _ptr(k_per_head), C.byref(shape.c),
                                  C.byref(params), _ptr(packed_k), _ptr(packed_v), _ptr(kept_idx), _ptr(head_off),
                                  int(row_capacity), _ptr(near_threshold_count), _ptr(ws),
                                  0 if ws is None else ws.numel() * ws.element_size(), _stream(stream))
    if rc:
        raise NkvError(rc, "nkv_select_compact")


def decode_workspace_bytes(shape: Shape, n_q_heads: int, rows: int) -> int:
    out = C.c_size_t(0)
    rc = lib().nkv_decode_workspace_bytes(C.byref(shape.c), int(n_q_heads), int(rows), C.byref(out))
    if rc:
        raise NkvError(rc, "nkv_decode_workspace_bytes")
    return int(out.value)


def decode_attention(q, packed_k, packed_v, head_off, rows: int, shape: Shape, params: nkv_params, n_q_heads: int,
                     scale: float, out, lse=None, ws=None, stream=None) -> None:
    """One new token's attention over the compressed cache: q [P,L,Hq,d] -> out [P,L,Hq,dv] fp32 (and lse
    [P,L,Hq]); see ``nkv_decode_attention`` in nkv.h."""
    rc = lib().nkv_decode_attention(_ptr(q), _ptr(packed_k), _ptr(packed_v), _ptr(head_off), int(rows),
                                    C.byref(shape.c), C.byref(params), int(n_q_heads), float(scale), _ptr(out),
                                    _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                    _stream(stream))
    if rc:
        raise NkvError(rc, "nkv_decode_attention")


def copy_probe(dst, src, stream=None) -> None:
    """Plain device copy src -> dst (same byte size), the bandwidth yardstick; dst None: loads only."""
    rc = lib().nkv_copy_probe(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream))
    if rc:
        raise NkvError(rc, "nkv_copy_probe")


_hip = None


def _hiprt() -> C.CDLL:
    global _hip
    if _hip is None:
        h = C.CDLL("libamdhip64.so")
        h.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        h.hipEventDestroy.argtypes = [C.c_void_p]
        h.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        h.hipEventSynchronize.argtypes = [C.c_void_p]
        h.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        _hip = h
    return _hip


class HipEvent:
    """A raw hipEvent_t, recorded by the library (kernel timing) or by the caller on a given stream."""

    def __init__(self):
        self.handle = C.c_void_p()
        rc = _hiprt().hipEventCreate(C.byref(self.handle))
        if rc:
            raise RuntimeError(f"hipEventCreate failed: {rc}")

    def record(self, stream=None) -> None:
        rc = _hiprt().hipEventRecord(self.handle, _stream(stream))
        if rc:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def synchronize(self) -> None:
        _hiprt().hipEventSynchronize(self.handle)

    def elapsed_ms(self, later: "HipEvent") -> float:
        ms = C.c_float(0)
        rc = _hiprt().hipEventElapsedTime(C.byref(ms), self.handle, later.handle)
        if rc:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def __del__(self):
        try:
            if self.handle:
                _hiprt().hipEventDestroy(self.handle)
        except Exception:
            pass


def with_kernel_timers(params: nkv_params, timers: dict) -> nkv_params:
    """A copy of ``params`` that asks the library to record ``timers[name] = (start, stop)`` HipEvents around
    the launch of the named kernel (names in KERNELS)."""
    q = nkv_params.from_buffer_copy(params)
    for name, (a, b) in timers.items():
        k = KERNELS.index(name)
        q.prof_start[k] = a.handle
        q.prof_stop[k] = b.handle
    return q


@dataclass
class Compressed:
    scores: "object"        # [L,H,T] fp32
    k_per_head: "object"    # [P,L,H] int32
    head_off: "object"      # [P*L*H+1] int64
    kept_idx: "object"      # [rows] int32
    packed_k: "object"      # [rows,d]
    packed_v: "object"      # [rows,dv]
    near_count: "object"    # [1] int64


class Compressor:
    """Owns the device buffers of one workload shape and runs the three calls back to back."""

    def __init__(self, shape: Shape, r_per_prompt: Sequence[float], params: Optional[nkv_params] = None,
                 device="cuda:0", kv_dtype=None):
        import torch
        self.torch = torch
        self.shape, self.params = shape, params or params_default()
        self.r = [float(x) for x in r_per_prompt]
        self.rows = packed_rows(shape, self.r)
        dev = torch.device(device)
        kv_dtype = kv_dtype or {DTYPE_F32: torch.float32, DTYPE_BF16: torch.bfloat16, DTYPE_F16: torch.float16,
                                DTYPE_F8_E4M3: torch.float8_e4m3fn}[shape.dtype]
        self.ws = torch.empty(max(workspace_bytes(shape, self.params), 256), dtype=torch.uint8, device=dev)
        self.scores = torch.empty(shape.L, shape.H, shape.T, dtype=torch.float32, device=dev)
        self.k_per_head = torch.empty(shape.n_prompts, shape.L, shape.H, dtype=torch.int32, device=dev)
        self.head_off = torch.empty(shape.n_units + 1, dtype=torch.int64, device=dev)
        self.kept_idx = torch.empty(max(self.rows, 1), dtype=torch.int32, device=dev)
        self.packed_k = torch.empty(max(self.rows, 1), shape.d, dtype=kv_dtype, device=dev)
        self.packed_v = torch.empty(max(self.rows, 1), shape.dv, dtype=kv_dtype, device=dev)
        self.near = torch.zeros(1, dtype=torch.int64, device=dev)

    def run(self, keys, values, stream=None) -> Compressed:
        score(keys, self.shape, self.params, self.scores, self.ws, stream)
        budget(self.scores, self.shape, self.params, self.r, self.k_per_head, self.ws, stream)
        select_compact(keys, values, self.scores, self.k_per_head, self.shape, self.params, self.packed_k,
                       self.packed_v, self.kept_idx, self.head_off, self.rows, self.near, self.ws, stream)
        return Compressed(self.scores, self.k_per_head, self.head_off, self.kept_idx[:self.rows],
                          self.packed_k[:self.rows], self.packed_v[:self.rows], self.near)
