"""Seeded synthetic key/value streams for the NestedKV compression pass.

This module only *draws inputs*.  It holds none of the method's arithmetic
(no normalisation, anchors, scores, budgets or selection) and is the one
piece of code shared by the CPU oracle's tests and the HIP path's tests and
benchmark.  torch is used as a seeded random-number source and as the owner
of the memory the tensors live in (CPU or GPU).

The streams stand in for the key caches of Qwen3 / Llama-3.2 prefill on the
long-context suites the paper evaluates on (Section 3.1, Table
"dataset-statistics"); neither the checkpoints nor the suites are available,
so keys are a mixture with the structure the method reacts to:

    k_i = 3 * u(i) + o_seg(i) + g_i,      g_i ~ N(0, I_d)

* ``u``      a random unit "mean direction" per (layer, head);
* ``o_seg``  one offset per 512-token segment, ``c`` times a random unit
             vector (c = 1.5, or one draw of U[0.5, 2] per layer);
* outliers   ``n_out`` positions >= 4, drawn without replacement, whose key is
             *replaced* by 6 times a unit Gaussian direction made orthogonal
             to ``u``;
* sinks      (optional) tokens 0..3 *replaced* by 10 * u;
* drift      (optional) u(i) = cos(phi_i) u + sin(phi_i) v with v a unit
             vector orthogonal to u and phi_i = 0.02 * i / 512 rad (continuous).

Values are N(0, 1).  bf16 workloads round K and V to bf16 (round to nearest
even) before anybody reads them.  A stream is a pure function of
(workload seed, prompt index, layer) and of the device type the generator
runs on (CPU and GPU generators give different, equally valid draws).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import torch

SEGMENT = 512


@dataclass(frozen=True)
class Workload:
    """Shape and mixture recipe of one synthetic workload."""

    name: str
    L: int
    H: int
    d: int
    dtype: str                      # "fp32" | "bf16" | "fp16" | "fp8" (8-bit E4M3, unscaled: the keys fit its range)
    prompt_lens: Tuple[int, ...]
    ratios: Tuple[float, ...]       # eviction ratios r the workload is run at
    n_out: int
    sinks: bool
    drift: bool
    per_layer_offset_norm: bool     # False: c = 1.5; True: c ~ U[0.5, 2] per layer
    seed: int
    dv: int = 0                     # 0 -> same as d

    @property
    def d_v(self) -> int:
        return self.dv or self.d

    @property
    def T(self) -> int:
        return int(sum(self.prompt_lens))

    @property
    def cu_seqlens(self) -> List[int]:
        cu = [0]
        for n in self.prompt_lens:
            cu.append(cu[-1] + int(n))
        return cu

    def torch_dtype(self) -> torch.dtype:
        return {"fp32": torch.float32, "bf16": torch.bfloat16, "fp16": torch.float16,
                "fp8": torch.float8_e4m3fn}[self.dtype]


WORKLOADS = {
    # tiny single-layer pass, fp32, the oracle finishes in seconds
    "tiny": Workload("tiny", 1, 2, 128, "fp32", (4096,), (0.5,), 16, False, False, False, 0),
    # Llama-3.2-1B-shaped prefill
    "llama1b_4k": Workload("llama1b_4k", 16, 8, 64, "bf16", (4096,), (0.5, 0.75), 64, False, False, True, 1),
    # Qwen3-4B-shaped prefill
    "qwen4b_16k": Workload("qwen4b_16k", 36, 8, 128, "bf16", (16384,), (0.75, 0.95), 128, True, False, True, 2),
    # Qwen3-4B-shaped long prefill (headline)
    "qwen4b_32k": Workload("qwen4b_32k", 36, 8, 128, "bf16", (32768,), (0.75,), 128, True, True, True, 3),
    # batched ragged serving shape, Llama-3.2-3B-shaped
    "llama3b_ragged": Workload(
        "llama3b_ragged", 28, 8, 128, "bf16",
        (4096, 8192, 16384, 32768, 32768, 16384, 8192, 4096), (0.95,), 128, True, True, True, 4),
    # beyond the paper's longest evaluated prompts (40k cap): the same Qwen3-4B shape at 40k and 128k tokens
    "qwen4b_40k": Workload("qwen4b_40k", 36, 8, 128, "bf16", (40960,), (0.75,), 128, True, True, True, 5),
    "qwen4b_128k": Workload("qwen4b_128k", 36, 8, 128, "bf16", (131072,), (0.75,), 128, True, True, True, 6),
    # the headline shape with an fp16 cache
    "qwen4b_32k_fp16": Workload("qwen4b_32k_fp16", 36, 8, 128, "fp16", (32768,), (0.75,), 128, True, True, True, 3),
    # the headline shape with an 8-bit (E4M3) cache
    "qwen4b_32k_fp8": Workload("qwen4b_32k_fp8", 36, 8, 128, "fp8", (32768,), (0.75,), 128, True, True, True, 3),
}


def small_workload(name: str, L: int, H: int, d: int, prompt_lens: Sequence[int], dtype: str = "bf16",
                   n_out: int = 8, sinks: bool = True, drift: bool = True, seed: int = 1234,
                   dv: int = 0) -> Workload:
    """An ad-hoc workload with the same mixture, for shape sweeps in tests."""
    return Workload(name, L, H, d, dtype, tuple(int(n) for n in prompt_lens), (0.5,), n_out, sinks, drift,
                    True, seed, dv)


def _gen(device: torch.device, *key: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for k in key:
        s = (s ^ (int(k) + 0x632BE59BD9B4E019)) * 0xBF58476D1CE4E5B9 % (1 << 63)
    g.manual_seed(s)
    return g


def _unit(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=-1, keepdim=True).clamp_min(1e-20)


def layer_keys_values(w: Workload, p: int, layer: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """K [H, N_p, d] and V [H, N_p, d_v] of prompt ``p`` at ``layer`` in the workload's dtype."""
    device = torch.device(device)
    N, H, d = int(w.prompt_lens[p]), w.H, w.d
    g = _gen(device, w.seed, p, layer)
    f32 = dict(dtype=torch.float32, device=device, generator=g)
    u = _unit(torch.randn(H, d, **f32))
    v = torch.randn(H, d, **f32)
    v = _unit(v - (v * u).sum(-1, keepdim=True) * u)
    nseg = (N + SEGMENT - 1) // SEGMENT
    c = 0.5 + 1.5 * torch.rand(1, **f32).item() if w.per_layer_offset_norm else 1.5
    off = c * _unit(torch.randn(H, nseg, d, **f32))
    keys = torch.randn(H, N, d, **f32)
    pos = torch.arange(N, device=device)
    seg = pos // SEGMENT
    if w.drift:
        phi = (0.02 / SEGMENT) * pos.to(torch.float32)
        ui = torch.cos(phi)[None, :, None] * u[:, None, :] + torch.sin(phi)[None, :, None] * v[:, None, :]
    else:
        ui = u[:, None, :].expand(H, N, d)
    keys += 3.0 * ui
    keys += off[:, seg, :]
    n_out = min(w.n_out, max(N - 4, 0))
    if n_out > 0:
        for h in range(H):
            perm = torch.randperm(N - 4, device=device, generator=g)[:n_out] + 4
            gdir = torch.randn(n_out, d, **f32)
            gdir = gdir - (gdir @ u[h])[:, None] * u[h][None, :]
            keys[h, perm] = 6.0 * _unit(gdir)
    if w.sinks:
        ns = min(4, N)
        keys[:, :ns, :] = 10.0 * u[:, None, :]
    values = torch.randn(H, N, w.d_v, **f32)
    dt = w.torch_dtype()
    return keys.to(dt), values.to(dt)


def make_kv(w: Workload, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Whole-workload tensors keys[L, H, T, d], values[L, H, T, d_v] (prompts concatenated along T)."""
    device = torch.device(device)
    dt = w.torch_dtype()
    K = torch.empty(w.L, w.H, w.T, w.d, dtype=dt, device=device)
    V = torch.empty(w.L, w.H, w.T, w.d_v, dtype=dt, device=device)
    cu = w.cu_seqlens
    for layer in range(w.L):
        for p in range(len(w.prompt_lens)):
            k, v = layer_keys_values(w, p, layer, device)
            K[layer, :, cu[p]:cu[p + 1]] = k
            V[layer, :, cu[p]:cu[p + 1]] = v
    return K, V


def recipe(w: Workload) -> dict:
    """Plain description of the mixture, recorded next to benchmark results."""
    return {
        "mixture": "k = 3*u(i) + o_seg(i) + N(0,I)", "segment": SEGMENT,
        "offset_norm": "U[0.5,2] per layer" if w.per_layer_offset_norm else 1.5,
        "outliers": f"{w.n_out}/head replaced by 6*unit orthogonal to u",
        "sinks": "tokens 0-3 replaced by 10*u" if w.sinks else "none",
        "drift": "0.02 rad per 512 tokens, continuous" if w.drift else "none",
        "values": "N(0,1)", "seed": w.seed,
    }


# ---------------------------------------------------------------------------------------------------------
# Inputs of the decode-side consumer (attention of one new token over a compressed cache).

def make_queries(w: Workload, n_q_heads: int, K: torch.Tensor) -> torch.Tensor:
    """q [P, L, n_q_heads, d] in the workload's dtype, one new token per prompt: Gaussian noise plus half of
    one randomly chosen key of the KV head the query head reads (j // G), so that the attention is peaked on
    a few positions the way a retrieving head's is.  K is keys[L, H, T, d] of the workload (any device)."""
    P, G = len(w.prompt_lens), n_q_heads // w.H
    g = _gen(K.device, w.seed, 424242)
    q = torch.randn(P, w.L, n_q_heads, w.d, dtype=torch.float32, device=K.device, generator=g)
    cu = w.cu_seqlens
    for p in range(P):
        j = torch.randint(0, int(w.prompt_lens[p]), (w.L, n_q_heads), device=K.device, generator=g) + cu[p]
        heads = (torch.arange(n_q_heads, device=K.device) // G)[None, :].expand(w.L, n_q_heads)
        layers = torch.arange(w.L, device=K.device)[:, None].expand(w.L, n_q_heads)
        q[p] += 0.5 * K[layers, heads, j].to(torch.float32)
    return q.to(w.torch_dtype())


def synthetic_head_lengths(w: Workload, r: float, seed: int = 0) -> torch.Tensor:
    """lens [P, L, H] (int64, CPU): retained rows per head with the structure head-wise budgets have -- every
    head of a layer gets a fifth of n = floor((1 - r) N) and the other four fifths of H * n are dealt to the
    heads by a seeded multinomial draw, so the lengths of a layer are ragged and add up to H * n."""
    P = len(w.prompt_lens)
    g = _gen(torch.device("cpu"), w.seed, seed, 515151)
    lens = torch.zeros(P, w.L, w.H, dtype=torch.int64)
    for p in range(P):
        N = int(w.prompt_lens[p])
        n = int((1.0 - r) * N + 1e-9)
        base = n // 5
        rest = w.H * (n - base)
        for l in range(w.L):
            share = torch.rand(w.H, generator=g) + 0.25
            part = torch.floor(share / share.sum() * rest).to(torch.int64)
            part[0] += rest - int(part.sum())
            lens[p, l] = torch.clamp(base + part, max=N)
    return lens


def synthetic_cache(w: Workload, K: torch.Tensor, V: torch.Tensor, lens: torch.Tensor, seed: int = 0):
    """A ragged cache with the layout the compression operator writes, without running it: for unit
    (p, l, h) a seeded random subset of lens[p, l, h] positions in ascending order, their K and V rows copied.
    Returns packed_k [rows, d], packed_v [rows, d_v], head_off [P*L*H + 1] int64 (on K's device)."""
    P = len(w.prompt_lens)
    g = _gen(K.device, w.seed, seed, 616161)
    cu = w.cu_seqlens
    flat = lens.reshape(-1)
    head_off = torch.zeros(flat.numel() + 1, dtype=torch.int64)
    head_off[1:] = torch.cumsum(flat, 0)
    rows = int(head_off[-1])
    pk = torch.empty(rows, w.d, dtype=K.dtype, device=K.device)
    pv = torch.empty(rows, w.d_v, dtype=V.dtype, device=K.device)
    u = 0
    for p in range(P):
        N = int(w.prompt_lens[p])
        for l in range(w.L):
            for h in range(w.H):
                n, o = int(flat[u]), int(head_off[u])
                idx = torch.sort(torch.randperm(N, device=K.device, generator=g)[:n]).values + cu[p]
                pk[o:o + n] = K[l, h, idx]
                pv[o:o + n] = V[l, h, idx]
                u += 1
    return pk, pv, head_off.to(K.device)
