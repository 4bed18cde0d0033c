"""Shared machinery of the GPU parity tests: run the HIP path through the C ABI, run the CPU oracle on the
same stored inputs, and compare element by element.

Bars (written here once, used by every parity test):
  * scores: |gpu - oracle| <= SCORE_TOL * max(1, |oracle|) on unpinned positions (scores live on a
    per-head [0,1] scale, fp32 accumulation against the oracle's fp64); pinned positions are equal;
  * nkv_budget and nkv_select_compact fed the ORACLE's fp32 scores (and budgets): k_per_head, head_off,
    kept_idx, packed K and packed V are bit-exact, no exceptions;
  * end to end (GPU scores -> GPU budgets -> GPU selection): a position may be kept by one side only if
    the oracle's score of it lies within NEAR_BAND = 1e-5 of the oracle's selection threshold of that head;
    such positions are counted and reported.  A head's budget may differ from the oracle's only by as many
    slots as the layer has scores within NEAR_BAND of the layer's admission threshold (the score of the last
    pool entry the oracle admits); the slots moved are counted and reported.  Packed rows always equal the
    input rows named by the GPU's own kept_idx.
"""
from __future__ import annotations

import numpy as np
import torch

import nkv_inputs
import oracle
import paper_2605_26678_amd as nkv

SCORE_TOL = 1e-5
NEAR_BAND = 1e-5


def oracle_params(params: nkv.nkv_params) -> oracle.Params:
    return oracle.Params(window=params.window, block_div=params.block_div, block_min=params.block_min,
                         block_max=params.block_max, n_sink=params.n_sink, gate_mode=params.gate_mode,
                         surprise_mode=params.surprise_mode, scale_mask=params.scale_mask or 7, top_frac=params.top_frac,
                         prior=tuple(params.prior), beta=params.beta, tau=params.tau, kappa=params.kappa,
                         safeguard=params.safeguard)


def shape_of(w: nkv_inputs.Workload) -> nkv.Shape:
    dtype = {"fp32": nkv.DTYPE_F32, "bf16": nkv.DTYPE_BF16, "fp16": nkv.DTYPE_F16, "fp8": nkv.DTYPE_F8_E4M3}[w.dtype]
    return nkv.Shape(w.L, w.H, w.d, w.d_v, dtype, w.cu_seqlens)


def bits(t: torch.Tensor) -> np.ndarray:
    """Bit pattern of a CPU/GPU tensor as a numpy integer array."""
    t = t.detach().cpu().contiguous()
    return t.view({1: torch.uint8, 2: torch.int16, 4: torch.int32}[t.element_size()]).numpy()


def check_scores(g: np.ndarray, o: np.ndarray, what: str) -> float:
    """g, o: [H, N] float32 of one prompt/layer.  Returns the worst error on unpinned positions."""
    pinned = o == oracle.PIN
    assert np.array_equal(g == oracle.PIN, pinned), f"{what}: pinned positions differ"
    err = np.abs(g.astype(np.float64) - o.astype(np.float64))
    err[pinned] = 0.0
    bound = SCORE_TOL * np.maximum(1.0, np.abs(o.astype(np.float64)))
    bad = np.argwhere(err > bound)
    assert bad.size == 0, f"{what}: {len(bad)} scores off by more than {SCORE_TOL}, worst {err.max():.3e} at {bad[0]}"
    return float(err.max())


def run_gpu(w: nkv_inputs.Workload, K: torch.Tensor, V: torch.Tensor, r, params=None, scores=None,
            k_per_head=None, use_ws=True):
    """The three ABI calls on cuda:0.  ``scores`` / ``k_per_head`` (device tensors) replace the library's own
    for stage-wise parity.  Returns the Compressed record (device tensors) after synchronising."""
    params = params or nkv.params_default()
    shape = shape_of(w)
    r = [r] * shape.n_prompts if np.isscalar(r) else list(r)
    comp = nkv.Compressor(shape, r, params)
    if scores is None:
        nkv.score(K, shape, params, comp.scores, comp.ws)
    else:
        comp.scores.copy_(scores)
    if k_per_head is None:
        nkv.budget(comp.scores, shape, params, r, comp.k_per_head, comp.ws if use_ws else None)
        rows = comp.rows
    else:
        comp.k_per_head.copy_(k_per_head)
        rows = int(k_per_head.sum().item())
        if rows > comp.rows:
            comp.kept_idx = torch.empty(rows, dtype=torch.int32, device=K.device)
            comp.packed_k = torch.empty(rows, shape.d, dtype=K.dtype, device=K.device)
            comp.packed_v = torch.empty(rows, shape.dv, dtype=V.dtype, device=K.device)
    nkv.select_compact(K, V, comp.scores, comp.k_per_head, shape, params, comp.packed_k, comp.packed_v,
                       comp.kept_idx, comp.head_off, rows, comp.near, comp.ws if use_ws else None)
    torch.cuda.synchronize()
    return nkv.Compressed(comp.scores, comp.k_per_head, comp.head_off, comp.kept_idx[:rows],
                          comp.packed_k[:rows], comp.packed_v[:rows], comp.near), shape


def oracle_layer(Kl: np.ndarray, r: float, op: oracle.Params):
    """Oracle on one prompt/layer: Kl [H, N, d] float32 -> scores, budgets, kept index lists."""
    s, _ = oracle.score_layer(Kl, op)
    B = oracle.budget_layer(s, r, op.safeguard)
    kept = [oracle.select_head(s[h], int(B[h])) for h in range(Kl.shape[0])]
    return s, B, kept


def near_threshold_count(s: np.ndarray, B: np.ndarray, tol: float) -> int:
    """Tokens within tol of their head's selection threshold (the B_h-th highest score), fp32 arithmetic."""
    n = 0
    for h in range(s.shape[0]):
        N = s.shape[1]
        if 0 < B[h] < N:
            t = np.sort(s[h])[::-1][B[h] - 1]
            n += int(np.sum(np.abs(s[h] - t) <= np.float32(tol)))
    return n


def layer_band_count(s: np.ndarray, B: np.ndarray, m_safe: int) -> int:
    """Scores of a layer within NEAR_BAND of the layer's admission threshold: the lowest score any head keeps
    beyond its protected m_safe, i.e. the score of the last pool entry admitted."""
    t = None
    for h in range(s.shape[0]):
        if B[h] > m_safe:
            th = float(np.sort(s[h])[::-1][B[h] - 1])
            t = th if t is None else min(t, th)
    if t is None:
        return 0
    return int(np.sum(np.abs(s.astype(np.float64) - t) <= NEAR_BAND))


def check_against_oracle(w, K, V, out, r, params=None, layers=None, label=""):
    """An output record of the three calls (device tensors, laid out as nkv.h says) against the oracle run on
    the dense keys K [L,H,T,d] and values V of workload w, on the given layers (all by default).

    Returns a dict of statistics (worst score error, near-threshold positions, mismatching positions)."""
    params = params or nkv.params_default()
    op = oracle_params(params)
    shape = shape_of(w)
    r_list = [r] * shape.n_prompts if np.isscalar(r) else list(r)
    layers = range(w.L) if layers is None else layers
    g_scores = out.scores.cpu().numpy()
    g_B = out.k_per_head.cpu().numpy()
    g_off = out.head_off.cpu().numpy()
    g_idx = out.kept_idx.cpu().numpy()
    cu = w.cu_seqlens
    stats = dict(worst=0.0, flipped=0, budget_moved=0, units=0, near_gpu=int(out.near_count.item()))
    # layout invariants over the whole output
    assert g_off[0] == 0 and np.all(np.diff(g_off) == g_B.reshape(-1))
    for p in range(shape.n_prompts):
        k0 = oracle.k0(cu[p + 1] - cu[p], r_list[p])
        assert np.all(g_B[p].sum(axis=1) == w.H * k0), "budgets of a layer must add up to H*k0"
        assert g_B[p].min() >= oracle.m_safe(k0, params.safeguard)
    assert g_off[-1] == nkv.packed_rows(shape, r_list) == g_idx.shape[0]
    pk, pv = bits(out.packed_k), bits(out.packed_v)
    for l in layers:
        Kb, Vb = {l: bits(K[l])}, {l: bits(V[l])}          # only the compared layers travel to the host
        for p in range(shape.n_prompts):
            lo, hi = cu[p], cu[p + 1]
            Kl = K[l, :, lo:hi].cpu().float().numpy()     # converted on the host, also 8-bit keys
            s, B, kept = oracle_layer(Kl, r_list[p], op)
            what = f"{label} prompt {p} layer {l}"
            stats["worst"] = max(stats["worst"], check_scores(g_scores[l, :, lo:hi], s, what))
            moved = int(np.abs(g_B[p, l] - B).sum())
            if moved:
                k0 = oracle.k0(hi - lo, r_list[p])
                band = layer_band_count(s, B, oracle.m_safe(k0, params.safeguard))
                assert moved <= band, (f"{what}: budgets moved by {moved} slots although only {band} scores lie "
                                       f"within {NEAR_BAND} of the layer's admission threshold")
            stats["budget_moved"] += moved
            for h in range(w.H):
                u = (p * w.L + l) * w.H + h
                gi = g_idx[g_off[u]:g_off[u + 1]]
                assert np.all(np.diff(gi) > 0), f"{what} head {h}: kept_idx not ascending"
                assert gi.size == 0 or (gi[0] >= 0 and gi[-1] < hi - lo)
                # packed rows are the input rows named by kept_idx, bit for bit
                assert np.array_equal(pk[g_off[u]:g_off[u + 1]], Kb[l][h, lo:hi][gi]), f"{what} head {h}: packed K"
                assert np.array_equal(pv[g_off[u]:g_off[u + 1]], Vb[l][h, lo:hi][gi]), f"{what} head {h}: packed V"
                diff = np.setxor1d(gi, kept[h])
                if diff.size:
                    # thresholds that matter for a position kept by one side only: the head's own cut on either
                    # side's budget (they differ when the layer's competition moved a slot)
                    srt = np.sort(s[h])[::-1]
                    cuts = [float(srt[min(max(int(b), 1), hi - lo) - 1]) for b in (B[h], g_B[p, l, h])]
                    sd = s[h][diff].astype(np.float64)
                    gap = np.minimum(np.abs(sd - cuts[0]), np.abs(sd - cuts[1]))
                    assert gap.max() <= NEAR_BAND, (f"{what} head {h}: position {diff[gap.argmax()]} kept by one "
                                                    f"side only although {gap.max():.2e} away from the threshold")
                    stats["flipped"] += int(diff.size)
                stats["units"] += 1
    return stats


def compare_end_to_end(w, K, V, r, params=None, layers=None, label=""):
    """Full-pass parity of the HIP path (dense layout) against the oracle on the given layers (all by default)."""
    out, _ = run_gpu(w, K, V, r, params)
    return check_against_oracle(w, K, V, out, r, params, layers, label)


def sub_layers(w, K, V, layers):
    """The workload restricted to some layers (contiguous copies), for stage parity at full per-layer size."""
    import dataclasses
    idx = torch.tensor(list(layers), device=K.device)
    return dataclasses.replace(w, L=len(layers)), K.index_select(0, idx).contiguous(), V.index_select(0, idx).contiguous()


def compare_stages(w, K, V, r, params=None, layers=None, label=""):
    """nkv_budget and nkv_select_compact fed the oracle's scores / budgets: bit-exact."""
    params = params or nkv.params_default()
    op = oracle_params(params)
    shape = shape_of(w)
    r_list = [r] * shape.n_prompts if np.isscalar(r) else list(r)
    if layers is not None:                                  # whole layers of a large workload, at their real shape
        w, K, V = sub_layers(w, K, V, layers)
        shape = shape_of(w)
    Kf = K.cpu().float().numpy()
    ref = oracle.compress(Kf, bits(K), bits(V), w.cu_seqlens, r_list, op)
    out, _ = run_gpu(w, K, V, r, params, scores=torch.from_numpy(ref.scores).to(K.device))
    assert np.array_equal(out.k_per_head.cpu().numpy(), ref.k_per_head), f"{label}: budgets differ"
    assert np.array_equal(out.head_off.cpu().numpy(), ref.head_off), f"{label}: head_off differs"
    assert np.array_equal(out.kept_idx.cpu().numpy(), ref.kept_idx), f"{label}: kept_idx differs"
    assert np.array_equal(bits(out.packed_k), ref.packed_k), f"{label}: packed K differs"
    assert np.array_equal(bits(out.packed_v), ref.packed_v), f"{label}: packed V differs"
    exp_near = 0
    cu = w.cu_seqlens
    for p in range(shape.n_prompts):
        for l in range(w.L):
            exp_near += near_threshold_count(ref.scores[l, :, cu[p]:cu[p + 1]], ref.k_per_head[p, l], params.near_tol)
    assert int(out.near_count.item()) == exp_near, f"{label}: near-threshold count {int(out.near_count.item())} != {exp_near}"
    return ref
