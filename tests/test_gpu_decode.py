"""Parity of the decode-side consumer (nkv_decode_attention, through the C ABI) against oracle/decode.py.

The cache a test feeds to both sides never comes from the HIP path: small cases take the CPU oracle's own
compression of a seeded workload, the full-size case a synthetic ragged cache drawn by nkv_inputs.

Bar: |out - oracle| <= DECODE_TOL * max(1, max|V|) and |lse - oracle| <= DECODE_TOL * max(1, |lse|).  The
kernel forms <q, k> from exact bf16 products accumulated in fp32 (d terms, rounding ~ sqrt(d) ulp of the
logit, logits of a few tens at most -> ~1e-5 absolute in the exponent at worst), uses the hardware's base-2
exponential (1 ulp) and fp32 running sums over the rows; the output is a convex combination of value rows,
so a relative weight error e gives at most e * max|V|.
"""
import numpy as np
import pytest
import torch

import nkv_inputs
import oracle
from oracle.decode import decode_attention as oracle_decode
import paper_2605_26678_amd as nkv
from parity_util import oracle_params, shape_of

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DECODE_TOL = 1e-5


def _f64(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def _run(w, q, pk, pv, head_off, rows, Hq, scale, want_lse=True):
    shape, params = shape_of(w), nkv.params_default()
    P = len(w.prompt_lens)
    ws = torch.empty(max(nkv.decode_workspace_bytes(shape, Hq, rows), 256), dtype=torch.uint8, device=DEV)
    out = torch.full((P, w.L, Hq, w.d_v), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((P, w.L, Hq), float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    nkv.decode_attention(q, pk, pv, head_off, rows, shape, params, Hq, scale, out, lse, ws)
    torch.cuda.synchronize()
    return out, lse


def _check(out, lse, o_out, o_lse, vmax, what):
    err = np.abs(out.cpu().numpy().astype(np.float64) - o_out).max()
    assert err <= DECODE_TOL * max(1.0, vmax), f"{what}: out off by {err:.3e}"
    if lse is not None:
        g = lse.cpu().numpy().astype(np.float64)
        fin = np.isfinite(o_lse)
        assert np.array_equal(np.isneginf(g), np.isneginf(o_lse)), what
        e2 = np.abs(g[fin] - o_lse[fin]) / np.maximum(1.0, np.abs(o_lse[fin]))
        assert e2.size == 0 or e2.max() <= DECODE_TOL, f"{what}: lse off by {e2.max():.3e}"
    return err


CASES = [
    # name, L, H, d, dv, lens, dtype, Hq, r
    ("qwen_like_g4", 2, 2, 128, 0, [1500, 300], "bf16", 8, 0.5),
    ("llama1b_like_d64_g4", 1, 2, 64, 0, [1100], "bf16", 8, 0.5),
    ("llama3b_like_g3", 1, 2, 128, 0, [900], "bf16", 6, 0.75),
    ("mha_g1", 1, 3, 128, 0, [700], "bf16", 3, 0.5),
    ("g8", 1, 1, 64, 0, [800], "bf16", 8, 0.25),
    ("keep_all", 1, 2, 128, 0, [513, 256], "bf16", 4, 0.0),
    ("keep_none", 1, 2, 128, 0, [300], "bf16", 4, 1.0),
    ("generic_fp32", 1, 2, 64, 0, [400], "fp32", 4, 0.5),
    ("generic_dv_differs", 1, 2, 128, 64, [500], "bf16", 4, 0.5),
    ("generic_d40", 1, 2, 40, 24, [300], "fp32", 2, 0.5),
    ("generic_g12", 1, 1, 64, 0, [300], "bf16", 12, 0.5),
    ("fp16_g4", 1, 2, 128, 0, [1500, 300], "fp16", 8, 0.5),
    ("fp16_d64_g2", 1, 2, 64, 0, [600], "fp16", 4, 0.5),
    ("generic_fp16_dv", 1, 2, 128, 64, [600], "fp16", 4, 0.5),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_decode_over_the_oracles_compressed_cache(case):
    name, L, H, d, dv, lens, dtype, Hq, r = case
    w = nkv_inputs.small_workload(name, L, H, d, lens, dtype=dtype, dv=dv)
    K, V = nkv_inputs.make_kv(w, "cpu")
    raw = torch.int32 if dtype == "fp32" else torch.int16
    comp = oracle.compress(K.float().numpy(), K.view(raw).numpy(), V.view(raw).numpy(), w.cu_seqlens,
                           [r] * len(lens), oracle_params(nkv.params_default()))
    pk = torch.from_numpy(comp.packed_k).view(K.dtype)
    pv = torch.from_numpy(comp.packed_v).view(V.dtype)
    head_off = torch.from_numpy(comp.head_off)
    rows = int(head_off[-1])
    q = nkv_inputs.make_queries(w, Hq, K)
    scale = 1.0 / np.sqrt(d)
    o_out, o_lse = oracle_decode(_f64(q), _f64(pk), _f64(pv), comp.head_off, H, scale)
    if rows == 0:                                        # nothing kept: the buffers may be empty
        pk, pv = torch.zeros(1, d, dtype=K.dtype), torch.zeros(1, w.d_v, dtype=V.dtype)
    out, lse = _run(w, q.to(DEV), pk.to(DEV), pv.to(DEV), head_off.to(DEV), rows, Hq, scale)
    err = _check(out, lse, o_out, o_lse, float(_f64(pv).__abs__().max()), name)
    print(f"\n[{name}] rows {rows}, worst |out - oracle| {err:.2e}")


def test_chunk_boundaries_empty_units_and_clamped_offsets():
    """Unit lengths around the 256-row chunk size, an empty unit in the middle, and a cache that holds fewer
    rows than head_off claims (entries are clamped to `rows`)."""
    lens = [1, 255, 256, 257, 0, 512, 513, 3]
    w = nkv_inputs.small_workload("edges", 2, 4, 128, [600])
    K, V = nkv_inputs.make_kv(w, "cpu")
    L = torch.tensor(lens, dtype=torch.int64).reshape(1, 2, 4)
    pk, pv, head_off = nkv_inputs.synthetic_cache(w, K, V, L)
    q = nkv_inputs.make_queries(w, 16, K)
    for rows in (int(head_off[-1]), 1000):
        ho = head_off.numpy().clip(max=rows)
        o_out, o_lse = oracle_decode(_f64(q), _f64(pk[:rows]), _f64(pv[:rows]), ho, 4, 0.1)
        out, lse = _run(w, q.to(DEV), pk[:rows].to(DEV).contiguous(), pv[:rows].to(DEV).contiguous(),
                        head_off.to(DEV), rows, 16, 0.1)
        _check(out, lse, o_out, o_lse, float(_f64(pv).__abs__().max()), f"edges rows={rows}")
    out2, _ = _run(w, q.to(DEV), pk.to(DEV), pv.to(DEV), head_off.to(DEV), int(head_off[-1]), 16, 0.1, want_lse=False)
    assert torch.isfinite(out2).all()


def test_decode_is_deterministic():
    w = nkv_inputs.small_workload("det", 1, 2, 128, [3000])
    K, V = nkv_inputs.make_kv(w, DEV)
    lens = nkv_inputs.synthetic_head_lengths(w, 0.5)
    pk, pv, head_off = nkv_inputs.synthetic_cache(w, K, V, lens)
    q = nkv_inputs.make_queries(w, 8, K)
    a, la = _run(w, q, pk, pv, head_off, pk.shape[0], 8, 0.09)
    b, lb = _run(w, q, pk, pv, head_off, pk.shape[0], 8, 0.09)
    assert torch.equal(a, b) and torch.equal(la, lb)


def test_headline_size_cache_sampled_units():
    """The launch configuration the benchmark times (36 x 8 heads, 32k-token prompt, a quarter retained,
    32 query heads): every output is computed, the oracle checks sampled (layer, query head) pairs."""
    w = nkv_inputs.WORKLOADS["qwen4b_32k"]
    K, V = nkv_inputs.make_kv(w, DEV)
    lens = nkv_inputs.synthetic_head_lengths(w, 0.75)
    assert int(lens.sum()) == w.L * w.H * 8192 and int(lens.min()) < int(lens.max())
    pk, pv, head_off = nkv_inputs.synthetic_cache(w, K, V, lens)
    Hq, G = 32, 4
    q = nkv_inputs.make_queries(w, Hq, K)
    scale = 1.0 / np.sqrt(w.d)
    out, lse = _run(w, q, pk, pv, head_off, pk.shape[0], Hq, scale)
    assert torch.isfinite(out).all() and torch.isfinite(lse).all()
    ho = head_off.cpu().numpy()
    rng = np.random.default_rng(0)
    worst = 0.0
    for l, j in [(0, 0), (35, 31)] + [(int(rng.integers(36)), int(rng.integers(32))) for _ in range(10)]:
        u = l * w.H + j // G
        a, b = int(ho[u]), int(ho[u + 1])
        o_out, o_lse = oracle_decode(_f64(q[:, l:l + 1, j:j + 1]), _f64(pk[a:b]), _f64(pv[a:b]), np.array([0, b - a]),
                                     1, scale)
        worst = max(worst, _check(out[:, l:l + 1, j:j + 1], lse[:, l:l + 1, j:j + 1], o_out, o_lse,
                                  float(pv[a:b].abs().max()), f"layer {l} query head {j}"))
    print(f"\n[decode qwen4b_32k] rows {pk.shape[0]}, sampled worst |out - oracle| {worst:.2e}")
