"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars are defined in tests/parity_util.py.  Sizes: the small workloads are compared in full; the 16k workload
runs at full size and is compared on sampled layers; the 32k headline and the ragged batch run at full size in
the launch configuration bench.py times and are compared on every layer, plus bit-exact stage parity on two
whole layers at their real shape."""
import numpy as np
import pytest
import torch

import nkv_inputs
import oracle
import paper_2605_26678_amd as nkv
from parity_util import (SCORE_TOL, bits, check_against_oracle, compare_end_to_end, compare_stages, oracle_params,
                         run_gpu, shape_of)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _kv(w, device=DEV):
    K, V = nkv_inputs.make_kv(w, device)
    return K.contiguous(), V.contiguous()


def _report(name, st):
    print(f"\n[{name}] worst score err {st['worst']:.2e}; units {st['units']}; positions kept by one side only "
          f"{st['flipped']}; budget moved by {st['budget_moved']}; near-threshold (GPU count) {st['near_gpu']}")


# ------------------------------------------------------------------ the named workloads
def test_tiny_fp32_full():
    w = nkv_inputs.WORKLOADS["tiny"]
    K, V = _kv(w)
    compare_stages(w, K, V, 0.5, label="tiny")
    _report("tiny", compare_end_to_end(w, K, V, 0.5, label="tiny"))


@pytest.mark.parametrize("r", [0.5, 0.75])
def test_llama1b_4k_full(r):
    w = nkv_inputs.WORKLOADS["llama1b_4k"]
    K, V = _kv(w)
    compare_stages(w, K, V, r, label=f"llama1b r={r}")
    _report(f"llama1b_4k r={r}", compare_end_to_end(w, K, V, r, label="llama1b"))


@pytest.mark.parametrize("r", [0.75, 0.95])
def test_qwen4b_16k_sampled_layers(r):
    w = nkv_inputs.WORKLOADS["qwen4b_16k"]
    K, V = _kv(w)
    _report(f"qwen4b_16k r={r}", compare_end_to_end(w, K, V, r, layers=[0, 17, 35], label="qwen16k"))


def test_qwen4b_32k_headline_all_layers():
    w = nkv_inputs.WORKLOADS["qwen4b_32k"]
    K, V = _kv(w)
    _report("qwen4b_32k r=0.75", compare_end_to_end(w, K, V, 0.75, label="qwen32k"))
    compare_stages(w, K, V, 0.75, layers=[5, 30], label="qwen32k stages")    # H=8, N=32768, k0=8192, 4 slices


def test_ragged_batch_all_layers():
    w = nkv_inputs.WORKLOADS["llama3b_ragged"]
    K, V = _kv(w)
    _report("llama3b_ragged r=0.95", compare_end_to_end(w, K, V, 0.95, label="ragged"))
    compare_stages(w, K, V, 0.95, layers=[3, 21], label="ragged stages")


# ------------------------------------------------------------------ shape sweep, ragged tails, degenerate cases
SWEEP = [
    # name, L, H, d, prompt_lens, dtype, dv
    ("one_token", 1, 1, 64, [1], "bf16", 0),
    ("below_sinks", 1, 2, 64, [3], "bf16", 0),
    ("below_window", 2, 2, 128, [37], "bf16", 0),
    ("one_short_block", 1, 3, 128, [100], "bf16", 0),
    ("block_tail", 2, 2, 128, [130], "bf16", 0),
    ("odd_len_64", 1, 4, 64, [1000], "bf16", 0),
    ("b_between", 1, 2, 128, [6400], "bf16", 0),          # b = 200, not a multiple of 64
    ("b_255", 1, 1, 128, [8191], "bf16", 0),
    ("ragged_small", 2, 2, 128, [5, 700, 64, 4133, 129], "bf16", 0),
    ("dv_differs", 1, 2, 128, [777], "bf16", 64),
    ("fp32_d64", 1, 2, 64, [900], "fp32", 0),
    ("fp32_ragged", 1, 2, 128, [300, 513], "fp32", 0),
    ("wide_head", 1, 1, 256, [600], "bf16", 0),
    ("d_40", 1, 2, 40, [500], "fp32", 24),
    ("fp16_ragged", 2, 2, 128, [700, 300], "fp16", 0),
    ("fp16_long", 1, 2, 128, [20000, 4133, 6400], "fp16", 0),   # fp16 keys through the matrix-core scan: several slices, b = 200
    ("fp8_d128", 1, 2, 128, [2000, 130], "fp8", 0),       # 8-bit E4M3 keys and values
    ("fp8_d64_dv", 2, 3, 64, [900], "fp8", 32),
    ("long_prompt", 1, 2, 64, [40000], "bf16", 0),        # beyond the register-resident per-head kernels
    ("many_heads", 1, 12, 64, [600, 90], "bf16", 0),      # beyond the 8-head layer budget kernels
    ("heads_32", 2, 32, 64, [1500, 90], "bf16", 0),       # the most heads a layer may have
    ("heads_16_long", 1, 16, 128, [20000], "bf16", 0),
    ("slice_edges", 1, 2, 128, [8193, 16385, 100, 24576], "bf16", 0),   # one token past a slice, exact slices
    ("slices_d64", 1, 3, 64, [17000], "bf16", 0),
    ("nine_slices", 1, 2, 128, [70000, 9000], "bf16", 0), # 274 blocks in the unit: two rounds of the dies' runs;
                                                          # more than the matrix-core scan takes: vector scan
    ("unit_256_blocks", 1, 2, 128, [65533, 300], "bf16", 0),   # the longest unit the matrix-core scan takes
    ("units_4096", 16, 8, 64, [60] * 31 + [9000], "bf16", 0),  # slice-wise selection, which also places the units in the output
    ("units_4224", 33, 8, 64, [50 + i for i in range(16)], "bf16", 0),   # more units than it places: the scan kernel in front
]


@pytest.mark.parametrize("case", SWEEP, ids=[c[0] for c in SWEEP])
@pytest.mark.parametrize("r", [0.5, 0.9])
def test_shape_sweep(case, r):
    name, L, H, d, lens, dtype, dv = case
    w = nkv_inputs.small_workload(name, L, H, d, lens, dtype=dtype, dv=dv, n_out=min(8, max(min(lens) - 4, 0)))
    K, V = _kv(w)
    compare_stages(w, K, V, r, label=name)
    compare_end_to_end(w, K, V, r, label=name)


@pytest.mark.parametrize("flags", [0, nkv.FLAG_GENERIC_KERNELS, nkv.FLAG_TWO_PASS_STABLE, nkv.FLAG_DEFER_STABLE])
def test_8bit_keys_of_every_finite_code(flags):
    """Keys and values made of uniformly random bytes (every finite E4M3 code, both zeros, subnormals, the
    largest values; the two NaN codes are replaced): the streaming kernels' load-time conversion, on each of
    their routes, and the generic kernels' decoder both have to agree with the oracle, which is fed the values
    the format's definition gives."""
    w = nkv_inputs.small_workload("fp8_codes", 2, 2, 128, [1500, 200], dtype="fp8")
    g = torch.Generator().manual_seed(99)
    def rand_codes(*shape):
        b = torch.randint(0, 256, shape, dtype=torch.uint8, generator=g)
        b[(b & 0x7f) == 0x7f] -= 1
        return b.view(torch.float8_e4m3fn).to(DEV)
    K, V = rand_codes(w.L, w.H, w.T, w.d), rand_codes(w.L, w.H, w.T, w.d_v)
    assert len(torch.unique(K.view(torch.uint8))) == 254
    st = compare_end_to_end(w, K, V, 0.5, params=nkv.params_default(flags=flags), label=f"fp8 codes flags={flags}")
    _report(f"fp8 codes flags={flags}", st)


@pytest.mark.parametrize("case", range(16))
def test_random_shapes_dtypes_and_routes(case):
    """Seeded random draws of layers, heads, head dim, value dim, element type, prompt lengths (from a single token to
    40 000, one to five prompts), eviction ratio (0 and 1 included) and code route: end to end and stage-wise
    against the oracle."""
    import random
    rnd = random.Random(7000 + case)
    dtype = rnd.choice(["bf16", "bf16", "fp16", "fp8", "fp32"])
    d = rnd.choice([64, 128, 128])
    L, H = rnd.randint(1, 3), rnd.choice([1, 2, 3, 4, 8])
    lens = []
    for _ in range(rnd.choice([1, 1, 2, 3, 5])):
        kind = rnd.random()
        lens.append(rnd.randint(1, 300) if kind < 0.2 else rnd.randint(300, 9000) if kind < 0.7 else rnd.randint(9000, 40000))
    if sum(lens) * L * H > 600000:
        L, H = 1, min(H, 2)
    dv = rnd.choice([0, 0, 64, 32]) if dtype != "fp8" else rnd.choice([0, 32])
    r = rnd.choice([0.0, 0.3, 0.5, 0.75, 0.9, 0.97, 1.0])
    flags = rnd.choice([0, 0, 0, nkv.FLAG_VECTOR_SCAN, nkv.FLAG_DEFER_STABLE, nkv.FLAG_TWO_PASS_STABLE,
                        nkv.FLAG_SELECT_PER_HEAD, nkv.FLAG_STATS_PER_HEAD, nkv.FLAG_BUDGET_PER_HEAD])
    if flags in (nkv.FLAG_SELECT_PER_HEAD, nkv.FLAG_STATS_PER_HEAD, nkv.FLAG_BUDGET_PER_HEAD) and max(lens) > 32768:
        flags = 0
    label = f"random {case}: L={L} H={H} d={d} dv={dv} {dtype} lens={lens} r={r} flags={flags}"
    print(label, flush=True)
    w = nkv_inputs.small_workload(f"random{case}", L, H, d, lens, dtype=dtype, dv=dv, n_out=min(8, max(min(lens) - 4, 0)),
                                  seed=7000 + case)
    K, V = _kv(w)
    p = nkv.params_default(flags=flags)
    compare_end_to_end(w, K, V, r, params=p, label=label)
    compare_stages(w, K, V, r, params=p, label=label)


TILE_CASES = ["below_window", "one_short_block", "block_tail", "b_between", "b_255", "ragged_small", "dv_differs",
              "slice_edges", "unit_256_blocks", "fp16_ragged", "fp16_long"]


@pytest.mark.parametrize("route", [0, nkv.FLAG_DEFER_STABLE, nkv.FLAG_NO_UNIT_SUMS])
@pytest.mark.parametrize("name", TILE_CASES)
def test_vector_scan_where_the_matrix_core_scan_is_the_default(name, route):
    """bf16 and fp16 keys of head dim 128 take the matrix-core formulation of the fused scan by default (the sweep and the
    named workloads exercise it); the vector-unit formulation, forced by flag, on the same shapes and on its
    three routes (unit sum found in time, every block deferred, every unit sum from the repair kernel), against
    the oracle."""
    _, L, H, d, lens, dtype, dv = next(c for c in SWEEP if c[0] == name)
    w = nkv_inputs.small_workload(name, L, H, d, lens, dtype=dtype, dv=dv, n_out=min(8, max(min(lens) - 4, 0)))
    K, V = _kv(w)
    st = compare_end_to_end(w, K, V, 0.5, params=nkv.params_default(flags=nkv.FLAG_VECTOR_SCAN | route),
                            label=f"vector {name} route={route}")
    _report(f"vector {name} route={route}", st)


LIMITS = [
    # the most prompts, head dims, heads and (layer, head) pairs a call accepts
    ("prompts_64", 1, 2, 64, [61 + 37 * (i % 9) + 500 * (i % 3 == 0) for i in range(64)], "bf16", 0),
    ("d_1024", 1, 1, 1024, [400], "bf16", 8),
    ("dv_1024", 1, 1, 64, [700], "bf16", 1024),
    ("d_1024_fp32", 1, 2, 1024, [300, 40], "fp32", 1024),
    ("units_65535", 2114, 31, 64, [5], "bf16", 0),        # L * H = 65534
]


@pytest.mark.parametrize("case", LIMITS, ids=[c[0] for c in LIMITS])
def test_documented_limits(case):
    name, L, H, d, lens, dtype, dv = case
    w = nkv_inputs.small_workload(name, L, H, d, lens, dtype=dtype, dv=dv, n_out=0, sinks=False)
    K, V = _kv(w)
    layers = None if L <= 4 else [0, 1, L // 2, L - 1]
    if layers is None:
        compare_stages(w, K, V, 0.5, label=name)
    compare_end_to_end(w, K, V, 0.5, layers=layers, label=name)


@pytest.mark.parametrize("r", [0.0, 1.0])
def test_keep_everything_and_keep_nothing(r):
    w = nkv_inputs.small_workload("extremes", 2, 2, 128, [300, 77])
    K, V = _kv(w)
    ref = compare_stages(w, K, V, r, label=f"r={r}")
    out, shape = run_gpu(w, K, V, r)
    if r == 0.0:                                    # every token kept, packed == input, bit for bit
        for p, (lo, hi) in enumerate(zip(w.cu_seqlens[:-1], w.cu_seqlens[1:])):
            for l in range(w.L):
                for h in range(w.H):
                    u = (p * w.L + l) * w.H + h
                    o = int(out.head_off[u])
                    assert np.array_equal(bits(out.packed_k[o:o + hi - lo]), bits(K[l, h, lo:hi]))
                    assert np.array_equal(bits(out.packed_v[o:o + hi - lo]), bits(V[l, h, lo:hi]))
    else:
        assert int(out.head_off[-1]) == 0 and out.kept_idx.numel() == 0


def test_constant_keys_ties_resolve_by_index():
    w = nkv_inputs.small_workload("const", 1, 2, 64, [40])
    K = torch.full((1, 2, 40, 64), 0.37, dtype=torch.bfloat16, device=DEV)
    V = torch.randn(1, 2, 40, 64, device=DEV).to(torch.bfloat16)
    out, _ = run_gpu(w, K, V, 0.5)
    assert out.k_per_head.reshape(-1).tolist() == [36, 4]
    assert out.kept_idx.tolist() == list(range(36)) + [0, 1, 2, 3]
    assert torch.all(out.scores[:, :, 4:] == 0)


def test_fp16_unit_sum_beyond_the_formats_range():
    """65 533 fp16 keys that all point along one axis: that component of the unit's sum is 65 533, more than fp16
    holds, and the matrix-core scan stages its anchors as fp16 terms.  The stable anomaly of every token is -1."""
    N = 65533
    w = nkv_inputs.small_workload("fp16_axis", 1, 1, 128, [N], dtype="fp16")
    K = torch.zeros(1, 1, N, 128, dtype=torch.float16, device=DEV)
    K[..., 5] = torch.linspace(0.5, 3.0, N, device=DEV).to(torch.float16)
    shape = shape_of(w)
    p = nkv.params_default()
    a = torch.empty(3, 1, 1, N, dtype=torch.float32, device=DEV)
    ws = torch.empty(nkv.workspace_bytes(shape, p), dtype=torch.uint8, device=DEV)
    nkv.score_raw(K, shape, p, a, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(a).all()
    assert (a + 1.0).abs().max().item() < 2e-6


@pytest.mark.parametrize("H,flags", [(4, 0), (12, 0), (12, nkv.FLAG_BUDGET_PER_HEAD), (32, 0)])
def test_heavy_ties_stage_parity(H, flags):
    """Quantised scores (many exact ties, also across heads) fed straight into budget and selection; with more
    than 8 heads the heads-parallel budget kernels, or (flag) the one-workgroup-per-layer kernel."""
    rng = np.random.default_rng(0)
    w = nkv_inputs.small_workload("ties", 2, H, 64, [257, 1500])
    K, V = _kv(w)
    sc = (np.round(rng.random((w.L, w.H, w.T)) * 8) / 8).astype(np.float32)
    sc[:, :, 0:4] = oracle.PIN
    sc[:, :, 257:261] = oracle.PIN
    sc[0, 1, 10:40] = -0.0                           # -0 ties with +0
    op = oracle.Params()
    for r in (0.3, 0.75, 0.97):
        ref = oracle.compress(K.float().cpu().numpy(), bits(K), bits(V), w.cu_seqlens, [r, r], op, scores=sc)
        out, _ = run_gpu(w, K, V, r, params=nkv.params_default(flags=flags), scores=torch.from_numpy(sc).to(DEV))
        assert np.array_equal(out.k_per_head.cpu().numpy(), ref.k_per_head)
        assert np.array_equal(out.kept_idx.cpu().numpy(), ref.kept_idx)
        assert np.array_equal(bits(out.packed_k), ref.packed_k) and np.array_equal(bits(out.packed_v), ref.packed_v)


@pytest.mark.parametrize("flags", [0, nkv.FLAG_BUDGET_PER_HEAD])
def test_budget_routes_meet_the_stage_bar(flags):
    """Slice-wise and per-head budget kernels on a shape both cover (one prompt of several slices, one short,
    one of exactly two slices), fed the oracle's scores: bit-exact budgets either way."""
    w = nkv_inputs.small_workload("budget_routes", 2, 4, 128, [20000, 700, 16384])
    K, V = _kv(w)
    for r in (0.5, 0.9, 0.97):
        compare_stages(w, K, V, r, params=nkv.params_default(flags=flags), label=f"budget flags={flags} r={r}")


@pytest.mark.parametrize("flags", [0, nkv.FLAG_STATS_PER_HEAD])
def test_statistics_routes_meet_the_score_bar(flags):
    """Slice-wise and per-head statistics kernels on a shape both cover (prompts of three slices, of less than
    one, and of exactly two), against the oracle; constant keys make every value of a scale fall into one
    bin, more than the slice-wise kernels' lists hold: their finishing wavefront walks the head itself."""
    w = nkv_inputs.small_workload("stat_routes", 1, 3, 128, [20000, 700, 16384])
    K, V = _kv(w)
    compare_end_to_end(w, K, V, 0.75, params=nkv.params_default(flags=flags), label=f"stats flags={flags}")
    compare_end_to_end(w, K, V, 0.75, params=nkv.params_default(flags=flags, scale_mask=3), label=f"stats two scales flags={flags}")
    Kc = K.clone()
    Kc[:, 1] = Kc[:, 1, :1]                                   # head 1: one key repeated
    compare_end_to_end(w, Kc, V, 0.75, params=nkv.params_default(flags=flags), label=f"stats const flags={flags}")


@pytest.mark.parametrize("flags", [0, nkv.FLAG_SELECT_PER_HEAD])
def test_selection_routes_meet_the_stage_bar(flags):
    """Slice-wise and per-unit selection kernels, fed the oracle's scores and budgets: bit-exact kept indices and
    packed rows either way, for ratios that keep nearly nothing, a quarter, nearly everything, and with one
    head of constant keys (all of its scores tie: more than the slice-wise kernels' lists hold, so their
    finishing wavefront walks the head itself)."""
    w = nkv_inputs.small_workload("select_routes", 2, 3, 128, [20000, 700, 16384])
    K, V = _kv(w)
    for r in (0.999, 0.75, 0.02):
        compare_stages(w, K, V, r, params=nkv.params_default(flags=flags), label=f"select flags={flags} r={r}")
    Kc = K.clone()
    Kc[:, 1] = Kc[:, 1, :1]
    compare_stages(w, Kc, V, 0.6, params=nkv.params_default(flags=flags), label=f"select const flags={flags}")


def test_budget_without_workspace_uses_the_generic_kernel():
    w = nkv_inputs.small_workload("nows", 2, 4, 64, [3000, 200])
    K, V = _kv(w)
    a, _ = run_gpu(w, K, V, 0.8)
    b, _ = run_gpu(w, K, V, 0.8, use_ws=False)
    assert torch.equal(a.k_per_head, b.k_per_head) and torch.equal(a.kept_idx, b.kept_idx)


def test_given_budgets_are_clamped_and_capacity_is_respected():
    w = nkv_inputs.small_workload("clamp", 1, 2, 64, [50])
    K, V = _kv(w)
    sc = torch.rand(1, 2, 50, device=DEV)
    kph = torch.tensor([[[60, -3]]], dtype=torch.int32, device=DEV)     # clamped to 50 and 0
    shape, p = shape_of(w), nkv.params_default()
    pk = torch.full((40, 64), 7.0, dtype=torch.bfloat16, device=DEV)
    pv = torch.full((40, 64), 7.0, dtype=torch.bfloat16, device=DEV)
    idx = torch.full((40,), -7, dtype=torch.int32, device=DEV)
    off = torch.empty(3, dtype=torch.int64, device=DEV)
    nkv.select_compact(K, V, sc, kph, shape, p, pk, pv, idx, off, 30)   # capacity below the 50 rows needed
    torch.cuda.synchronize()
    assert off.tolist() == [0, 50, 50]
    assert idx[:30].tolist() == list(range(30)) and torch.all(idx[30:] == -7)
    assert np.array_equal(bits(pk[:30]), bits(K[0, 0, :30])) and torch.all(pk[30:] == 7.0)


@pytest.mark.parametrize("dtype,d,dv", [("bf16", 128, 128), ("fp32", 64, 32), ("fp8", 128, 64)])
@pytest.mark.parametrize("r", [0.75, 0.05, 0.999])
def test_compaction_in_place_against_the_oracle(dtype, d, dv, r):
    """NKV_FLAG_COMPACT_IN_PLACE, fed the oracle's scores and budgets: rows 0 .. B_u - 1 of every unit inside the
    caller's own K and V tensors hold the oracle's packed rows of that unit bit for bit, the rows behind them are
    untouched, head_off and kept_idx are the oracle's.  Ratios that keep a quarter, nearly all (rows barely move,
    sources and destinations of neighbouring pieces interleave) and nearly nothing."""
    w = nkv_inputs.small_workload("inplace", 2, 3, d, [9000, 700, 130, 4097], dtype=dtype, dv=dv)
    K, V = _kv(w)
    shape, op = shape_of(w), oracle_params(nkv.params_default())
    r_list = [r] * shape.n_prompts
    ref = oracle.compress(K.cpu().float().numpy(), bits(K), bits(V), w.cu_seqlens, r_list, op)
    p = nkv.params_default(flags=nkv.FLAG_COMPACT_IN_PLACE)
    Kw, Vw = K.clone(), V.clone()
    rows = int(ref.head_off[-1])
    idx = torch.empty(max(rows, 1), dtype=torch.int32, device=DEV)
    off = torch.empty(shape.n_units + 1, dtype=torch.int64, device=DEV)
    ws = torch.empty(nkv.workspace_bytes(shape, p), dtype=torch.uint8, device=DEV)
    nkv.select_compact(Kw, Vw, torch.from_numpy(ref.scores).to(DEV), torch.from_numpy(ref.k_per_head).to(DEV), shape, p,
                       None, None, idx, off, rows, None, ws)
    torch.cuda.synchronize()
    assert np.array_equal(off.cpu().numpy(), ref.head_off) and np.array_equal(idx[:rows].cpu().numpy(), ref.kept_idx)
    Kb, Vb, K0, V0, cu = bits(Kw), bits(Vw), bits(K), bits(V), w.cu_seqlens
    for pr in range(shape.n_prompts):
        for l in range(w.L):
            for h in range(w.H):
                u = (pr * w.L + l) * w.H + h
                a, b = int(ref.head_off[u]), int(ref.head_off[u + 1])
                lo, hi = cu[pr], cu[pr + 1]
                assert np.array_equal(Kb[l, h, lo:lo + b - a], ref.packed_k[a:b]), f"unit {u}: K rows"
                assert np.array_equal(Vb[l, h, lo:lo + b - a], ref.packed_v[a:b]), f"unit {u}: V rows"
                assert np.array_equal(Kb[l, h, lo + b - a:hi], K0[l, h, lo + b - a:hi]), f"unit {u}: K rows behind"
                assert np.array_equal(Vb[l, h, lo + b - a:hi], V0[l, h, lo + b - a:hi]), f"unit {u}: V rows behind"
    # packed buffers together with the flag, and row widths the in-place kernels do not take, are refused
    with pytest.raises(nkv.NkvError):
        nkv.select_compact(Kw, Vw, torch.from_numpy(ref.scores).to(DEV), torch.from_numpy(ref.k_per_head).to(DEV), shape, p,
                           Kw, Vw, idx, off, rows, None, ws)


# ------------------------------------------------------------------ parameters and variants
VARIANTS = [
    dict(gate_mode=1), dict(gate_mode=2), dict(surprise_mode=1), dict(beta=0.0),
    dict(prior=(1.0, 0.0, 0.0), beta=0.0, gate_mode=1), dict(n_sink=0), dict(n_sink=9),
    dict(window=16), dict(window=200), dict(block_min=32, block_max=96, block_div=8),
    dict(block_min=16, block_max=64, block_div=64),      # blocks of one wavefront
    dict(block_min=300, block_max=512), dict(top_frac=0.25, safeguard=0.5), dict(safeguard=1.0),
    dict(kappa=25.0, tau=0.2),
    dict(scale_mask=3), dict(scale_mask=5), dict(scale_mask=6), dict(scale_mask=1), dict(scale_mask=4, gate_mode=2),
    dict(scale_mask=3, surprise_mode=1), dict(scale_mask=0),
]


@pytest.mark.parametrize("over", VARIANTS, ids=[",".join(f"{k}={v}" for k, v in o.items()) for o in VARIANTS])
def test_parameter_variants(over):
    w = nkv_inputs.small_workload("variants", 1, 3, 128, [1111, 300])
    K, V = _kv(w)
    params = nkv.params_default(**over)
    compare_stages(w, K, V, 0.6, params=params, label=str(over))
    compare_end_to_end(w, K, V, 0.6, params=params, label=str(over))


@pytest.mark.parametrize("dtype", ["bf16", "fp16"])
def test_generic_and_streaming_kernels_agree_with_oracle(dtype):
    """The shape-generic scoring kernels, forced by flag, and every route of the streaming kernels meet the same
    bar on a streaming-eligible shape, for 16-bit keys of either format."""
    w = nkv_inputs.small_workload("generic", 2, 2, 128, [2000, 321], dtype=dtype)
    K, V = _kv(w)
    compare_end_to_end(w, K, V, 0.5, params=nkv.params_default(flags=nkv.FLAG_GENERIC_KERNELS), label="generic")
    compare_end_to_end(w, K, V, 0.5, params=nkv.params_default(flags=nkv.FLAG_TWO_PASS_STABLE), label="two-pass")
    compare_end_to_end(w, K, V, 0.5, params=nkv.params_default(flags=nkv.FLAG_DEFER_STABLE), label="deferred")
    compare_end_to_end(w, K, V, 0.5, params=nkv.params_default(flags=nkv.FLAG_NO_UNIT_SUMS), label="no unit sums")
    compare_end_to_end(w, K, V, 0.5, label="default")


def test_raw_anomalies_match_oracle():
    w = nkv_inputs.small_workload("raw", 1, 2, 128, [1500, 200])
    K, _ = _kv(w)
    shape, p = shape_of(w), nkv.params_default()
    a = torch.empty(3, w.L, w.H, w.T, dtype=torch.float32, device=DEV)
    ws = torch.empty(nkv.workspace_bytes(shape, p), dtype=torch.uint8, device=DEV)
    nkv.score_raw(K, shape, p, a, ws)
    torch.cuda.synchronize()
    a = a.cpu().numpy()
    for pi, (lo, hi) in enumerate(zip(w.cu_seqlens[:-1], w.cu_seqlens[1:])):
        _, dbg = oracle.score_layer(K[0, :, lo:hi].float().cpu().numpy(), debug=("a_raw",))
        np.testing.assert_allclose(a[:, 0, :, lo:hi], dbg["a_raw"], atol=2e-6)


def test_scale_invariance_on_device():
    """Scaling each key by its own power of two leaves the scores bit-identical (Section 2.1)."""
    w = nkv_inputs.small_workload("scale", 1, 2, 128, [1024])
    K, V = _kv(w)
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    sc = torch.exp2(torch.randint(-5, 6, (1, 2, 1024, 1), device=DEV, generator=g).float()).to(torch.bfloat16)
    out0, _ = run_gpu(w, K, V, 0.5)
    out1, _ = run_gpu(w, (K * sc).contiguous(), V, 0.5)
    assert torch.equal(out0.scores, out1.scores)
    assert torch.equal(out0.kept_idx, out1.kept_idx)


def test_deterministic_and_untouched_neighbours():
    """Two runs give identical bits; nothing is written outside the output tensors (canaries)."""
    w = nkv_inputs.small_workload("det", 2, 2, 128, [3000, 500])
    K, V = _kv(w)
    shape, p = shape_of(w), nkv.params_default()
    rows = nkv.packed_rows(shape, [0.7, 0.7])
    pad = 64
    results = []
    for _ in range(2):
        scores = torch.full((w.L * w.H * w.T + 2 * pad,), -5.0, device=DEV)
        pk = torch.full(((rows + 2) * w.d,), 3.0, dtype=torch.bfloat16, device=DEV)
        pv = torch.full(((rows + 2) * w.d,), 3.0, dtype=torch.bfloat16, device=DEV)
        idx = torch.full((rows + 2 * pad,), -9, dtype=torch.int32, device=DEV)
        kph = torch.full((shape.n_units + 2 * pad,), -9, dtype=torch.int32, device=DEV)
        off = torch.full((shape.n_units + 1 + 2 * pad,), -9, dtype=torch.int64, device=DEV)
        ws = torch.empty(nkv.workspace_bytes(shape, p), dtype=torch.uint8, device=DEV)
        s_view = scores[pad:-pad]
        nkv.score(K, shape, p, s_view, ws)
        nkv.budget(s_view, shape, p, [0.7, 0.7], kph[pad:-pad])
        nkv.select_compact(K, V, s_view, kph[pad:-pad], shape, p, pk[w.d:-w.d], pv[w.d:-w.d], idx[pad:-pad],
                           off[pad:-pad], rows)
        torch.cuda.synchronize()
        for t, val in ((scores, -5.0), (idx, -9), (kph, -9), (off, -9)):
            assert torch.all(t[:pad] == val) and torch.all(t[-pad:] == val)
        assert torch.all(pk[:w.d] == 3.0) and torch.all(pk[-w.d:] == 3.0)
        assert torch.all(pv[:w.d] == 3.0) and torch.all(pv[-w.d:] == 3.0)
        results.append([t.clone() for t in (scores, pk.view(torch.int16), pv.view(torch.int16), idx, kph, off)])
    for a, b in zip(*results):
        assert torch.equal(a, b)


def test_deferred_stable_route_gives_the_same_bits():
    """A block whose workgroup does not wait for its unit's sum gets its stable anomaly from a later kernel;
    which of the two routes a block takes depends on timing, so both must produce identical scores."""
    for name, L, H, d, lens, dtype in (("defer128", 2, 3, 128, [3000, 500, 129], "bf16"), ("defer64", 1, 4, 64, [2500, 64], "bf16"),
                                       ("defer128_fp16", 2, 2, 128, [2100, 300], "fp16")):
        w = nkv_inputs.small_workload(name, L, H, d, lens, dtype=dtype)
        K, V = _kv(w)
        a, _ = run_gpu(w, K, V, 0.6)
        b, _ = run_gpu(w, K, V, 0.6, params=nkv.params_default(flags=nkv.FLAG_DEFER_STABLE))
        assert torch.equal(a.scores, b.scores) and torch.equal(a.kept_idx, b.kept_idx)
        # and a unit sum that the pass itself did not form is filled in afterwards, with the same bits
        c, _ = run_gpu(w, K, V, 0.6, params=nkv.params_default(flags=nkv.FLAG_NO_UNIT_SUMS))
        assert torch.equal(a.scores, c.scores) and torch.equal(a.kept_idx, c.kept_idx)


@pytest.mark.parametrize("d", [128, 64])
def test_scan_counters_report_the_route_taken(d):
    """The optional health counters of the fused scan: no summing workgroup gives up and few blocks take the
    deferred route in normal operation; the flags that force those routes show up in them exactly."""
    w = nkv_inputs.small_workload("counters", 2, 3, d, [3000, 500, 129])
    K, _ = _kv(w)
    shape = shape_of(w)
    blocks = sum((n + nkv.block_size(n) - 1) // nkv.block_size(n) for n in w.prompt_lens) * w.L * w.H
    units = len(w.prompt_lens) * w.L * w.H
    cnt = torch.full((2,), 77, dtype=torch.int32, device=DEV)
    sc = torch.empty(w.L, w.H, w.T, dtype=torch.float32, device=DEV)
    # head dim 128 takes the matrix-core scan, whose units are added up by integer atomics: nothing there can give up
    gave_up = 0 if d == 128 else units
    for flags, want in ((0, None), (nkv.FLAG_DEFER_STABLE, (0, blocks)), (nkv.FLAG_NO_UNIT_SUMS, (gave_up, blocks)),
                        (nkv.FLAG_TWO_PASS_STABLE, (0, 0)), (nkv.FLAG_GENERIC_KERNELS, (0, 0))):
        p = nkv.params_default(flags=flags, scan_counters=cnt.data_ptr())
        ws = torch.empty(nkv.workspace_bytes(shape, p), dtype=torch.uint8, device=DEV)
        cnt.fill_(77)
        nkv.score(K, shape, p, sc, ws)
        torch.cuda.synchronize()
        got = tuple(cnt.tolist())
        if want is None:
            assert got[0] == 0 and got[1] <= blocks // 2, got
        else:
            assert got == want, (flags, got, want)


def test_ragged_batch_is_reproducible():
    """The ragged serving shape, several times over: identical bits every time (no wait may run out)."""
    w = nkv_inputs.WORKLOADS["llama3b_ragged"]
    K, V = _kv(w)
    ref, _ = run_gpu(w, K, V, 0.95)
    assert not torch.isnan(ref.scores).any()
    for _ in range(6):
        out, _ = run_gpu(w, K, V, 0.95)
        assert torch.equal(out.scores, ref.scores) and torch.equal(out.kept_idx, ref.kept_idx)


# ------------------------------------------------------------------ strided K/V (a framework's own cache tensors)
def _run_with_layout(w, K, V, r, shape, params=None):
    params = params or nkv.params_default()
    comp = nkv.Compressor(shape, [r] * shape.n_prompts, params)
    out = comp.run(K, V)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("flags", [0, nkv.FLAG_TWO_PASS_STABLE, nkv.FLAG_GENERIC_KERNELS, nkv.FLAG_NO_UNIT_SUMS])
def test_strided_layouts_give_the_same_bits(flags):
    """Keys and values that live in slabs of their own -- one [H][N_max][d] slab per prompt, as a framework's
    per-layer cache tensor has them, or heads padded apart -- give the outputs of the dense layout bit for bit
    and meet the oracle's bar themselves; the padding holds NaNs and is never read."""
    w = nkv_inputs.small_workload("strided", 2, 3, 128, [700, 1333])
    K, V = _kv(w)
    params = nkv.params_default(flags=flags)
    ref, _ = run_gpu(w, K, V, 0.6, params=params)
    L, H, d, cu = w.L, w.H, w.d, w.cu_seqlens
    nmax = 1400
    # [L][P][H][nmax][d]: per-prompt slabs, right-padded
    Kp = torch.full((L, 2, H, nmax, d), float("nan"), dtype=K.dtype, device=DEV)
    Vp = torch.full((L, 2, H, nmax, d), float("nan"), dtype=V.dtype, device=DEV)
    for p in range(2):
        Kp[:, p, :, :cu[p + 1] - cu[p]] = K[:, :, cu[p]:cu[p + 1]]
        Vp[:, p, :, :cu[p + 1] - cu[p]] = V[:, :, cu[p]:cu[p + 1]]
    st = (2 * H * nmax * d, nmax * d, H * nmax * d)
    shape = nkv.Shape(L, H, d, d, nkv.DTYPE_BF16, cu, key_strides=st, value_strides=st)
    out = _run_with_layout(w, Kp, Vp, 0.6, shape, params)
    check_against_oracle(w, K, V, out, 0.6, params, label=f"per-prompt slabs flags={flags}")
    for name in ("scores", "k_per_head", "head_off", "kept_idx"):
        assert torch.equal(getattr(out, name), getattr(ref, name)), name
    assert np.array_equal(bits(out.packed_k), bits(ref.packed_k)) and np.array_equal(bits(out.packed_v), bits(ref.packed_v))
    # concatenated prompts, heads padded apart; values dense
    T = w.T
    Kh = torch.full((L, H, T + 24, d), float("nan"), dtype=K.dtype, device=DEV)
    Kh[:, :, :T] = K
    shape = nkv.Shape(L, H, d, d, nkv.DTYPE_BF16, cu, key_strides=(H * (T + 24) * d, (T + 24) * d, 0))
    out = _run_with_layout(w, Kh, V, 0.6, shape, params)
    check_against_oracle(w, K, V, out, 0.6, params, label=f"padded heads flags={flags}")
    assert torch.equal(out.scores, ref.scores) and torch.equal(out.kept_idx, ref.kept_idx)
    assert np.array_equal(bits(out.packed_k), bits(ref.packed_k)) and np.array_equal(bits(out.packed_v), bits(ref.packed_v))


@pytest.mark.parametrize("case", range(12))
def test_random_layouts_types_and_masks(case):
    """Seeded random draws of shape, element type (bf16, fp16, 8-bit, fp32), scale mask and code route in one of four
    layouts -- per-prompt slabs with NaN padding, heads padded apart, one tensor per layer, or dense with the
    compaction done in place -- against the oracle on the dense tensors."""
    import random
    rnd = random.Random(9000 + case)
    dtype = rnd.choice(["bf16", "fp16", "fp8", "fp32"])
    tdt, ndt = {"bf16": (torch.bfloat16, nkv.DTYPE_BF16), "fp16": (torch.float16, nkv.DTYPE_F16),
                "fp32": (torch.float32, nkv.DTYPE_F32), "fp8": (torch.float8_e4m3fn, nkv.DTYPE_F8_E4M3)}[dtype]
    d = rnd.choice([64, 128, 128])
    L, H, P = rnd.randint(1, 3), rnd.choice([1, 2, 4, 8]), rnd.choice([1, 2, 3])
    lens = [rnd.choice([rnd.randint(1, 400), rnd.randint(400, 9000), rnd.randint(9000, 30000)]) for _ in range(P)]
    if sum(lens) * L * H > 400000:
        L, H = 1, min(H, 2)
    r = rnd.choice([0.3, 0.5, 0.75, 0.95])
    mask = rnd.choice([7, 7, 7, 3, 5, 6, 1])
    flags = rnd.choice([0, 0, nkv.FLAG_VECTOR_SCAN, nkv.FLAG_DEFER_STABLE])
    layout = ["slabs", "padded_heads", "layer_tensors", "in_place"][case % 4]
    label = f"random layout {case}: {layout} L={L} H={H} d={d} {dtype} lens={lens} r={r} mask={mask} flags={flags}"
    print(label, flush=True)
    w = nkv_inputs.small_workload(f"layout{case}", L, H, d, lens, dtype=dtype, n_out=min(8, max(min(lens) - 4, 0)), seed=9000 + case)
    K, V = _kv(w)
    cu, T = w.cu_seqlens, w.T
    p = nkv.params_default(flags=flags, scale_mask=mask)

    def padding(*shape):
        if tdt == torch.float8_e4m3fn:
            return torch.full(shape, 0x7f, dtype=torch.uint8, device=DEV).view(tdt)      # the format's NaN code
        return torch.full(shape, float("nan"), dtype=tdt, device=DEV)

    if layout == "slabs":
        nmax = max(lens) + rnd.choice([0, 8, 40])
        Kp, Vp = padding(L, P, H, nmax, d), padding(L, P, H, nmax, d)
        for q in range(P):
            Kp[:, q, :, :lens[q]] = K[:, :, cu[q]:cu[q + 1]]
            Vp[:, q, :, :lens[q]] = V[:, :, cu[q]:cu[q + 1]]
        st = (P * H * nmax * d, nmax * d, H * nmax * d)
        out = _run_with_layout(w, Kp, Vp, r, nkv.Shape(L, H, d, d, ndt, cu, key_strides=st, value_strides=st), p)
    elif layout == "padded_heads":
        pad = rnd.choice([8, 24, 64])
        Kh = padding(L, H, T + pad, d)
        Kh[:, :, :T] = K
        out = _run_with_layout(w, Kh, V, r, nkv.Shape(L, H, d, d, ndt, cu, key_strides=(H * (T + pad) * d, (T + pad) * d, 0)), p)
    elif layout == "layer_tensors":
        order = list(range(L))
        rnd.shuffle(order)                                       # allocation order: some offsets come out negative
        Kl, Vl = [None] * L, [None] * L
        for l in order:
            Kl[l], Vl[l] = K[l].clone(), V[l].clone()
        out = _run_with_layout(w, Kl[0], Vl[0], r, nkv.Shape(L, H, d, d, ndt, cu, key_layers=Kl, value_layers=Vl), p)
    else:
        shape = shape_of(w)
        comp = nkv.Compressor(shape, [r] * P, p)
        out = comp.run(K, V)
        torch.cuda.synchronize()
        K2, V2 = K.clone(), V.clone()
        nkv.select_compact(K2, V2, comp.scores, comp.k_per_head, shape,
                           nkv.params_default(flags=flags | nkv.FLAG_COMPACT_IN_PLACE, scale_mask=mask), None, None,
                           comp.kept_idx, comp.head_off, comp.rows, comp.near, comp.ws)
        torch.cuda.synchronize()
        ho, pk, pv, K2b, V2b = comp.head_off.cpu().numpy(), bits(out.packed_k), bits(out.packed_v), bits(K2), bits(V2)
        u = 0
        for q in range(P):
            for l in range(L):
                for h in range(H):
                    B = int(ho[u + 1] - ho[u])
                    assert np.array_equal(K2b[l, h, cu[q]:cu[q] + B], pk[ho[u]:ho[u + 1]]), (label, "K rows", q, l, h)
                    assert np.array_equal(V2b[l, h, cu[q]:cu[q] + B], pv[ho[u]:ho[u + 1]]), (label, "V rows", q, l, h)
                    u += 1
    check_against_oracle(w, K, V, out, r, p, label=label)


@pytest.mark.parametrize("flags", [0, nkv.FLAG_TWO_PASS_STABLE, nkv.FLAG_GENERIC_KERNELS, nkv.FLAG_DEFER_STABLE])
def test_one_tensor_per_layer_gives_the_same_bits(flags):
    """A framework's list of per-layer cache tensors, each an allocation of its own ([B][H][N_max][d] with one
    slab per prompt for the keys, dense [H][T][d_v] for the values), allocated in an order that makes some
    layer offsets negative: one call over all layers meets the oracle's bar and gives the dense layout's outputs
    bit for bit."""
    w = nkv_inputs.small_workload("layer_list", 5, 2, 128, [900, 17000, 333])
    K, V = _kv(w)
    params = nkv.params_default(flags=flags)
    ref, _ = run_gpu(w, K, V, 0.7, params=params)
    L, H, d, cu = w.L, w.H, w.d, w.cu_seqlens
    P, nmax = 3, 17024
    order = [3, 0, 4, 1, 2]                                  # allocation order != layer order
    Kl, Vl, pad = [None] * L, [None] * L, []
    for l in order:
        Kl[l] = torch.full((P, H, nmax, d), float("nan"), dtype=K.dtype, device=DEV)
        pad.append(torch.empty(1000 + 64 * l, device=DEV))  # something else in between
        Vl[l] = V[l].clone()
        for p in range(P):
            Kl[l][p, :, :cu[p + 1] - cu[p]] = K[l, :, cu[p]:cu[p + 1]]
    shape = nkv.Shape(L, H, d, d, nkv.DTYPE_BF16, cu, key_strides=(0, nmax * d, H * nmax * d), key_layers=Kl,
                      value_layers=Vl)
    print("layer offsets (elements):", list(shape.klo), list(shape.vlo))
    out = _run_with_layout(w, Kl[0], Vl[0], 0.7, shape, params)
    check_against_oracle(w, K, V, out, 0.7, params, layers=[0, 3], label=f"layer tensors flags={flags}")
    for name in ("scores", "k_per_head", "head_off", "kept_idx"):
        assert torch.equal(getattr(out, name), getattr(ref, name)), name
    assert np.array_equal(bits(out.packed_k), bits(ref.packed_k)) and np.array_equal(bits(out.packed_v), bits(ref.packed_v))


def test_layer_by_layer_calls_equal_the_batched_call():
    """The pass is independent per layer (Section 2, "independently at each layer"): calling it with L = 1 on
    each layer's slice, as a prefill loop would right after the layer's keys exist, meets the oracle's bar
    and gives the rows of the one call over all layers."""
    w = nkv_inputs.small_workload("per_layer", 3, 4, 128, [2100, 260])
    K, V = _kv(w)
    ref, _ = run_gpu(w, K, V, 0.75)
    shape1 = nkv.Shape(1, w.H, w.d, w.d_v, nkv.DTYPE_BF16, w.cu_seqlens)
    comp = nkv.Compressor(shape1, [0.75] * 2)
    import dataclasses
    w1 = dataclasses.replace(w, L=1)
    for l in range(w.L):
        out = comp.run(K[l], V[l])
        torch.cuda.synchronize()
        check_against_oracle(w1, K[l:l + 1], V[l:l + 1], out, 0.75, label=f"L=1 call on layer {l}")
        assert torch.equal(out.scores[0], ref.scores[l])
        assert torch.equal(out.k_per_head[:, 0], ref.k_per_head[:, l])
        for p in range(2):
            for h in range(w.H):
                u1, u = p * w.H + h, (p * w.L + l) * w.H + h
                a, b = int(out.head_off[u1]), int(out.head_off[u1 + 1])
                o = int(ref.head_off[u])
                assert b - a == int(ref.head_off[u + 1]) - o
                assert torch.equal(out.kept_idx[a:b], ref.kept_idx[o:o + b - a])
                assert np.array_equal(bits(out.packed_k[a:b]), bits(ref.packed_k[o:o + b - a]))
                assert np.array_equal(bits(out.packed_v[a:b]), bits(ref.packed_v[o:o + b - a]))


def test_recompression_of_a_uniformly_compressed_cache():
    """Decode-time recompression, in the one form the calls express as they are: with a uniform budget
    (safeguard = 1) every head of a layer keeps k0 rows, so the packed cache is a dense [L][H][k0][d] tensor; new rows
    appended per head make a dense [L][H][k0 + m][d] one, and compressing that again is the same three calls on it
    (the retained rows, in cache order, are the sequence that windows and blocks run over -- the paper leaves the
    incremental update open, this is this build's reading).  Both passes against the oracle."""
    w = nkv_inputs.small_workload("recompress", 2, 4, 128, [9000], n_out=8)
    K, V = _kv(w)
    p = nkv.params_default(safeguard=1.0)
    first, _ = run_gpu(w, K, V, 0.5, params=p)
    check_against_oracle(w, K, V, first, 0.5, p, label="recompress, first pass")
    k0 = nkv.k0(9000, 0.5)
    assert first.k_per_head.reshape(-1).tolist() == [k0] * (w.L * w.H)
    m = 700
    g = torch.Generator().manual_seed(5)
    grow = lambda packed: torch.cat([packed.reshape(w.L, w.H, k0, 128),
                                     torch.randn(w.L, w.H, m, 128, generator=g).to(torch.bfloat16).to(DEV)], dim=2).contiguous()
    K2, V2 = grow(first.packed_k), grow(first.packed_v)
    w2 = nkv_inputs.small_workload("recompress2", 2, 4, 128, [k0 + m], n_out=0)
    second, _ = run_gpu(w2, K2, V2, 0.3, params=p)
    st = check_against_oracle(w2, K2, V2, second, 0.3, p, label="recompress, second pass")
    _report("recompress second pass", st)
    assert second.k_per_head.reshape(-1).tolist() == [nkv.k0(k0 + m, 0.3)] * (w.L * w.H)


def test_the_three_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """The calls only enqueue kernels on the given stream (no allocation, no synchronisation, no memset
    nodes), so a serving loop can record them once and replay: every replay, with eager work and
    synchronisations in between, gives the eager result bit for bit."""
    w = nkv_inputs.small_workload("graph", 2, 4, 128, [20000, 700])      # slice-wise and per-head kernels
    K, V = _kv(w)
    ref, shape = run_gpu(w, K, V, 0.75)                       # eager, also warms every lazily initialised path
    ref = [t.clone() for t in (ref.scores, ref.k_per_head, ref.head_off, ref.kept_idx, ref.packed_k.view(torch.int16),
                               ref.packed_v.view(torch.int16))]
    comp = nkv.Compressor(shape, [0.75, 0.75])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        comp.run(K, V, side)                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            comp.run(K, V, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (comp.scores, comp.kept_idx, comp.packed_k, comp.packed_v):
            t.zero_()                                          # eager work between the replays
        comp.k_per_head.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (comp.scores, comp.k_per_head, comp.head_off, comp.kept_idx[:comp.rows],
               comp.packed_k[:comp.rows].view(torch.int16), comp.packed_v[:comp.rows].view(torch.int16))
        for a, b in zip(got, ref):
            assert torch.equal(a, b), f"replay {rep}"
