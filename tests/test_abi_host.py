"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, validates arguments before touching the device, and evaluates the paper's closed forms."""
import ctypes as C
import os
import re

import pytest

import paper_2605_26678_amd as nkv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "nkv.h")).read()
    declared = set(re.findall(r"\b(nkv_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(nkv.EXPORTS)
    for name in declared:
        assert hasattr(nkv.lib(), name), name


def test_params_default_are_the_papers_constants():
    p = nkv.params_default()
    assert p.struct_size == C.sizeof(nkv.nkv_params)
    assert (p.window, p.block_div, p.block_min, p.block_max, p.n_sink) == (64, 32, 128, 256, 4)
    assert list(p.prior) == [0.4, 0.4, 0.2]
    assert (p.beta, p.tau, p.kappa, p.safeguard, p.top_frac) == (3.0, 0.60, 10.0, 0.20, 0.10)
    assert p.scale_mask == 7
    assert nkv.lib().nkv_params_default(None) == nkv.NKV_EINVAL


def test_closed_forms_match_golden_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "schedule_integers.txt")) if l.strip() and l[0] != "#"]
    for N, r, b, k0, ms, mp in rows:
        N, r = int(N), float(r)
        assert nkv.block_size(N) == int(b)
        assert nkv.k0(N, r) == int(k0)
        assert nkv.m_safe(nkv.k0(N, r)) == int(ms)
        assert nkv.m_p(N) == int(mp)
    assert nkv.k0(10, 0.9) == 1 and nkv.k0(10, 1.5) == -1 and nkv.m_p(0) == -1


def test_packed_rows_and_workspace():
    s = nkv.Shape(36, 8, 128, 128, nkv.DTYPE_BF16, [0, 32768])
    assert nkv.packed_rows(s, [0.75]) == 36 * 8 * 8192
    assert nkv.workspace_bytes(s) >= 3 * 36 * 8 * 32768 * 4
    rag = nkv.Shape(2, 8, 128, 128, nkv.DTYPE_BF16, [0, 4096, 12288])
    assert nkv.packed_rows(rag, [0.95, 0.5]) == 2 * 8 * (204 + 4096)


def test_argument_errors_are_reported_before_any_device_work():
    p = nkv.params_default()
    good = nkv.Shape(1, 2, 64, 64, nkv.DTYPE_BF16, [0, 100])
    L = nkv.lib()
    fake = 4096      # never dereferenced: every call below must fail in validation
    assert L.nkv_score(0, C.byref(good.c), C.byref(p), fake, fake, 1 << 30, 0) == nkv.NKV_EINVAL
    assert L.nkv_score(fake, C.byref(good.c), C.byref(p), fake, 0, 0, 0) == nkv.NKV_EWORKSPACE
    assert L.nkv_score(fake, C.byref(good.c), C.byref(p), fake, fake + 8, 1 << 30, 0) == nkv.NKV_EWORKSPACE
    assert L.nkv_score(fake, C.byref(good.c), C.byref(p), fake, fake, 16, 0) == nkv.NKV_EWORKSPACE
    assert L.nkv_score(fake + 2, C.byref(good.c), C.byref(p), fake, fake, 1 << 30, 0) == nkv.NKV_EINVAL
    for bad in (nkv.Shape(0, 2, 64, 64, 1, [0, 100]), nkv.Shape(1, 33, 64, 64, 1, [0, 100]),
                nkv.Shape(1, 2, 60, 64, 1, [0, 100]), nkv.Shape(1, 2, 64, 2048, 1, [0, 100]),
                nkv.Shape(1, 2, 64, 64, 1, [0, 100, 100]), nkv.Shape(1, 2, 64, 64, 1, [1, 100]),
                nkv.Shape(1, 2, 64, 64, 1, list(range(0, 66 * 10, 10)))):
        assert L.nkv_score(fake, C.byref(bad.c), C.byref(p), fake, fake, 1 << 30, 0) == nkv.NKV_ESHAPE
    assert L.nkv_score(fake, C.byref(nkv.Shape(1, 2, 64, 64, 7, [0, 100]).c), C.byref(p), fake, fake, 1 << 30,
                       0) == nkv.NKV_EINVAL
    for field, val in (("window", 0), ("block_max", 1), ("gate_mode", 3), ("top_frac", 0.0), ("safeguard", 1.5),
                       ("beta", float("nan")), ("struct_size", 8), ("n_sink", -1), ("scale_mask", 8), ("scale_mask", -1)):
        q = nkv.params_default(**{field: val})
        assert L.nkv_score(fake, C.byref(good.c), C.byref(q), fake, fake, 1 << 30, 0) == nkv.NKV_EINVAL, field
    # strided layouts: misaligned strides, overlapping units
    for ks in ((64 * 100 * 2 + 4, 64 * 100, 0), (0, 64 * 99, 0), (0, 64 * 100, 64 * 100), (-8, 64 * 100, 0)):
        bad = nkv.Shape(1, 2, 64, 64, 1, [0, 60, 100], key_strides=ks)
        assert L.nkv_score(fake, C.byref(bad.c), C.byref(p), fake, fake, 1 << 30, 0) == nkv.NKV_EINVAL, ks
    # one tensor per layer: entry 0 must be 0, entries 16-byte multiples, layers apart, at most 128 of them
    per = 2 * 100 * 64                                        # elements of one dense layer tensor
    for off in ((8, per), (0, per + 4), (0, per - 8), (0, -per + 8)):
        bad = nkv.Shape(2, 2, 64, 64, 1, [0, 60, 100])
        bad.klo = (C.c_int64 * 2)(*off)
        bad.c.key_layer_offsets = bad.klo
        assert L.nkv_score(fake, C.byref(bad.c), C.byref(p), fake, fake, 1 << 30, 0) == nkv.NKV_EINVAL, off
    many = nkv.Shape(129, 1, 64, 64, 1, [0, 100], key_layers=[4096 + 2 * 6400 * l for l in range(129)])
    assert L.nkv_score(fake, C.byref(many.c), C.byref(p), fake, fake, 1 << 30, 0) == nkv.NKV_EINVAL
    fine = nkv.Shape(3, 2, 64, 64, 1, [0, 60, 100], key_layers=[1 << 20, 1 << 16, 1 << 24],
                     value_layers=[1 << 30, (1 << 30) + 2 * per, (1 << 30) - 2 * per])
    assert list(fine.klo) == [0, ((1 << 16) - (1 << 20)) // 2, ((1 << 24) - (1 << 20)) // 2]
    assert nkv.workspace_bytes(fine) > 0
    ok = nkv.Shape(3, 2, 64, 64, 1, [0, 60, 100], key_strides=(64 * 128 * 4, 64 * 128, 64 * 128 * 2),
                   value_strides=(64 * 300, 64 * 100, 0))
    assert nkv.workspace_bytes(ok) > 0
    r_bad = (C.c_double * 1)(1.5)
    assert L.nkv_budget(fake, C.byref(good.c), C.byref(p), r_bad, fake, 0, 0, 0) == nkv.NKV_EINVAL
    assert L.nkv_budget(fake, C.byref(good.c), C.byref(p), None, fake, 0, 0, 0) == nkv.NKV_EINVAL
    assert L.nkv_select_compact(fake, fake, fake, fake, C.byref(good.c), C.byref(p), fake, fake, fake, fake, -1,
                                0, 0, 0, 0) == nkv.NKV_EINVAL
    assert L.nkv_select_compact(fake, fake, fake, fake, C.byref(good.c), C.byref(p), 0, fake, fake, fake, 10,
                                0, 0, 0, 0) == nkv.NKV_EINVAL
    # compaction in place: no packed buffers with the flag, and only rows of 32 .. 1024 bytes, a power of two
    pin = nkv.params_default(flags=nkv.FLAG_COMPACT_IN_PLACE)
    assert L.nkv_select_compact(fake, fake, fake, fake, C.byref(good.c), C.byref(pin), fake, fake, fake, fake, 10,
                                0, 0, 0, 0) == nkv.NKV_EINVAL
    odd = nkv.Shape(1, 2, 96, 64, nkv.DTYPE_BF16, [0, 100])              # 192-byte key rows
    assert L.nkv_select_compact(fake, fake, fake, fake, C.byref(odd.c), C.byref(pin), 0, 0, fake, fake, 10,
                                0, 0, 0, 0) == nkv.NKV_EUNSUPPORTED
    # 8-bit caches: rows are moved as 16-byte vectors, attention over them is refused
    f8 = nkv.DTYPE_F8_E4M3
    assert L.nkv_score(fake, C.byref(nkv.Shape(1, 2, 72, 64, f8, [0, 100]).c), C.byref(p), fake, fake, 1 << 30,
                       0) == nkv.NKV_ESHAPE
    assert L.nkv_score(fake, C.byref(nkv.Shape(1, 2, 64, 24, f8, [0, 100]).c), C.byref(p), fake, fake, 1 << 30,
                       0) == nkv.NKV_ESHAPE
    assert nkv.workspace_bytes(nkv.Shape(1, 2, 64, 32, f8, [0, 100])) > 0
    nbytes = C.c_size_t(0)
    assert L.nkv_decode_workspace_bytes(C.byref(nkv.Shape(1, 2, 64, 64, f8, [0, 100]).c), 4, 50,
                                        C.byref(nbytes)) == nkv.NKV_EUNSUPPORTED
    with pytest.raises(nkv.NkvError):
        nkv.workspace_bytes(nkv.Shape(1, 2, 64, 64, 1, [0, 0]))
    assert "workspace" in nkv.strerror(nkv.NKV_EWORKSPACE)


def test_input_generator_is_deterministic_and_shaped():
    import torch
    import nkv_inputs
    w = nkv_inputs.small_workload("t", 2, 2, 64, [300, 200])
    k1, v1 = nkv_inputs.make_kv(w)
    k2, v2 = nkv_inputs.make_kv(w)
    assert k1.shape == (2, 2, 500, 64) and v1.dtype == torch.bfloat16
    assert torch.equal(k1.view(torch.int16), k2.view(torch.int16)) and torch.equal(v1.view(torch.int16), v2.view(torch.int16))
    assert torch.allclose(k1[0, 0, 0].float().norm(), torch.tensor(10.0), atol=0.1)      # sink-like key


def test_8bit_test_inputs_follow_the_published_format():
    """The parity tests hand the oracle 8-bit keys converted to fp32 by torch on the host; this pins that
    conversion to the E4M3 format's definition (sign, 4 exponent bits with bias 7, 3 mantissa bits, no
    infinities, S.1111.111 = NaN) for all 256 codes, so that the kernels' own decoder is checked against the
    format and not against a library's reading of it."""
    import math
    import torch
    got = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).tolist()
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            assert math.isnan(got[code])
            continue
        mag = m / 8.0 * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
        assert got[code] == (-mag if s else mag) and math.copysign(1.0, got[code]) == (-1.0 if s else 1.0), code
    assert max(v for v in got if not math.isnan(v)) == 448.0


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py says so and exits instead of pretending to scale."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
