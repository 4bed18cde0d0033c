"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no worked numeric example of a score, weight, budget or kept set, so every pin here is a
closed form, an invariant, a special case that reduces to a numpy / scipy routine the oracle does not call,
or brute force on tiny inputs.  None of them retypes the oracle's own loops.  What cannot be pinned this way
-- agreement with the authors' code on the readings the paper leaves open (size of the top/bottom sets, the
order min-max -> centre -> rectify of the surprise, the value used for pinning, H*k0 as the layer budget) --
is "parity unpinned".
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.spatial.distance as ssd
import scipy.special

import oracle
from oracle import Params

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_keys(H, N, d, seed=0, mean=2.0):
    rng = np.random.default_rng(seed)
    u = rng.standard_normal((H, 1, d))
    u /= np.linalg.norm(u, axis=-1, keepdims=True)
    return (rng.standard_normal((H, N, d)) + mean * u).astype(np.float32)


# --------------------------------------------------------------------------- closed-form integers
def test_schedule_integers_golden():
    """Section 2.2 block schedule; Appendix A k0 / safeguard; Section 2.4 p = 10 %."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "schedule_integers.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 12
    for N, r, b, k0, ms, mp in rows:
        N, r = int(N), float(r)
        assert oracle.block_size(N) == int(b), (N, r)
        assert oracle.k0(N, r) == int(k0), (N, r)
        assert oracle.m_safe(oracle.k0(N, r)) == int(ms), (N, r)
        assert oracle.m_p(N) == int(mp), (N, r)


def test_k0_decimal_ratios_do_not_lose_one():
    # (1 - 0.9) * 10 is 0.9999999999999998 in binary floating point; the floor must still be 1
    assert oracle.k0(10, 0.9) == 1
    assert oracle.k0(100, 0.7) == 30
    assert oracle.k0(1000, 0.3) == 700


# --------------------------------------------------------------------------- hand-worked 2-D example
def test_hand_worked_four_tokens():
    """d = 2, N = 4, W = 2, b = 2; angles 0, 90, 45, 0 degrees (Sections 2.2-2.3).

    Bisector geometry gives every cosine in closed form: a block or window holding two unit vectors at
    angles t1, t2 has its mean along (t1+t2)/2, so each member sees cos((t1-t2)/2).
    """
    keys = np.array([[[1, 0], [0, 2], [3, 3], [0.5, 0]]], dtype=np.float32)   # norms differ on purpose
    p = Params(window=2, block_div=1000, block_min=2, block_max=2)
    _, dbg = oracle.score_layer(keys, p, debug=("a_raw", "mu_s", "mu_e", "mu_c"))
    a_s, a_e, a_c = dbg["a_raw"][:, 0]
    r2 = math.sqrt(0.5)
    c8 = math.cos(math.pi / 8)
    np.testing.assert_allclose(a_e, [-r2, -r2, -c8, -c8], atol=1e-14)
    np.testing.assert_allclose(a_c, [-1.0, -r2, -c8, -c8], atol=1e-14)
    sx, sy = 2 + r2, 1 + r2                       # sum of the four unit vectors
    ns = math.hypot(sx, sy)
    np.testing.assert_allclose(a_s, [-sx / ns, -sy / ns, -(sx + sy) * r2 / ns, -sx / ns], atol=1e-14)
    np.testing.assert_allclose(dbg["mu_s"][0], [sx / 4, sy / 4], atol=1e-15)
    np.testing.assert_allclose(dbg["mu_e"][0], [[0.5, 0.5], [(1 + r2) / 2, r2 / 2]], atol=1e-15)
    np.testing.assert_allclose(dbg["mu_c"][0, 0], [1, 0], atol=1e-15)          # window of one token
    np.testing.assert_allclose(dbg["mu_c"][0, 2], [r2 / 2, (1 + r2) / 2], atol=1e-15)


def test_window_and_block_extent_closed_form():
    """Token 0 = e0, all others = e1: the only thing that varies is whether token 0 is inside a block or a
    window, which pins W, the inclusive causal window [max(0,i-W+1), i], b and the block origin."""
    N, d = 300, 8
    keys = np.zeros((1, N, d), np.float32)
    keys[0, 0, 0] = 1.0
    keys[0, 1:, 1] = 5.0
    p = Params()
    _, dbg = oracle.score_layer(keys, p, debug=("a_raw",))
    a_s, a_e, a_c = dbg["a_raw"][:, 0]
    i = np.arange(N, dtype=np.float64)
    W, b = 64, 128                                           # floor(300/32) = 9 -> clipped to 128
    exp_c = np.where(i < W, -i / np.sqrt(1 + i * i), -1.0)   # token 0 leaves the window at i = W
    exp_c[0] = -1.0
    np.testing.assert_allclose(a_c, exp_c, atol=1e-14)
    exp_e = np.full(N, -1.0)
    exp_e[1:b] = -(b - 1) / math.sqrt(1 + (b - 1) ** 2)
    exp_e[0] = -1 / math.sqrt(1 + (b - 1) ** 2)
    np.testing.assert_allclose(a_e, exp_e, atol=1e-14)
    exp_s = np.full(N, -(N - 1) / math.sqrt(1 + (N - 1) ** 2))
    exp_s[0] = -1 / math.sqrt(1 + (N - 1) ** 2)
    np.testing.assert_allclose(a_s, exp_s, atol=1e-14)


def test_short_last_block_divides_by_own_length():
    """N = 130, b = 128: the last block holds 2 tokens at right angles -> both see cos 45 deg."""
    N, d = 130, 4
    keys = np.zeros((1, N, d), np.float32)
    keys[0, :, 0] = 1.0
    keys[0, 128] = [0, 1, 0, 0]
    keys[0, 129] = [0, 0, 1, 0]
    _, dbg = oracle.score_layer(keys, debug=("a_raw", "mu_e"))
    np.testing.assert_allclose(dbg["a_raw"][1, 0, 128:], [-math.sqrt(0.5)] * 2, atol=1e-14)
    np.testing.assert_allclose(dbg["mu_e"][0, 1], [0, 0.5, 0.5, 0], atol=1e-15)   # a mean, not a sum


# --------------------------------------------------------------------------- anchors vs independent means
def test_anchors_equal_naive_means_and_cumsum():
    """Stable / block / window anchors equal means computed here two other ways (direct slices; the
    cumulative-sum form Appendix A mentions)."""
    H, N, d = 2, 700, 16
    keys = _rand_keys(H, N, d, seed=3)
    _, dbg = oracle.score_layer(keys, debug=("mu_s", "mu_e", "mu_c"))
    kh = keys.astype(np.float64)
    kh /= np.linalg.norm(kh, axis=-1, keepdims=True)
    np.testing.assert_allclose(dbg["mu_s"], kh.mean(axis=1), atol=1e-13)
    b = 128
    for blk in range((N + b - 1) // b):
        np.testing.assert_allclose(dbg["mu_e"][:, blk], kh[:, blk * b:(blk + 1) * b].mean(axis=1), atol=1e-13)
    cs = np.concatenate([np.zeros((H, 1, d)), np.cumsum(kh, axis=1)], axis=1)
    for i in (0, 1, 62, 63, 64, 65, 400, N - 1):
        lo = max(0, i - 63)
        np.testing.assert_allclose(dbg["mu_c"][:, i], kh[:, lo:i + 1].mean(axis=1), atol=1e-13)
        np.testing.assert_allclose(dbg["mu_c"][:, i], (cs[:, i + 1] - cs[:, lo]) / (i + 1 - lo), atol=1e-12)


def test_anomalies_are_scipy_cosine_distance_minus_one():
    """a = -cos, checked with scipy's cosine distance (1 - cos) against anchors rebuilt with numpy."""
    H, N, d = 1, 300, 12
    keys = _rand_keys(H, N, d, seed=5)
    _, dbg = oracle.score_layer(keys, debug=("a_raw",))
    kh = keys[0].astype(np.float64)
    kh /= np.linalg.norm(kh, axis=-1, keepdims=True)
    mu = kh.mean(axis=0)
    for i in (0, 7, 150, 299):
        assert dbg["a_raw"][0, 0, i] == pytest.approx(ssd.cosine(kh[i], mu) - 1.0, abs=1e-13)
        assert dbg["a_raw"][1, 0, i] == pytest.approx(ssd.cosine(kh[i], kh[(i // 128) * 128:(i // 128 + 1) * 128].sum(0)) - 1.0, abs=1e-13)
        assert dbg["a_raw"][2, 0, i] == pytest.approx(ssd.cosine(kh[i], kh[max(0, i - 63):i + 1].sum(0)) - 1.0, abs=1e-13)


# --------------------------------------------------------------------------- invariants
def test_scale_invariance_bit_exact_for_powers_of_two():
    """Scores depend on key directions only (Section 2.1): scaling each key by its own power of two changes
    nothing, bit for bit."""
    keys = _rand_keys(2, 500, 32, seed=7)
    rng = np.random.default_rng(8)
    scale = np.exp2(rng.integers(-6, 7, size=(2, 500, 1))).astype(np.float32)
    s0, _ = oracle.score_layer(keys)
    s1, _ = oracle.score_layer(keys * scale)
    assert np.array_equal(s0, s1)
    s2, _ = oracle.score_layer(keys * rng.uniform(0.3, 3.0, size=(2, 500, 1)).astype(np.float32))
    np.testing.assert_allclose(s2[:, 4:], s0[:, 4:], atol=2e-6)   # inputs re-rounded to fp32


def test_ranges_and_orderings():
    keys = _rand_keys(3, 900, 24, seed=9)
    s, dbg = oracle.score_layer(keys, debug=("a_raw", "a_tilde", "w", "blend", "win", "alpha", "surprise"))
    at = dbg["a_tilde"]
    assert np.all(at.min(axis=2) == 0.0) and np.all(at.max(axis=2) == 1.0)
    np.testing.assert_allclose(dbg["w"].sum(axis=1), 1.0, atol=1e-15)
    assert np.all(dbg["a_raw"][2, :, 0] == -1.0)              # window of the first token is the token
    assert np.all(dbg["blend"] <= dbg["win"] + 1e-15)
    un = s[:, 4:].astype(np.float64)
    assert np.all(un >= dbg["blend"][:, 4:] - 1e-7) and np.all(un <= dbg["win"][:, 4:] + 1e-7)
    assert np.all((un >= 0) & (un <= 1))
    assert np.all(s[:, :4] == oracle.PIN)
    assert np.all((dbg["alpha"] > 0) & (dbg["alpha"] < 1)) and np.all(dbg["surprise"] >= 0)


def test_minmax_is_affine_invariant_per_scale():
    """min-max within the head: rebuilt from a_raw with numpy's min / max / ptp."""
    keys = _rand_keys(2, 400, 16, seed=10)
    _, dbg = oracle.score_layer(keys, debug=("a_raw", "a_tilde"))
    a = dbg["a_raw"]
    np.testing.assert_allclose(dbg["a_tilde"], (a - a.min(2, keepdims=True)) / np.ptp(a, axis=2, keepdims=True),
                               atol=1e-15)


def test_reliability_gap_matches_numpy_sort():
    """Delta_k from np.sort / np.partition on the normalised scores (Section 2.4, p = 10 %)."""
    keys = _rand_keys(2, 1000, 16, seed=11)
    _, dbg = oracle.score_layer(keys, debug=("a_tilde", "delta"))
    m = 100
    for h in range(2):
        for k in range(3):
            x = np.sort(dbg["a_tilde"][k, h])
            assert dbg["delta"][h, k] == pytest.approx(x[-m:].mean() - x[:m].mean(), abs=1e-14)
    # tiny N: the sets hold max(1, floor(0.1 N)) = 1 element, so every gap is max - min = 1
    _, dbg = oracle.score_layer(_rand_keys(1, 7, 8, seed=12), debug=("delta",))
    np.testing.assert_allclose(dbg["delta"], 1.0, atol=1e-15)


def test_weights_are_scipy_softmax_of_logprior_plus_beta_delta():
    keys = _rand_keys(2, 600, 16, seed=13)
    for beta in (0.0, 3.0, 7.5):
        _, dbg = oracle.score_layer(keys, Params(beta=beta), debug=("delta", "w"))
        z = np.log([0.4, 0.4, 0.2])[None, :] + beta * dbg["delta"]
        np.testing.assert_allclose(dbg["w"], scipy.special.softmax(z, axis=1), atol=1e-15)
        if beta == 0.0:
            np.testing.assert_allclose(dbg["w"], [[0.4, 0.4, 0.2]] * 2, atol=1e-15)   # falls back on the prior


def test_equal_gaps_fall_back_on_prior_ratio():
    """N <= b makes the episodic reading identical to the stable one, so their gaps are equal and the
    weight ratio w_s / w_e must be the prior ratio (= 1), whatever beta is."""
    keys = _rand_keys(1, 100, 16, seed=14)
    _, dbg = oracle.score_layer(keys, Params(beta=5.0), debug=("a_raw", "w", "delta"))
    np.testing.assert_allclose(dbg["a_raw"][0], dbg["a_raw"][1], atol=1e-14)
    assert dbg["w"][0, 0] == pytest.approx(dbg["w"][0, 1], rel=1e-12)


def test_surprise_gate_and_route_from_numpy():
    """s = numpy population std over the three readings; min-max, centre, rectify; scipy expit gate; route."""
    keys = _rand_keys(2, 800, 16, seed=15)
    p = Params()
    s, dbg = oracle.score_layer(keys, p, debug=("a_tilde", "w", "surprise", "alpha", "blend", "win"))
    at = dbg["a_tilde"]
    sd = at.std(axis=0)                                     # ddof = 0
    sd = (sd - sd.min(1, keepdims=True)) / np.ptp(sd, axis=1, keepdims=True)
    sp = np.maximum(sd - sd.mean(1, keepdims=True), 0.0)
    np.testing.assert_allclose(dbg["surprise"], sp, atol=1e-14)
    alpha = scipy.special.expit(p.kappa * (sp - p.tau))
    np.testing.assert_allclose(dbg["alpha"], alpha, atol=1e-14)
    np.testing.assert_allclose(dbg["blend"], np.einsum("hk,khn->hn", dbg["w"], at), atol=1e-14)
    np.testing.assert_allclose(dbg["win"], at.max(axis=0), atol=0)
    star = (1 - alpha) * dbg["blend"] + alpha * dbg["win"]
    np.testing.assert_array_equal(s[:, 4:], star[:, 4:].astype(np.float32))
    # literal reading of the gate (raw std) is reachable too
    _, dbg1 = oracle.score_layer(keys, Params(surprise_mode=1), debug=("surprise",))
    np.testing.assert_allclose(dbg1["surprise"], at.std(axis=0), atol=1e-14)


def test_std_convention_is_immaterial_after_minmax():
    keys = _rand_keys(2, 500, 16, seed=16)
    s0, _ = oracle.score_layer(keys, Params(std_ddof=0))
    s1, _ = oracle.score_layer(keys, Params(std_ddof=1))
    np.testing.assert_allclose(s0[:, 4:], s1[:, 4:], atol=1e-7)


def test_two_scale_variant_is_the_two_reading_computation():
    """Appendix "Component and Scale Ablations", row "Stable + episodic (no current)": with the current scale
    switched off (scale_mask 3) blend, winner and surprise are those of the two remaining readings -- scipy
    softmax over two logits, numpy maximum and numpy std over two rows, scipy expit gate.  The reading of the
    switched-off scale must not enter anywhere: replacing it changes nothing."""
    keys = _rand_keys(2, 900, 16, seed=31)
    p = Params(scale_mask=3)
    s, dbg = oracle.score_layer(keys, p, debug=("a_tilde", "delta", "w"))
    at = dbg["a_tilde"][:2]                                  # stable, episodic
    w = scipy.special.softmax(np.log([0.4, 0.4])[None, :] + p.beta * dbg["delta"][:, :2], axis=1)
    np.testing.assert_allclose(dbg["w"][:, :2], w, atol=1e-15)
    np.testing.assert_array_equal(dbg["w"][:, 2], 0.0)
    blend = np.einsum("hk,khn->hn", w, at)
    win = np.maximum(at[0], at[1])
    sd = np.std(at, axis=0)                                  # population std of two numbers = |x - y| / 2
    np.testing.assert_allclose(sd, np.abs(at[0] - at[1]) / 2, atol=1e-15)
    sd = (sd - sd.min(1, keepdims=True)) / np.ptp(sd, axis=1, keepdims=True)
    sp = np.maximum(sd - sd.mean(1, keepdims=True), 0.0)
    alpha = scipy.special.expit(p.kappa * (sp - p.tau))
    star = (1 - alpha) * blend + alpha * win
    np.testing.assert_allclose(s[:, 4:], star[:, 4:], atol=1e-7)
    # the switched-off reading does not enter: window 1 makes every current anomaly -1 (a flat scale)
    s_flat, _ = oracle.score_layer(keys, Params(scale_mask=3, window=1))
    np.testing.assert_array_equal(s, s_flat)
    # and it differs from merely giving the scale a zero prior weight, which still lets it win and surprise
    s_prior0, _ = oracle.score_layer(keys, Params(prior=(0.4, 0.4, 0.0)))
    assert np.abs(s_prior0[:, 4:] - s[:, 4:]).max() > 1e-3
    # all three scales on is the default, bit for bit
    np.testing.assert_array_equal(oracle.score_layer(keys, Params(scale_mask=7))[0], oracle.score_layer(keys)[0])


def test_single_scale_mask_is_the_single_anchor_score():
    """One scale left: std of one reading is 0, blend = winner = that reading ("Single-scale stable score")."""
    keys = _rand_keys(1, 300, 16, seed=32)
    for k in range(3):
        s, dbg = oracle.score_layer(keys, Params(scale_mask=1 << k, n_sink=0), debug=("a_tilde",))
        np.testing.assert_allclose(s[0], dbg["a_tilde"][k, 0], atol=1e-7)
    with pytest.raises(RuntimeError):
        oracle.score_layer(keys, Params(scale_mask=0))


def test_flat_range_rule():
    """Min-max of a range below 1e-6 gives all zeros, of a range above it the plain (a - min) / (max - min).
    The bound is this build's own constant (the paper says only "min-max normalized within its head").  Keys on
    a narrow arc of the unit circle make the spread of a scale as small as wanted: for angles within +-t of the
    mean direction the stable anomalies -cos span about t^2 / 2."""
    for t, flat in ((1.0e-3, True), (2.5e-3, False)):         # ranges ~5e-7 and ~3e-6
        ang = np.linspace(-t, t, 41)
        keys = np.stack([np.cos(ang), np.sin(ang)], axis=-1)[None].astype(np.float32)
        p = Params(block_div=1000, block_min=64, block_max=64, window=41, n_sink=0)
        _, dbg = oracle.score_layer(keys, p, debug=("a_raw", "a_tilde"))
        a = dbg["a_raw"][0, 0]
        rng_ = a.max() - a.min()
        assert (rng_ < 1e-6) == flat, rng_
        want = np.zeros_like(a) if flat else (a - a.min()) / (a.max() - a.min())
        np.testing.assert_allclose(dbg["a_tilde"][0, 0], want, atol=1e-12)


# --------------------------------------------------------------------------- special cases (ablation variants)
def test_single_anchor_variant_is_minmaxed_negative_cosine_to_mean():
    """Prior (1,0,0), beta = 0, 'only average' -> the single-anchor key-distinctiveness score of the
    'w/o continuum' ablation (Section 3.4): min-max of -cos(k_hat, mean k_hat)."""
    keys = _rand_keys(2, 300, 16, seed=17)
    s, _ = oracle.score_layer(keys, Params(prior=(1.0, 0.0, 0.0), beta=0.0, gate_mode=1, n_sink=0))
    kh = keys.astype(np.float64)
    kh /= np.linalg.norm(kh, axis=-1, keepdims=True)
    for h in range(2):
        a = np.array([ssd.cosine(kh[h, i], kh[h].mean(0)) - 1.0 for i in range(300)])
        a = (a - a.min()) / (a.max() - a.min())
        np.testing.assert_allclose(s[h], a, atol=1e-7)


def test_only_max_variant():
    keys = _rand_keys(1, 300, 16, seed=18)
    s, dbg = oracle.score_layer(keys, Params(gate_mode=2, n_sink=0), debug=("a_tilde",))
    np.testing.assert_array_equal(s[0], dbg["a_tilde"][:, 0].max(axis=0).astype(np.float32))


def test_window_covering_prompt_equals_stable_at_last_token():
    keys = _rand_keys(1, 50, 16, seed=19)
    _, dbg = oracle.score_layer(keys, Params(window=50), debug=("a_raw",))
    assert dbg["a_raw"][2, 0, -1] == pytest.approx(dbg["a_raw"][0, 0, -1], abs=1e-14)
    assert abs(dbg["a_raw"][2, 0, 10] - dbg["a_raw"][0, 0, 10]) > 1e-6


def test_constant_keys_give_zero_scores_and_first_indices():
    keys = np.ones((2, 40, 8), np.float32) * np.float32(0.37)
    s, dbg = oracle.score_layer(keys, debug=("a_tilde",))
    assert np.all(dbg["a_tilde"] == 0.0) and np.all(s[:, 4:] == 0.0)
    B = oracle.budget_layer(s, 0.5)
    # pins first; m_safe = 4 marks exactly the pins; the remaining 32 slots go to the lowest flat indices
    assert B.tolist() == [36, 4]
    assert oracle.select_head(s[0], 36).tolist() == list(range(36))
    assert oracle.select_head(s[1], 4).tolist() == [0, 1, 2, 3]


def test_zero_key_is_harmless():
    keys = _rand_keys(1, 200, 8, seed=20)
    keys[0, 17] = 0.0
    s, dbg = oracle.score_layer(keys, debug=("a_raw",))
    assert np.all(np.isfinite(s)) and np.all(dbg["a_raw"][:, 0, 17] == 0.0)


def test_sink_counts():
    keys = _rand_keys(1, 3, 8, seed=21)
    assert np.all(oracle.score_layer(keys)[0] == oracle.PIN)             # N <= n_sink: everything pinned
    s, _ = oracle.score_layer(_rand_keys(1, 30, 8, seed=22), Params(n_sink=0))
    assert np.all(s <= 1.0)


# --------------------------------------------------------------------------- budgets
def _brute_budget(scores, k0, ms):
    """Independent statement of the competition: python sorts on tuples."""
    H, N = scores.shape
    B = [ms] * H
    pool = []
    for h in range(H):
        order = sorted(range(N), key=lambda i: (-float(scores[h, i]), i))
        pool += [(-float(scores[h, i]), h, i) for i in order[ms:]]
    pool.sort()
    for _, h, _ in pool[:H * k0 - H * ms]:
        B[h] += 1
    return B


def _threshold_budget(scores, k0, ms):
    """The same allocation in threshold form: B_h = max(m_safe, #{i: (h,i) among the layer's best that fit})."""
    H, N = scores.shape
    flat = sorted(((-float(scores[h, i]), h, i) for h in range(H) for i in range(N)))
    # grow the number of globally admitted pairs until the total with floors reaches H*k0
    cnt = [0] * H
    total = H * ms
    for _, h, _ in flat:
        if total == H * k0:
            break
        cnt[h] += 1
        if cnt[h] > ms:
            total += 1
    return [max(ms, c) for c in cnt]


@pytest.mark.parametrize("seed", range(6))
def test_budget_matches_brute_force_and_threshold_form(seed):
    rng = np.random.default_rng(seed)
    H, N = int(rng.integers(1, 5)), int(rng.integers(5, 60))
    scores = rng.random((H, N)).astype(np.float32)
    if seed % 2:
        scores = np.round(scores * 4) / 4                   # heavy ties
    scores[:, :min(4, N)] = oracle.PIN
    for r in (0.0, 0.3, 0.5, 0.9, 1.0):
        k0 = oracle.k0(N, r)
        ms = oracle.m_safe(k0)
        B = oracle.budget_layer(scores, r)
        assert B.tolist() == _brute_budget(scores, k0, ms)
        assert B.tolist() == _threshold_budget(scores, k0, ms)
        assert B.sum() == H * k0 and B.min() >= ms and B.max() <= N


def test_budget_special_cases():
    rng = np.random.default_rng(0)
    s = rng.random((4, 100)).astype(np.float32)
    assert oracle.budget_layer(s, 0.0).tolist() == [100] * 4                 # r = 0 keeps everything
    assert oracle.budget_layer(s, 1.0).tolist() == [0] * 4
    assert oracle.budget_layer(s, 0.6, safeguard=1.0).tolist() == [40] * 4   # uniform budget ("w/o adaptive")
    s[2] += 10.0                                                             # one head dominates the layer
    B = oracle.budget_layer(s, 0.5)                                          # k0 = 50, m_safe = 10
    assert B.tolist() == [10, 10, 100, 80] or (B[2] == 100 and B.sum() == 200 and B.min() >= 10)


# --------------------------------------------------------------------------- selection
def test_selection_exhaustive_ties_tiny():
    """Every score pattern over {0, 1, 2}^N for N = 5 and every budget, against python's sorted()."""
    N = 5
    for pattern in itertools.product((0.0, 1.0, 2.0), repeat=N):
        s = np.array(pattern, np.float32)
        for B in range(N + 1):
            exp = sorted(sorted(range(N), key=lambda i: (-pattern[i], i))[:B])
            assert oracle.select_head(s, B).tolist() == exp


def test_selection_random_vs_argsort_and_gather_bitwise():
    rng = np.random.default_rng(1)
    for N in (1, 2, 17, 64, 257):
        s = (np.round(rng.random(N) * 20) / 20).astype(np.float32)
        rows = rng.integers(0, 2 ** 16, size=(N, 6), dtype=np.uint16)
        for B in {0, 1, N // 2, N}:
            kept = oracle.select_head(s, B)
            order = np.lexsort((np.arange(N), -s.astype(np.float64)))      # score desc, index asc
            assert kept.tolist() == sorted(order[:B].tolist())
            assert np.all(np.diff(kept) > 0)
            assert np.array_equal(oracle.gather_rows(rows, kept), rows[kept])


def test_negative_zero_ties_with_positive_zero():
    s = np.array([0.0, -0.0, 0.0, -0.0, 1.0], np.float32)
    assert oracle.select_head(s, 3).tolist() == [0, 1, 4]


def test_r_zero_keeps_everything_bitwise():
    H, N, d = 2, 70, 8
    keys = _rand_keys(H, N, d, seed=30)
    vals = _rand_keys(H, N, d, seed=31)
    out = oracle.compress(keys[None], keys[None].view(np.uint32), vals[None].view(np.uint32), [0, N], [0.0])
    assert out.k_per_head.reshape(-1).tolist() == [N, N]
    assert np.array_equal(out.packed_k.reshape(H, N, d), keys.view(np.uint32))
    assert np.array_equal(out.packed_v.reshape(H, N, d), vals.view(np.uint32))
    assert out.kept_idx.tolist() == list(range(N)) * 2


def test_planted_outliers_are_kept_on_tiny_workload():
    """Sanity on the synthetic mixture (not a paper claim): keys planted orthogonal to the mean direction are
    the most anomalous under every anchor and must survive r = 0.5."""
    import nkv_inputs
    w = nkv_inputs.WORKLOADS["tiny"]
    k, _ = nkv_inputs.layer_keys_values(w, 0, 0)
    kf = k.float().numpy()
    s, _ = oracle.score_layer(kf)
    B = oracle.budget_layer(s, 0.5)
    for h in range(w.H):
        kept = set(oracle.select_head(s[h], int(B[h])).tolist())
        planted = np.where(np.abs(np.linalg.norm(kf[h].astype(np.float64), axis=-1) - 6.0) < 1e-3)[0]
        assert len(planted) == w.n_out                      # ordinary keys have norm ~ sqrt(d + 11)
        assert set(planted.tolist()) <= kept
