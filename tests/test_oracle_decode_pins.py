"""Pins of the decode-attention oracle (oracle/decode.py) against library routines, closed forms and
invariants; no GPU.  The operation is plain softmax attention over the rows the compression operator kept
(paper Section 2.5 for the cache layout, Appendix A for "retained keys and values are unchanged")."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

from oracle.decode import decode_attention


def _cache(P, L, H, d, dv, lens, seed=0):
    """Random ragged cache: lens[u] rows for unit u in (p, l, h) order."""
    rng = np.random.default_rng(seed)
    head_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = int(head_off[-1])
    return rng.standard_normal((rows, d)), rng.standard_normal((rows, dv)), head_off


def test_matches_scipy_softmax_and_logsumexp_row_by_row():
    P, L, H, Hq, d, dv = 2, 2, 2, 6, 8, 5
    rng = np.random.default_rng(1)
    lens = rng.integers(1, 9, size=P * L * H)
    K, V, off = _cache(P, L, H, d, dv, lens, seed=2)
    q = rng.standard_normal((P, L, Hq, d))
    out, lse = decode_attention(q, K, V, off, H, 0.37)
    G = Hq // H
    for p in range(P):
        for l in range(L):
            for j in range(Hq):
                u = (p * L + l) * H + j // G
                rows = range(int(off[u]), int(off[u + 1]))
                s = np.array([0.37 * sum(q[p, l, j, c] * K[i, c] for c in range(d)) for i in rows])
                w = softmax(s)
                want = sum(w[n] * V[i] for n, i in enumerate(rows))
                assert np.allclose(out[p, l, j], want, rtol=0, atol=1e-13)
                assert abs(lse[p, l, j] - logsumexp(s)) < 1e-13


def test_full_cache_equals_torch_sdpa_with_repeated_kv_heads():
    """Nothing evicted and equal lengths: the library's scaled-dot-product attention, KV heads repeated G times."""
    P, L, H, Hq, d, n = 1, 3, 2, 8, 16, 37
    rng = np.random.default_rng(3)
    K, V, off = _cache(P, L, H, d, d, [n] * (P * L * H), seed=4)
    q = rng.standard_normal((P, L, Hq, d))
    out, _ = decode_attention(q, K, V, off, H, 1.0 / np.sqrt(d))
    G = Hq // H
    for l in range(L):
        Kl = torch.tensor(K[l * H * n:(l + 1) * H * n].reshape(H, n, d)).repeat_interleave(G, dim=0)
        Vl = torch.tensor(V[l * H * n:(l + 1) * H * n].reshape(H, n, d)).repeat_interleave(G, dim=0)
        ql = torch.tensor(q[0, l]).unsqueeze(1)                       # [Hq, 1, d]
        want = torch.nn.functional.scaled_dot_product_attention(ql[None], Kl[None], Vl[None])[0, :, 0]
        assert np.allclose(out[0, l], want.numpy(), rtol=0, atol=1e-12)


def test_single_row_returns_that_value_row_and_its_logit():
    K, V, off = _cache(1, 1, 1, 4, 3, [1], seed=5)
    q = np.array([[[[1.0, -2.0, 0.5, 3.0]]]])
    out, lse = decode_attention(q, K, V, off, 1, 0.5)
    assert np.array_equal(out[0, 0, 0], V[0])
    assert abs(lse[0, 0, 0] - 0.5 * float(K[0] @ q[0, 0, 0])) < 1e-15


def test_zero_scale_is_the_mean_of_the_values():
    K, V, off = _cache(1, 1, 2, 4, 6, [7, 3], seed=6)
    q = np.random.default_rng(7).standard_normal((1, 1, 4, 4))
    out, lse = decode_attention(q, K, V, off, 2, 0.0)
    for j in range(4):
        a, b = (0, 7) if j < 2 else (7, 10)
        assert np.allclose(out[0, 0, j], V[a:b].mean(axis=0), atol=1e-15)
        assert abs(lse[0, 0, j] - np.log(b - a)) < 1e-15


def test_row_order_inside_a_unit_does_not_matter():
    K, V, off = _cache(1, 1, 1, 8, 8, [20], seed=8)
    q = np.random.default_rng(9).standard_normal((1, 1, 2, 8))
    a, la = decode_attention(q, K, V, off, 1, 0.3)
    perm = np.random.default_rng(10).permutation(20)
    b, lb = decode_attention(q, K[perm], V[perm], off, 1, 0.3)
    assert np.allclose(a, b, atol=1e-14) and np.allclose(la, lb, atol=1e-14)


def test_query_head_j_reads_kv_head_j_div_g_and_units_are_ordered_prompt_layer_head():
    P, L, H, Hq, d = 2, 3, 2, 6, 4
    lens = np.arange(1, P * L * H + 1)
    K, _, off = _cache(P, L, H, d, 1, lens, seed=11)
    V = np.concatenate([np.full((n, 1), float(u)) for u, n in enumerate(lens)])      # value = unit index
    q = np.random.default_rng(12).standard_normal((P, L, Hq, d))
    out, _ = decode_attention(q, K, V, off, H, 1.0)
    for p in range(P):
        for l in range(L):
            for j in range(Hq):
                assert abs(out[p, l, j, 0] - ((p * L + l) * H + j // 3)) < 1e-13


def test_two_parts_merge_through_lse_to_the_whole():
    K, V, _ = _cache(1, 1, 1, 8, 5, [30], seed=13)
    q = np.random.default_rng(14).standard_normal((1, 1, 1, 8))
    whole, lw = decode_attention(q, K, V, np.array([0, 30]), 1, 0.4)
    a, la = decode_attention(q, K[:11], V[:11], np.array([0, 11]), 1, 0.4)
    b, lb = decode_attention(q, K[11:], V[11:], np.array([0, 19]), 1, 0.4)
    wa, wb = np.exp(la - lw), np.exp(lb - lw)
    assert abs(float((wa + wb).item()) - 1.0) < 1e-13
    assert np.allclose(wa * a + wb * b, whole, atol=1e-13)


def test_empty_unit_gives_zeros_and_minus_infinity():
    K, V, off = _cache(1, 1, 2, 4, 4, [0, 5], seed=15)
    q = np.ones((1, 1, 2, 4))
    out, lse = decode_attention(q, K, V, off, 2, 1.0)
    assert np.array_equal(out[0, 0, 0], np.zeros(4)) and lse[0, 0, 0] == -np.inf
    assert np.isfinite(lse[0, 0, 1])


def test_large_logits_do_not_overflow():
    K = np.array([[100.0], [99.0]])
    V = np.array([[1.0], [0.0]])
    out, lse = decode_attention(np.array([[[[10.0]]]]), K, V, np.array([0, 2]), 1, 1.0)
    assert abs(out[0, 0, 0, 0] - 1.0 / (1.0 + np.exp(-10.0))) < 1e-15
    assert abs(lse[0, 0, 0] - (1000.0 + np.log1p(np.exp(-10.0)))) < 1e-12
