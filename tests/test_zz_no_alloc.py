"""The entry point that allocates nothing (nkv_budget_noalloc) gives nkv_budget's budgets bit for bit.

Two calls in a row on one stream, the second on a smaller input, so that whatever the first call left in the
library's static scratch array is there when the second one starts."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_26678_amd as nkv

pytestmark = pytest.mark.gpu


def _scores(L, H, cu, seed):
    """Seeded scores on a [0, 1] scale with many exact ties and pinned sink positions."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    T = cu[-1]
    s = torch.rand(L, H, T, generator=g)
    s = torch.where(torch.rand(L, H, T, generator=g) < 0.3, torch.round(s * 64) / 64, s)   # ties
    for p in range(len(cu) - 1):
        s[:, :, cu[p]:min(cu[p] + 4, cu[p + 1])] = nkv.PIN
    return s.contiguous()


def _both(L, H, cu, r, seed, flags=0):
    shape = nkv.Shape(L, H, 128, 128, nkv.DTYPE_BF16, cu)
    params = nkv.params_default(flags=flags)
    s = _scores(L, H, cu, seed).cuda()
    ws = torch.empty(max(nkv.workspace_bytes(shape, params), 256), dtype=torch.uint8, device="cuda")
    want = torch.full((shape.n_prompts, L, H), -1, dtype=torch.int32, device="cuda")
    got = torch.full_like(want, -2)
    nkv.budget(s, shape, params, r, want, ws)
    nkv.budget_noalloc(s, shape, params, r, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want), f"L={L} H={H} cu={cu}: budgets differ"
    return s.cpu().numpy(), got.cpu().numpy(), params


@pytest.mark.parametrize("flags", [0, nkv.FLAG_BUDGET_PER_HEAD])
def test_two_calls_in_a_row_match_nkv_budget(flags):
    # slice-wise kernels (a prompt of more than 8192 tokens), then a smaller ragged input
    big = _both(3, 8, [0, 20000, 20700], [0.75, 0.5], 11, flags)
    small = _both(2, 4, [0, 333, 2381], [0.9, 0.75], 12, flags)
    for (s, B, params), cu, r in ((big, [0, 20000, 20700], [0.75, 0.5]), (small, [0, 333, 2381], [0.9, 0.75])):
        for p in range(len(cu) - 1):                      # and the oracle agrees on a layer of each
            ref = oracle.budget_layer(s[0, :, cu[p]:cu[p + 1]], r[p], params.safeguard)
            assert np.array_equal(B[p, 0], ref)


def test_shape_beyond_the_static_scratch_is_refused():
    shape = nkv.Shape(36, 8, 128, 128, nkv.DTYPE_BF16, [0, 131072 * 2])
    params = nkv.params_default()
    s = torch.empty(8, device="cuda")                     # never read: the call must fail on the host
    k = torch.empty(36 * 8, dtype=torch.int32, device="cuda")
    with pytest.raises(nkv.NkvError) as e:
        nkv.budget_noalloc(s, shape, params, [0.75], k)
    assert e.value.status == nkv.NKV_ESCRATCH
