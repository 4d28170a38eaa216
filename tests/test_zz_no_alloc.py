"""The entry point that allocates nothing, proxykv_topk_static, against proxykv_topk through the C ABI: same kept
indices, bit for bit (and the oracle's), on two calls in a row, the second with a smaller input, so that what the
first call left in the library's fixed scratch array is in the way of the second."""
import ctypes

import pytest
import torch

import oracle
from paper_2605_16360_amd import binding as pk
from paper_2605_16360_amd import synth

pytestmark = pytest.mark.gpu


def _scores(rows, N, seed):
    s = synth.normal_tensor((rows, N), seed, 61, device="cuda")
    s[1] = torch.round(s[1] * 4) / 4              # heavy ties
    s[2] = 0.5                                    # all equal
    return s


def test_topk_static_matches_topk_on_two_calls_in_a_row():
    ctx = pk.proxykv_create(pk.config_for_case(synth.CASES["tiny"]))
    lib = pk.load()
    # the first call on a device looks up the scratch array's address (the runtime loads the device image then)
    warm = torch.zeros(1, 8, device="cuda")
    warm_idx = torch.empty(1, 2, dtype=torch.int32, device="cuda")
    assert lib.proxykv_topk_static(ctx.handle, warm.data_ptr(), 1, 8, 2, warm_idx.data_ptr(), None) == pk.PROXYKV_OK
    torch.cuda.synchronize()
    assert warm_idx.tolist() == [[0, 1]]
    # long rows first (four parts per row: the scratch holds histograms and counters), then shorter rows with fewer
    # parts and a different K, then rows that need no scratch at all
    for (rows, N, K) in ((6, 170000, 51000), (4, 73729, 20000), (5, 32768, 9830)):
        s = _scores(rows, N, N)
        ref = pk.proxykv_topk(ctx, s, K)
        torch.cuda.synchronize()
        got = torch.full((rows, K), -1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.mem_get_info()[0]              # free device memory, whoever allocates
        status = lib.proxykv_topk_static(ctx.handle, s.data_ptr(), rows, N, K, got.data_ptr(), None)
        assert status == pk.PROXYKV_OK
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == before
        assert torch.equal(got, ref), (rows, N, K)
        assert torch.equal(got[:3].cpu(), oracle.topk(s[:3].cpu(), K)), (rows, N, K)
    pk.proxykv_destroy(ctx)


def test_topk_static_rejects_what_does_not_fit_before_any_device_work():
    ctx = pk.proxykv_create(pk.config_for_case(synth.CASES["tiny"]))
    lib = pk.load()
    limit = pk.proxykv_topk_static_limit()
    assert limit == 8 << 20
    one = ctypes.c_void_p(16)                     # never dereferenced
    rows = limit // ((1040 + 257 * 4) * 4) + 1    # one row too many at N = 170 000 (four parts per row)
    assert lib.proxykv_topk_static(ctx.handle, one, rows, 170000, 10, one, None) == pk.PROXYKV_ELIMIT
    assert lib.proxykv_topk_static(ctx.handle, one, 1, 8, 9, one, None) == pk.PROXYKV_EINVAL
    assert lib.proxykv_topk_static(ctx.handle, None, 1, 8, 2, one, None) == pk.PROXYKV_EINVAL
    pk.proxykv_destroy(ctx)
