"""The entry point that allocates nothing (octo_op_nms_static) against octo_op_nms, through the C ABI."""
import numpy as np
import pytest

from oracle import postprocess as pp
from helpers import cands_to_records

pytestmark = pytest.mark.gpu


def _lists(rng, sizes, n_classes=3):
    out = []
    for n in sizes:
        xy = rng.uniform(0, 60, (n, 2)); wh = rng.uniform(5, 40, (n, 2))
        c = pp.Candidates(np.concatenate([xy, xy + wh], 1).astype(np.float32), rng.uniform(0.3, 1, n).astype(np.float32),
                          rng.integers(0, n_classes, n).astype(np.int32), rng.permutation(n).astype(np.int32))
        out.append(pp.topk(c, 1000))
    return out


def test_nms_without_allocation_two_calls_the_second_smaller(octo):
    """Two calls in a row on the library's static scratch array, the second with fewer and shorter lists (the array then
    still holds the first call's mask words): keep lists identical to octo_op_nms and to the oracle; sizes beyond the
    array are refused with nothing written."""
    import torch
    rng = np.random.default_rng(31)
    for sizes, k_cap, max_det in (((900, 64, 1, 0, 513, 1000), 1024, 300), ((130, 0, 70), 192, 7)):
        lists = _lists(rng, sizes)
        cand, count = octo.cands_to_device([cands_to_records(c) for c in lists], k_cap)
        ref_keep, ref_nk = octo.op_nms(cand, count, 0.45, max_det)
        keep = torch.full((len(sizes), max_det), -7, dtype=torch.int32, device="cuda")
        nk = torch.full((len(sizes),), -7, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        assert octo.op_nms_static(cand, count, 0.45, max_det, keep, nk) == octo.OK
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        keep, nk, ref_keep, ref_nk = keep.cpu().numpy(), nk.cpu().numpy(), ref_keep.cpu().numpy(), ref_nk.cpu().numpy()
        assert np.array_equal(nk, ref_nk)
        for f, c in enumerate(lists):
            want = pp.nms(c, 0.45, max_det).tolist()
            assert keep[f, :nk[f]].tolist() == ref_keep[f, :ref_nk[f]].tolist() == want, f
            assert np.all(keep[f, nk[f]:] == -7)
    # 65 items at k_cap 1024 need more than the static array holds: refused, outputs untouched
    n, k_cap = 65, 1024
    assert octo.lib().octo_op_nms_scratch_bytes(n, k_cap) > octo.NMS_STATIC_BYTES
    cand = torch.zeros((n, k_cap, 32), dtype=torch.uint8, device="cuda")
    count = torch.zeros(n, dtype=torch.int32, device="cuda")
    keep = torch.full((n, 4), -7, dtype=torch.int32, device="cuda")
    nk = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    assert octo.op_nms_static(cand, count, 0.45, 4, keep, nk) == octo.ECAP
    torch.cuda.synchronize()
    assert int((keep != -7).sum()) == 0 and int((nk != -7).sum()) == 0
    # exactly the limit is accepted
    assert octo.lib().octo_op_nms_scratch_bytes(64, k_cap) == octo.NMS_STATIC_BYTES
    assert octo.op_nms_static(cand[:64], count[:64], 0.45, 4, keep[:64], nk[:64]) == octo.OK
    torch.cuda.synchronize()
    assert int(nk[:64].abs().sum()) == 0
