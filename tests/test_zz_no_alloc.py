"""alcs_topn_mask_static, the selection entry point that allocates nothing (its state lives in a
device array inside the library), against alcs_topn_mask with a caller-provided workspace: same
flags and per-segment counts, bit for bit, on two calls in a row that share the array - the second
on a smaller input with fewer segments, so that anything the first call left behind would show."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs

pytestmark = pytest.mark.gpu


def scores(n, seed):
    rng = np.random.default_rng(seed)
    s = (rng.random(n) ** 3).astype(np.float32)
    s[rng.integers(0, n, n // 8)] = np.float32(0.125)   # ties
    s[rng.integers(0, n, n // 16)] = np.float32(0.0)
    return s


def check(n, cuts, N, seed):
    import torch
    s = scores(n, seed)
    sd = torch.from_numpy(s).cuda()
    ref_mask, ref_counts = alcs.alcs_topn_mask(sd, N, seg_starts=cuts)
    mask = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    counts = alcs.alcs_topn_mask_static(sd, N, seg_starts=cuts, mask=mask)
    torch.cuda.synchronize()
    got = mask.cpu().numpy()
    assert got.tobytes() == ref_mask.cpu().numpy().tobytes(), "n=%d N=%d" % (n, N)
    assert list(counts) == list(ref_counts)
    assert got.tobytes() == oracle.topn_mask(s, N).tobytes()
    assert int(counts.sum()) == N


def test_two_calls_in_a_row_second_smaller():
    check(70001, [0, 5, 9000, 9000, 33333, 60000, 70001], 23456, 1)
    check(5000, [0, 1200, 5000], 777, 2)
    # counts only, one segment, everything / nothing kept
    import torch
    sd = torch.from_numpy(scores(300, 3)).cuda()
    assert list(alcs.alcs_topn_mask_static(sd, 300)) == [300]
    assert list(alcs.alcs_topn_mask_static(sd, 0)) == [0]


def test_too_many_segments_is_rejected():
    import torch
    n = 4000
    sd = torch.from_numpy(scores(n, 4)).cuda()
    cuts = list(range(0, 1025)) + [n]        # 1025 segments
    with pytest.raises(alcs.AlcsError) as e:
        alcs.alcs_topn_mask_static(sd, 10, seg_starts=cuts)
    assert e.value.status == -2              # ALCS_E_UNSUPPORTED
    cuts = list(range(0, 1024)) + [n]        # 1024 segments: the maximum
    mask = torch.empty((n,), dtype=torch.uint8, device="cuda")
    counts = alcs.alcs_topn_mask_static(sd, 1500, seg_starts=cuts, mask=mask)
    ref_mask, ref_counts = alcs.alcs_topn_mask(sd, 1500, seg_starts=cuts)
    assert mask.cpu().numpy().tobytes() == ref_mask.cpu().numpy().tobytes()
    assert list(counts) == list(ref_counts)
