"""quaff_check_outliers: the device-side validity scan of an outlier channel set (Sec. 3.3 fixes O before
fine-tuning; every per-step call uses its entries as column indices unchecked)."""
import numpy as np
import pytest
import torch

from paper_2505_14742_amd import binding as q
from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _check(values, c_in):
    O = torch.tensor(values, dtype=torch.int32, device=DEV) if len(values) else None
    res = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    q.check_outliers(O, c_in, res)
    torch.cuda.synchronize()
    return int(res.item())


def test_valid_lists():
    assert _check([], 64) == 0
    assert _check([0], 64) == 0
    assert _check([0, 1, 2, 63], 64) == 0
    assert _check(list(range(0, 8192, 10)), 8192) == 0           # longer than one pass of the workgroup
    for cfg in (2, 3, 4, 5, 6):
        for p in synth.CONFIGS[cfg]:
            assert _check(synth.outlier_indices(p).tolist(), p.c_in) == 0, (cfg, p.name)


def test_invalid_lists_report_the_first_offending_position():
    assert _check([5, 5], 64) == 2                               # duplicate
    assert _check([3, 9, 7, 20], 64) == 3                        # descending pair
    assert _check([3, 9, 64], 64) == 3                           # out of range above
    assert _check([-1, 4], 64) == 1                              # out of range below
    assert _check([1, 2, 3, 4, 9, 8, 2, 1], 64) == 6             # several offenders: the first is reported
    long = list(range(0, 4000))
    long[3000] = 2999                                            # one duplicate deep inside a long list
    assert _check(long, 4096) == 3001
    rng = np.random.default_rng(5)
    for _ in range(5):
        v = np.sort(rng.choice(5000, 700, replace=False)).tolist()
        k = int(rng.integers(1, 700))
        v[k] = v[k - 1] - int(rng.integers(0, 3))
        assert _check(v, 5000) == k + 1
