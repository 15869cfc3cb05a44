"""GPU parity of the outlier-channel identification (Eq. 6) and the selection of O against the CPU oracle."""
import sys

import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run(X, offs, budgets, tag, ratio=100.0):
    import torch
    from oracle import api as orc
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV, bf16_dev, host
    t_total, c_in = X.shape
    ns = len(offs) - 1
    _say("%s: rows=%d c_in=%d samples=%d" % (tag, t_total, c_in, ns))
    Xd = bf16_dev(X)
    od = torch.from_numpy(np.asarray(offs, np.int64)).to(DEV)
    ws = torch.empty(q.calibrate_workspace_bytes(c_in, ns), dtype=torch.int8, device=DEV)
    xi_o = orc.outlier_criterion(X, np.asarray(offs, np.int64), ratio)
    for budget in budgets:
        xi = torch.full((c_in,), -7, dtype=torch.int32, device=DEV)
        O = torch.full((max(budget, 1),), -1, dtype=torch.int32, device=DEV)
        n = torch.full((1,), -1, dtype=torch.int32, device=DEV)
        q.calibrate_outliers(Xd, od, ratio, budget, xi, O if budget else None, n if budget else None, ws)
        assert np.array_equal(host(xi), xi_o), tag + " xi"
        if budget:
            want = orc.select_outliers(xi_o, budget)
            got_n = int(host(n)[0])
            assert got_n == want.size, tag + " |O| %d vs %d" % (got_n, want.size)
            assert np.array_equal(host(O)[:got_n], want), tag + " O (budget %d)" % budget
            assert np.all(host(O)[got_n:] == -1), tag + " O tail written"
    return xi_o


def test_calibrate_hand_built_ragged_samples():
    rng = np.random.default_rng(3)
    lens = [5, 0, 9, 1, 12, 130]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    K = 4096 + 64      # two column chunks, the second almost empty
    x = rng.uniform(0.5, 1.5, (sum(lens), K)).astype(np.float32) * rng.choice([-1, 1], (sum(lens), K))
    for i, chans in {0: [3, 17], 2: [17, 4100], 3: [], 4: [3, 17, 40], 5: [0, K - 1, 17]}.items():
        for c in chans:
            x[offs[i] + (c % max(lens[i], 1)), c] = -500.0 if c == 17 else 400.0
    X = synth.f32_to_bf16(x).reshape(x.shape)
    xi = _run(X, offs, [0, 1, 2, 3, 5, 64], "hand-built")
    assert xi[17] == 4 and xi[3] == 2 and xi[4100] == 1 and xi.sum() == 4 + 2 + 1 + 1 + 1 + 1


def test_calibrate_threshold_is_strict():
    row = np.ones((1, 208), np.float32)
    row[0, 0] = 200.0                      # mean = (200 + 207) / 208 < 2: 200 > 100 * mean
    X = synth.f32_to_bf16(row).reshape(1, 208)
    xi = _run(X, [0, 1], [1], "threshold")
    assert xi[0] == 1
    # exactly at the threshold: 16 columns [M, 1 x 15] with M = 100 * mean  <=>  M = 1500 / (16 - 100) < 0: impossible;
    # use ratio 4: M = 4 (M + 15) / 16  <=>  M = 5
    row = np.ones((1, 16), np.float32)
    row[0, 7] = 5.0
    X = synth.f32_to_bf16(row).reshape(1, 16)
    assert _run(X, [0, 1], [1], "threshold-equal", ratio=4.0).sum() == 0
    row[0, 7] = 5.03125
    X = synth.f32_to_bf16(row).reshape(1, 16)
    assert _run(X, [0, 1], [1], "threshold-above", ratio=4.0)[7] == 1


@pytest.mark.parametrize("cfg,name,samples,rows", [(3, "down", 8, 64), (2, "qkv", 16, 128), (5, "q", 4, 512)])
def test_calibrate_workload_recipes(cfg, name, samples, rows):
    p = synth.projection(cfg, name)
    X = np.concatenate([synth.activations(p, s, rows=slice(0, rows)) for s in range(samples)])
    offs = np.arange(samples + 1, dtype=np.int64) * rows
    planted = synth.outlier_indices(p)
    xi = _run(X, offs, [planted.size, planted.size // 2, 4 * planted.size], "cfg%d %s" % (cfg, name))
    flagged = np.flatnonzero(xi > 0)
    _say("cfg%d %s: planted %d, ever flagged %d, flagged in every sample %d" % (
        cfg, name, planted.size, flagged.size, int(np.sum(xi == samples))))
    assert flagged.size > 0
