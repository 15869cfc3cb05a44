"""quaff_scale_update_static (the entry point that allocates nothing: its scratch is static device memory inside
the library) against quaff_scale_update (caller's workspace), through the C ABI: identical bits, on two calls in a
row of which the second is smaller (fewer tokens, fewer outlier channels, so that stale scratch would show)."""
import numpy as np
import pytest
import torch

from paper_2505_14742_amd import binding as q
from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layer_state(n, c_out, n_pad):
    f32, i8 = torch.float32, torch.int8
    return dict(s=torch.ones(n, dtype=f32, device=DEV), cs=torch.ones(0, dtype=f32, device=DEV),
                what=torch.full((c_out, n_pad), 77, dtype=i8, device=DEV),
                dwh=torch.full((c_out,), -1.0, dtype=f32, device=DEV), cmax=torch.empty(n, dtype=f32, device=DEV))


def _run_case(t, c_in, c_out, outliers, seed, steps=2):
    from tests.gpu_harness import bf16_dev
    ec = synth.EdgeCase("no_alloc", t, c_in, c_out, outliers, 0)
    X, _dY, W, O, _A, _B = synth.edge_case_inputs(ec, seed)
    n, n_pad = int(O.size), q.padded_outliers(int(O.size))
    Od = torch.from_numpy(O.astype(np.int32)).to(DEV)
    W_O = torch.from_numpy(np.ascontiguousarray(W[O])).to(DEV)
    wmax = W_O.abs().amax(dim=1).contiguous()
    Xd = bf16_dev(X)
    ws = torch.empty(q.workspace_bytes(t, c_in, c_out, n, 0), dtype=torch.int8, device=DEV)
    a, b = _layer_state(n, c_out, n_pad), _layer_state(n, c_out, n_pad)
    a["cs"] = torch.ones(c_in, dtype=torch.float32, device=DEV)
    b["cs"] = torch.ones(c_in, dtype=torch.float32, device=DEV)
    for step in range(steps):   # the scales carry over from step to step on both sides
        q.scale_update(Xd, Od, W_O, wmax, c_out, 0.2, a["s"], a["cs"], a["what"], a["dwh"], a["cmax"], ws)
        q.scale_update_static(Xd, Od, W_O, wmax, c_out, 0.2, b["s"], b["cs"], b["what"], b["dwh"], b["cmax"])
        torch.cuda.synchronize()
        for key in ("s", "cs", "what", "dwh", "cmax"):
            assert torch.equal(a[key], b[key]), "%s differs at step %d (t=%d n=%d)" % (key, step, t, n)
        assert float(a["s"].max()) > 1.0, "the case must move the scales"


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    assert q.scale_update_static_max_outliers() == 1024
    big = sorted(set(int(v) for v in np.linspace(0, 2047, 90)))          # gather path, many slabs
    _run_case(2051, 2048, 1024, big, 11)
    _run_case(300, 512, 384, [3, 64, 65, 500], 12)                         # smaller in every dimension
    dense = list(range(0, 1024, 8))                                         # n * 64 >= c_in: the dense abs-max path
    _run_case(515, 1024, 256, dense, 13)


def test_static_scratch_rejects_sizes_beyond_its_maximum():
    A16 = 0x1000
    import ctypes as C
    st = q.lib().quaff_scale_update_static(A16, 64, 2048, 2048, A16, 1025, A16, A16, 64, C.c_float(0.2), A16, A16, A16,
                                           A16, None, None)
    assert st == q.ERR_SHAPE
