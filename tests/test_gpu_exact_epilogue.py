"""The product path's epilogue (LDS-staged correction product, split launch with accumulation, edge-tile clamps) with
every scale equal to 1: then Eq. 9's second line is  Y = acc1 + acc2  and the dX product is  dX = acc, exactly
representable in fp32 as long as |acc| < 2^24 - so the fp32 outputs of quaff_linear_fwd / quaff_linear_bwd_dx must
equal the integer products element for element, with no tolerance at all."""
import numpy as np
import pytest
import torch

from paper_2505_14742_amd import binding as q
from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

#        t     c_in  c_out  n_outlier
CASES = [(300, 512, 384, 0),        # edge tiles in both directions, no correction product
         (300, 512, 384, 64),       # one full outlier slice
         (257, 1024, 832, 128),     # two slices (the widest set staged in one launch)
         (2051, 3072, 3072, 31),    # the 128x192 tile's one-pass epilogue plus a ragged row tile
         (515, 1024, 576, 200),     # more than two slices: correction launch + accumulating main launch
         (2048, 256, 9216, 65),     # the 256x288 tile
         (64, 208, 144, 5),         # contraction not a multiple of 64: the register-staged kernel
         (1280, 3072, 12288, 0)]    # dX contracts over 12288 channels into a 1280 x 3072 output: the contraction is
                                    # split over two workgroups per tile, which exchange int32 partial sums


def _small_ints(seed, stream, shape, lim):
    u = synth.uniform(seed, stream, int(np.prod(shape)))
    return np.floor(u * (2 * lim + 1)).astype(np.int64).reshape(shape) - lim


@pytest.mark.parametrize("t,c_in,c_out,n", CASES, ids=["t%d_k%d_n%d_o%d" % c for c in CASES])
def test_unit_scales_give_the_integer_products_exactly(t, c_in, c_out, n):
    print("exact epilogue t=%d c_in=%d c_out=%d n=%d" % (t, c_in, c_out, n), flush=True)
    seed = 77000 + t + c_in + c_out + n
    # W holds small integers and one 127 per output channel: per-channel step 127 / 127 = 1 and codes = W
    Wi = _small_ints(seed, 1, (c_in, c_out), 7)
    Wi[0, :] = 127
    Wd = torch.from_numpy(Wi.astype(np.float32)).to(DEV)
    Wp = torch.empty(q.packed_weight_bytes(c_in, c_out), dtype=torch.int8, device=DEV)
    dw = torch.empty(c_out, dtype=torch.float32, device=DEV)
    ws = torch.empty(q.prepare_workspace_bytes(c_in, c_out), dtype=torch.int8, device=DEV)
    q.prepare_weight(Wd, None, Wp, dw, None, None, None, ws)
    torch.cuda.synchronize()
    assert torch.all(dw == 1.0)
    n_pad = q.padded_outliers(n)
    Xq = _small_ints(seed, 2, (t, c_in), 7)
    xo = np.zeros((t, max(n_pad, 1)), np.int64)
    wh = np.zeros((c_out, max(n_pad, 1)), np.int64)
    if n:
        xo[:, :n] = _small_ints(seed, 3, (t, n), 9)
        wh[:, :n] = _small_ints(seed, 4, (c_out, n), 9)
    # (float64 products of these small integers are exact and run on the BLAS)
    want = (Xq.astype(np.float64) @ Wi.astype(np.float64) + xo.astype(np.float64) @ wh.T.astype(np.float64))
    assert np.abs(want).max() < 2 ** 24
    ones_t = torch.ones(t, dtype=torch.float32, device=DEV)
    ones_c = torch.ones(c_out, dtype=torch.float32, device=DEV)
    Xq_d = torch.from_numpy(Xq.astype(np.int8)).to(DEV)
    xo_d = torch.from_numpy(xo.astype(np.int8)).to(DEV)
    wh_d = torch.from_numpy(wh.astype(np.int8)).to(DEV)
    for ldy in (c_out, c_out + 24):        # dense and strided output
        Ybuf = torch.full((t, ldy), float("nan"), dtype=torch.float32, device=DEV)
        Y = Ybuf[:, :c_out]
        q.linear_fwd(Xq_d, ones_t, xo_d if n else None, Wp, dw, c_in, c_out, wh_d if n else None, ones_c if n else None,
                     n, None, None, None, 0, 0.0, Y, None)
        torch.cuda.synchronize()
        got = Y.cpu().numpy().astype(np.float64)
        bad = np.argwhere(got != want)
        assert bad.size == 0, "Y != acc1 + acc2 at %s (ldy %d): %r vs %r" % (
            bad[0], ldy, got[tuple(bad[0])], want[tuple(bad[0])])
        if ldy > c_out:
            assert torch.isnan(Ybuf[:, c_out:]).all(), "the product wrote past its c_out columns"
    # ---- dX: dY holds small integers and one 127 per token row, delta_w = 1: codes = dY, step 1, dX = dY Wq^T
    G = _small_ints(seed, 5, (t, c_out), 7)
    G[:, 1] = 127
    dY_d = torch.from_numpy(synth.f32_to_bf16(G.astype(np.float32).ravel()).reshape(t, c_out).view(np.int16)).to(DEV)
    want_dx = G.astype(np.float64) @ Wi.T.astype(np.float64)
    assert np.abs(want_dx).max() < 2 ** 24
    wsb = torch.empty(q.workspace_bytes(t, c_in, c_out, 0, 0), dtype=torch.int8, device=DEV)
    dXbuf = torch.full((t, c_in + 8), float("nan"), dtype=torch.float32, device=DEV)
    dX = dXbuf[:, :c_in]
    # the second pass forces every bounded device-side wait to give up at once (a split contraction then computes
    # its partner's half itself): the kernels still finish and the result is the same
    for ticks in (None, 0):
        prev = q.debug_grid_wait_ticks(ticks) if ticks is not None else None
        try:
            dXbuf.fill_(float("nan"))
            q.linear_bwd_dx(dY_d, Wp, dw, c_in, c_out, None, None, 0, 0.0, dX, wsb)
            torch.cuda.synchronize()
        finally:
            if prev is not None:
                q.debug_grid_wait_ticks(prev)
        got = dX.cpu().numpy().astype(np.float64)
        bad = np.argwhere(got != want_dx)
        assert bad.size == 0, "dX != acc at %s (wait bound %s): %r vs %r" % (
            bad[0], ticks, got[tuple(bad[0])], want_dx[tuple(bad[0])])
        assert torch.isnan(dXbuf[:, c_in:]).all()
