"""Shared helpers for the GPU parity tests: run the HIP path through the C ABI and the CPU oracle on the same
seeded inputs and compare.  Integer results must match bit for bit; fp32 outputs within 1e-3."""
from __future__ import annotations

import numpy as np
import torch

from oracle import api as orc
from paper_2505_14742_amd import binding as q

DEV = "cuda:0"
REL_TOL = 1e-3


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype)
    return t.to(DEV)


def bf16_dev(a_u16):
    """uint16 bit patterns -> device tensor of the same bits (viewed as int16: only the bytes matter)."""
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.int16)).to(DEV)


def host(t):
    return t.cpu().numpy()


def assert_close_fp32(got, want, what):
    """|a-b| <= 1e-3 |b| + 1e-3 rms(b) for every element, and the Frobenius error <= 1e-3."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    rms = np.sqrt(np.mean(want * want)) if want.size else 0.0
    err = np.abs(got - want)
    lim = REL_TOL * np.abs(want) + REL_TOL * rms
    worst = np.max(err - lim) if err.size else 0.0
    assert worst <= 0.0, "%s: element-wise tolerance exceeded by %g (rms %g)" % (what, worst, rms)
    fro = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert fro <= REL_TOL, "%s: Frobenius error %g" % (what, fro)
    return fro


class Layer:
    """Device-side state of one quantized linear layer, driven only through the C ABI."""

    def __init__(self, W, O, A, B, lora_scale, t):
        self.c_in, self.c_out = W.shape
        self.n = int(O.size)
        self.n_pad = q.padded_outliers(self.n)
        self.r = int(A.shape[1]) if A is not None else 0
        self.lora_scale = float(lora_scale)
        self.t = t
        self.W = dev(W)
        self.O = dev(O.astype(np.int32)) if self.n else None
        self.A = bf16_dev(A) if self.r else None
        self.B = bf16_dev(B) if self.r else None
        i8, f32 = torch.int8, torch.float32
        self.Wq_packed = torch.empty(q.packed_weight_bytes(self.c_in, self.c_out), dtype=i8, device=DEV)
        self.delta_w = torch.empty(self.c_out, dtype=f32, device=DEV)
        self.W_O = torch.empty((max(self.n, 1), self.c_out), dtype=f32, device=DEV)
        self.wmax_O = torch.empty(max(self.n, 1), dtype=f32, device=DEV)
        self.Wq_plain = torch.empty((self.c_in, self.c_out), dtype=i8, device=DEV)
        ws = torch.empty(q.prepare_workspace_bytes(self.c_in, self.c_out), dtype=i8, device=DEV)
        q.prepare_weight(self.W, self.O, self.Wq_packed, self.delta_w, self.W_O if self.n else None,
                         self.wmax_O if self.n else None, self.Wq_plain, ws)
        self.s_O = torch.ones(max(self.n, 1), dtype=f32, device=DEV)
        self.colscale = torch.ones(self.c_in, dtype=f32, device=DEV)
        self.what_int = torch.full((self.c_out, max(self.n_pad, 1)), 77, dtype=i8, device=DEV)
        self.delta_what = torch.full((self.c_out,), -1.0, dtype=f32, device=DEV)
        self.cmax = torch.empty(max(self.n, 1), dtype=f32, device=DEV)
        self.alloc(t)

    def alloc(self, t):
        i8, f32 = torch.int8, torch.float32
        self.t = t
        self.ws = torch.empty(q.workspace_bytes(t, self.c_in, self.c_out, self.n, self.r), dtype=i8, device=DEV)
        self.Xq = torch.empty((t, self.c_in), dtype=i8, device=DEV)
        self.delta_x = torch.empty(t, dtype=f32, device=DEV)
        self.xq_O = torch.full((t, max(self.n_pad, 1)), 55, dtype=i8, device=DEV)
        self.Y = torch.empty((t, self.c_out), dtype=f32, device=DEV)
        self.dX = torch.empty((t, self.c_in), dtype=f32, device=DEV)

    # --- the four per-step calls
    def scale_update(self, X, gamma):
        q.scale_update(X, self.O, self.W_O, self.wmax_O, self.c_out, gamma, self.s_O, self.colscale, self.what_int,
                       self.delta_what, self.cmax, self.ws)

    def quant_act(self, X):
        q.quant_act(X, self.colscale, self.O, self.Xq, self.delta_x, self.xq_O if self.n else None)

    def linear_fwd(self, X):
        q.linear_fwd(self.Xq, self.delta_x, self.xq_O if self.n else None, self.Wq_packed, self.delta_w, self.c_in,
                     self.c_out, self.what_int if self.n else None, self.delta_what if self.n else None, self.n,
                     X if self.r else None, self.A, self.B, self.r, self.lora_scale, self.Y, self.ws)

    def fwd_step(self, X, gamma):
        """The three forward calls as one (quaff_linear_fwd_step), on a workspace of its own."""
        if not hasattr(self, "ws_step") or self.ws_step_t != self.t:
            self.ws_step = torch.empty(q.fwd_step_workspace_bytes(self.t, self.c_in, self.c_out, self.n, self.r),
                                       dtype=torch.int8, device=DEV)
            self.ws_step_t = self.t
        q.linear_fwd_step(X, self.O, self.W_O if self.n else None, self.wmax_O if self.n else None, self.c_out, gamma,
                          self.s_O, self.colscale, self.what_int, self.delta_what, self.cmax, self.Xq, self.delta_x,
                          self.xq_O if self.n else None, self.Wq_packed, self.delta_w, self.A, self.B, self.r,
                          self.lora_scale, self.Y, self.ws_step)

    def linear_fwd_acc(self):
        acc1 = torch.empty((self.t, self.c_out), dtype=torch.int32, device=DEV)
        acc2 = torch.empty((self.t, self.c_out), dtype=torch.int32, device=DEV)
        q.linear_fwd_acc(self.Xq, self.xq_O if self.n else None, self.Wq_packed, self.c_in, self.c_out,
                         self.what_int if self.n else None, self.n, acc1, acc2)
        return acc1, acc2

    def linear_bwd_dx(self, dY):
        q.linear_bwd_dx(dY, self.Wq_packed, self.delta_w, self.c_in, self.c_out, self.A, self.B, self.r,
                        self.lora_scale, self.dX, self.ws)

    def linear_bwd_dx_acc(self, dY):
        Gq = torch.empty((self.t, self.c_out), dtype=torch.int8, device=DEV)
        dg = torch.empty(self.t, dtype=torch.float32, device=DEV)
        acc = torch.empty((self.t, self.c_in), dtype=torch.int32, device=DEV)
        q.linear_bwd_dx_acc(dY, self.Wq_packed, self.delta_w, self.c_in, self.c_out, Gq, dg, acc)
        return Gq, dg, acc


class OracleLayer:
    """The same layer on the CPU oracle."""

    def __init__(self, W, O, A, B, lora_scale):
        self.W, self.O = W, O.astype(np.int32)
        self.A, self.B = (A, B) if A is not None and A.shape[1] > 0 else (None, None)
        self.lora_scale = float(lora_scale)
        self.Wq, self.dw = orc.weight_quantize(W)
        self.W_O, self.wmax = orc.outlier_rows(W, self.O)
        self.s = np.ones(self.O.size, np.float32)
        self.colscale = np.ones(W.shape[0], np.float32)

    def scale_update(self, X, gamma):
        self.s, self.colscale, self.what, self.dwh, self.cmax = orc.scale_update(
            X, self.O, self.W_O, self.wmax, gamma, self.s, self.colscale)


def sample_rows(t, every=16, block=256):
    """Deterministic row subset: every `every`-th row plus the first and last row of every `block`-row block.  An odd
    stride walks through every row position of the 32-row blocks and every swizzle slot of the LDS stages."""
    rows = set(range(0, t, every))
    for b in range(0, t, block):
        rows.add(b)
        rows.add(min(t, b + block) - 1)
    rows.add(t - 1)
    return np.array(sorted(rows), dtype=np.int64)


def check_prepare(L: Layer, R: OracleLayer):
    assert np.array_equal(host(L.delta_w), R.dw), "delta_w"
    assert np.array_equal(host(L.Wq_plain), R.Wq), "W_int"
    if L.n:
        assert np.array_equal(host(L.W_O), R.W_O) and np.array_equal(host(L.wmax_O), R.wmax), "W_O / wmax"
    # the packed copy: element (j, k) of the [c_out x c_in] codes at (j // 2) * 2 * cpad + (k // 64) * 128 + (j % 2) * 64 + k % 64
    cpad = (L.c_in + 63) // 64 * 64
    j, k = np.meshgrid(np.arange(L.c_out), np.arange(L.c_in), indexing="ij")
    off = (j // 2) * (2 * cpad) + (k // 64) * 128 + (j % 2) * 64 + (k % 64)
    assert np.array_equal(host(L.Wq_packed)[off], R.Wq.T), "packed codes"


def check_step(L: Layer, R: OracleLayer, X_u16, dY_u16, gamma, rows=None, backward=True, tag=""):
    """One full step on both sides.  rows = None compares everything; otherwise the products are compared on
    that row subset (every step of the path is row-independent except the column maximum)."""
    t = X_u16.shape[0]
    Xd = bf16_dev(X_u16)
    # ---- scale update (Eq. 7, 8; what)
    if L.n:
        L.scale_update(Xd, gamma)
        R.scale_update(X_u16, gamma)
        assert np.array_equal(host(L.cmax)[:L.n], R.cmax), tag + " cmax"
        s_gpu = host(L.s_O)[:L.n]
        np.testing.assert_allclose(s_gpu, R.s, rtol=REL_TOL, err_msg=tag + " s")
        assert np.array_equal(s_gpu, R.s), tag + " s is expected to be bit-exact (fully specified fp32 sequence)"
        assert np.array_equal(host(L.colscale), R.colscale), tag + " colscale"
        wh = host(L.what_int)
        assert np.array_equal(wh[:, :L.n], R.what.T), tag + " what_int"
        assert not wh[:, L.n:].any(), tag + " what_int padding"
        assert np.array_equal(host(L.delta_what), R.dwh), tag + " delta_what"
    else:
        L.scale_update(Xd, gamma)   # legal no-op
        R.what = np.zeros((0, L.c_out), np.int8)
        R.dwh = np.zeros(L.c_out, np.float32)
    # ---- scale + per-token quantization (Eq. 5, Eq. 1)
    L.quant_act(Xd)
    Xq_o, dx_o, xo_o = orc.quant_act(X_u16, R.colscale, R.O)
    assert np.array_equal(host(L.Xq), Xq_o), tag + " activation codes"
    assert np.array_equal(host(L.delta_x), dx_o), tag + " delta_x"
    if L.n:
        xo = host(L.xq_O)
        assert np.array_equal(xo[:, :L.n], xo_o) and not xo[:, L.n:].any(), tag + " xq_O"
    # ---- integer forward (Eq. 9) + LoRA
    sel = slice(None) if rows is None else rows
    A, B = R.A, R.B
    Y_o, a1_o, a2_o = orc.linear_fwd(Xq_o[sel], dx_o[sel], xo_o[sel], R.Wq, R.dw, R.what, R.dwh, X_u16[sel], A, B,
                                     R.lora_scale)
    acc1, acc2 = L.linear_fwd_acc()
    idx = slice(None) if rows is None else torch.from_numpy(rows).to(DEV)
    assert np.array_equal(host(acc1[idx]), a1_o), tag + " acc1"
    assert np.array_equal(host(acc2[idx]), a2_o), tag + " acc2"
    del acc1, acc2
    L.linear_fwd(Xd)
    out = {"fwd_err": assert_close_fp32(host(L.Y[idx]), Y_o, tag + " Y")}
    # ---- backward dX
    if backward:
        dYd = bf16_dev(dY_u16)
        dX_o, Gq_o, dg_o, acc_o = orc.linear_bwd_dx(dY_u16[sel], R.Wq, R.dw, A, B, R.lora_scale)
        Gq, dg, acc = L.linear_bwd_dx_acc(dYd)
        assert np.array_equal(host(Gq[idx]), Gq_o), tag + " gradient codes"
        assert np.array_equal(host(dg[idx]), dg_o), tag + " delta_g"
        assert np.array_equal(host(acc[idx]), acc_o), tag + " backward accumulators"
        del Gq, dg, acc
        L.linear_bwd_dx(dYd)
        out["bwd_err"] = assert_close_fp32(host(L.dX[idx]), dX_o, tag + " dX")
    torch.cuda.synchronize()
    return out
