"""Seeded synthetic inputs for the Quaff quantized-linear hot path.

This module holds no arithmetic of the method itself (no quantizer, no scale
update, no matmul): it only draws numbers.  Both the CPU oracle's tests and the
HIP path's tests/bench take their inputs from here, so the two sides see the
same bytes.  Everything is derived from a counter-based generator
(SplitMix64 finaliser over seed/stream/counter), so a value depends only on
(seed, stream, index) and never on generation order, chunking or platform.

Workloads follow the model shapes the paper fine-tunes (Phi-3-mini, LLaMA-2-7B,
and a 13B-shaped long-sequence case; Sec. "Experiment", Table 5) and the value
structure it describes: a few fixed input channels carry magnitudes one to two
orders above the rest (Sec. 2.2), positions stay fixed while magnitudes drift
between steps (Fig. 2 caption, App. "static vs dynamic scale").
"""
from __future__ import annotations

import os
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 250514742
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


# ----------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------
def _mix64(z: np.ndarray) -> np.ndarray:
    """SplitMix64 output function on a uint64 array (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _key(seed: int, stream: int) -> np.uint64:
    k = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & 0xFFFFFFFFFFFFFFFF
    return _mix64(np.array([k], dtype=np.uint64))[0]


def rng_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """count raw 64-bit draws for counters start .. start+count-1."""
    ctr = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(ctr * np.uint64(0x9E3779B97F4A7C15) + _key(seed, stream))


def uniform(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    """fp64 uniforms in (0, 1): never 0, so log() is safe."""
    u = rng_u64(seed, stream, start, count)
    return ((u >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    """fp64 standard normals (Box-Muller on two independent streams)."""
    u1 = uniform(seed, 2 * stream, count, start)
    u2 = uniform(seed, 2 * stream + 1, count, start)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def student_t3(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    """Student-t with 3 degrees of freedom: Z / sqrt(chi2_3 / 3)."""
    z = normal(seed, 4 * stream, count, start)
    c = np.zeros(count, dtype=np.float64)
    for j in range(3):
        g = normal(seed, 4 * stream + 1 + j, count, start)
        c += g * g
    return z / np.sqrt(c / 3.0)


# ----------------------------------------------------------------------------
# bf16 storage helpers (storage format only; no method arithmetic)
# ----------------------------------------------------------------------------
BF16_MAX = 3.3895313892515355e38


def f32_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(h: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# workload description
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Projection:
    """One quantized linear layer of a workload."""
    config: int
    index: int            # position inside the config (feeds the seed)
    name: str
    t: int                # tokens
    c_in: int
    c_out: int
    n_outlier: int
    lora_rank: int
    lora_scale: float
    gamma: float          # momentum coefficient of Eq. 7
    steps: int
    backward: bool
    dist: str = "normal"              # "normal" | "student_t3"
    m_lo: float = 20.0                # outlier multiplier range at step 0
    m_hi: float = 100.0
    m_fixed: float | None = None      # all multipliers start here if set
    drift: str = "lognormal_reflect"  # "uniform_ratio" | "lognormal_reflect" | "lognormal_free"
    clustered_runs: int = 0           # >0: outliers sit in this many contiguous runs

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 * self.config + 10 * self.index


def _phi3(cfg, idx, name, k, n, n_out, steps, **kw):
    return Projection(cfg, idx, name, 2048, k, n, n_out, 16, 1.0, 0.2, steps, True, **kw)


CONFIGS: dict[int, list[Projection]] = {
    # small single layer, forward only, momentum coefficient 0.9, x40 outliers drifting by U(0.8,1.25)
    1: [Projection(1, 0, "single", 256, 512, 512, 8, 0, 0.0, 0.9, 10, False,
                   m_fixed=40.0, drift="uniform_ratio")],
    # Phi-3-mini attention projections
    2: [_phi3(2, 0, "qkv", 3072, 9216, 31, 4), _phi3(2, 1, "o_proj", 3072, 3072, 31, 4)],
    # Phi-3-mini MLP (down-proj input: 0.5 % of channels at x200, clustered)
    3: [_phi3(3, 0, "gate_up", 3072, 16384, 31, 50),
        _phi3(3, 1, "down", 8192, 3072, 41, 50, m_fixed=200.0, drift="lognormal_free", clustered_runs=4)],
    # LLaMA-2-7B decoder layer, seven projections, rank 64
    4: [Projection(4, i, nm, 4096, k, n, 40, 64, 1.0, 0.2, 3, True)
        for i, (nm, k, n) in enumerate([("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096),
                                        ("o", 4096, 4096), ("gate", 4096, 11008), ("up", 4096, 11008),
                                        ("down", 11008, 4096)])],
    # LLaMA-2-13B-shaped long-sequence stress, heavy-tailed activations
    5: [Projection(5, i, nm, 16384, k, n, 64, 16, 1.0, 0.2, 2, True, dist="student_t3", m_lo=50.0, m_hi=500.0)
        for i, (nm, k, n) in enumerate([("q", 5120, 5120), ("k", 5120, 5120), ("v", 5120, 5120),
                                        ("o", 5120, 5120), ("gate", 5120, 13824), ("up", 5120, 13824),
                                        ("down", 13824, 5120)])],
    # beyond the five baseline workloads: the paper's own outlier budget (Sec. "Experimental settings": up to 4 % of
    # c_in on o_proj and 10 % on down_proj) at the Phi-3-mini shapes - the correction product and the column
    # abs-max become first-order costs
    6: [_phi3(6, 0, "o_proj", 3072, 3072, 123, 2), _phi3(6, 1, "down", 8192, 3072, 819, 2)],
}


def projection(config: int, name: str) -> Projection:
    for p in CONFIGS[config]:
        if p.name == name:
            return p
    raise KeyError((config, name))


# stream ids (each draws from an independent counter space)
_S_OUTLIER_IDX, _S_MULT0, _S_DRIFT, _S_W, _S_A, _S_B, _S_X, _S_DY = 1, 2, 3, 4, 5, 6, 100, 5000


_POOL = None


def _pool():
    global _POOL
    if _POOL is None:
        from concurrent.futures import ThreadPoolExecutor
        _POOL = ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1))
    return _POOL


def _chunked(fn, seed, stream, count, start=0, chunk=1 << 20):
    """fp32 array of `count` draws of fn for counters start..start+count-1 (chunks are drawn in parallel;
    a value depends only on its counter, so the result does not depend on the chunking)."""
    out = np.empty(count, dtype=np.float32)

    def work(s):
        e = min(count, s + chunk)
        out[s:e] = fn(seed, stream, e - s, start + s)

    list(_pool().map(work, range(0, count, chunk)))
    return out


def outlier_indices(p: Projection) -> np.ndarray:
    """Sorted, unique int32 channel indices O, fixed for the whole run."""
    n, k = p.n_outlier, p.c_in
    if n == 0:
        return np.zeros(0, dtype=np.int32)
    if p.clustered_runs > 0:
        runs = p.clustered_runs
        per = -(-n // runs)
        u = uniform(p.seed, _S_OUTLIER_IDX, runs)
        seg = k // runs
        idx = []
        for r in range(runs):
            start = r * seg + int(u[r] * (seg - per))
            idx.extend(range(start, start + per))
        return np.array(sorted(idx)[:n], dtype=np.int32)
    # draw without replacement: rank the first k uniforms, take the n smallest
    u = uniform(p.seed, _S_OUTLIER_IDX, k)
    return np.sort(np.argsort(u, kind="stable")[:n]).astype(np.int32)


def outlier_multipliers(p: Projection, step: int) -> np.ndarray:
    """Per-outlier-channel magnitude multipliers m_k(step), fp64, following the config's drift rule."""
    n = p.n_outlier
    if n == 0:
        return np.zeros(0)
    if p.m_fixed is not None:
        m = np.full(n, float(p.m_fixed))
    else:
        u = uniform(p.seed, _S_MULT0, n)
        m = np.exp(np.log(p.m_lo) + u * (np.log(p.m_hi) - np.log(p.m_lo)))
    for s in range(step):
        if p.drift == "uniform_ratio":
            m = m * (0.8 + 0.45 * uniform(p.seed, _S_DRIFT, n, s * n))
        else:
            lm = np.log(m) + 0.1 * normal(p.seed, _S_DRIFT, n, s * n)
            if p.drift == "lognormal_reflect":
                lo, hi = np.log(p.m_lo), np.log(p.m_hi)
                lm = np.where(lm > hi, 2 * hi - lm, lm)
                lm = np.where(lm < lo, 2 * lo - lm, lm)
            m = np.exp(lm)
    return m


def weight(p: Projection) -> np.ndarray:
    """Frozen full-precision weight W [c_in x c_out] fp32, N(0, 0.02^2)."""
    w = _chunked(normal, p.seed, _S_W, p.c_in * p.c_out)
    w *= np.float32(0.02)
    return w.reshape(p.c_in, p.c_out)


def lora(p: Projection):
    """LoRA factors as bf16 bit patterns: A [c_in x r] ~ N(0, 1/c_in), B [r x c_out] ~ N(0, 0.02^2) (non-zero B)."""
    r = p.lora_rank
    if r == 0:
        return np.zeros((p.c_in, 0), np.uint16), np.zeros((0, p.c_out), np.uint16)
    a = normal(p.seed, _S_A, p.c_in * r) / np.sqrt(p.c_in)
    b = normal(p.seed, _S_B, r * p.c_out) * 0.02
    return (f32_to_bf16(a.astype(np.float32)).reshape(p.c_in, r),
            f32_to_bf16(b.astype(np.float32)).reshape(r, p.c_out))


def activations(p: Projection, step: int, rows: slice | None = None) -> np.ndarray:
    """X [t x c_in] bf16 bit patterns for one step: base noise with the outlier columns multiplied by m_k(step)."""
    fn = student_t3 if p.dist == "student_t3" else normal
    r0, r1 = (0, p.t) if rows is None else (rows.start, rows.stop)
    base = p.c_in * p.t * step + r0 * p.c_in
    x = _chunked(fn, p.seed, _S_X, (r1 - r0) * p.c_in, base).reshape(r1 - r0, p.c_in)
    o = outlier_indices(p)
    if o.size:
        x[:, o] *= outlier_multipliers(p, step).astype(np.float32)[None, :]
    np.clip(x, -BF16_MAX, BF16_MAX, out=x)
    return f32_to_bf16(x).reshape(r1 - r0, p.c_in)


def out_grad(p: Projection, step: int) -> np.ndarray:
    """dY [t x c_out] bf16 bit patterns, N(0,1) * 2^-6."""
    g = _chunked(normal, p.seed, _S_DY + step, p.t * p.c_out)
    g *= np.float32(2.0 ** -6)
    return f32_to_bf16(g).reshape(p.t, p.c_out)


@dataclass
class EdgeCase:
    """Hand-shaped parity case beyond the five workloads."""
    name: str
    t: int
    c_in: int
    c_out: int
    outliers: list = field(default_factory=list)
    lora_rank: int = 0
    zero_rows: list = field(default_factory=list)
    max_in_outlier_rows: list = field(default_factory=list)
    seed: int = BASE_SEED + 99000


EDGE_CASES = [
    EdgeCase("first_last_channel", 67, 256, 128, [0, 255], 16),
    EdgeCase("adjacent", 130, 512, 256, [7, 8, 9, 10, 300, 301], 16),
    EdgeCase("no_outliers", 96, 256, 192, [], 16),
    EdgeCase("one_outlier", 33, 128, 64, [77], 0),
    EdgeCase("n65_not_multiple_of_64", 200, 1024, 320, list(range(3, 1024, 16))[:65], 32),
    EdgeCase("zero_row_and_outlier_max", 259, 384, 272, [5, 100, 383], 16, zero_rows=[0, 17, 258],
             max_in_outlier_rows=[1, 2]),
    EdgeCase("ragged_rows", 2048 + 3, 512, 528, [1, 2, 3, 500], 16),
    EdgeCase("single_row", 1, 256, 256, [9], 16),
    EdgeCase("channels_not_multiples_of_64", 70, 208, 144, [0, 100, 207], 16),
    EdgeCase("ragged_in_channels_fast_gradient_product", 300, 208, 256, [3, 100], 16),
    # shapes that reach every output-tile shape of the GEMM with short contractions (cheap on the CPU), crossed
    # with outlier counts of one to four 64-wide slices and LoRA ranks of one or two 32-column slices
    EdgeCase("wide_out_n65_r64", 2048, 256, 9216, list(range(1, 256, 3))[:65], 64),
    EdgeCase("wide_out_odd_steps_r48", 2048, 192, 9216, [0, 50, 100, 150, 191], 48),
    EdgeCase("very_wide_out_n70_r32", 1024, 256, 16384, list(range(2, 256, 3))[:70], 32),
    EdgeCase("mid_out_n200_r16", 2048, 256, 4096, list(range(0, 250))[:200], 16),
    EdgeCase("mid_out_n130_r64", 2048, 256, 4096, list(range(0, 256, 1))[60:190], 64),
    EdgeCase("mid_in_short_contraction", 2048, 4096, 128, [5, 4000], 16),     # input-gradient product on the 256x128 tile
    # 2048 x 3072 outputs (the 128x192 tile) with more than two outlier slices: the correction product is a launch of
    # its own and the main product accumulates onto it in the one-pass epilogue; the second case also has an edge tile
    EdgeCase("o_shape_n200_accumulate", 2048, 256, 3072, list(range(0, 250))[:200], 16),
    EdgeCase("o_shape_ragged_n140_accumulate", 2000, 256, 3056, list(range(10, 150)), 32),
    # long inputs (at least 256 row blocks of 16) at rank 16: the persistent down-projection with the abs-max inside;
    # outliers at both ends, on both sides of the boundary between the two contraction parts (576 | 2112) and next to
    # each other inside one lane's eight columns; ragged rows
    EdgeCase("long_rows_short_slices", 4099, 1040, 64, [0, 1, 7, 8, 519, 575, 576, 1039], 16),
    EdgeCase("long_rows_six_steps", 4112, 4208, 64, [0, 63, 64, 2111, 2112, 2113, 3000, 3001, 3002, 3003, 4207], 16,
             zero_rows=[0, 4111]),
]


def edge_case_inputs(ec: EdgeCase, idx: int):
    """X, dY (bf16 bits), W (fp32), O, A, B for an edge case."""
    seed = ec.seed + 10 * idx
    x = _chunked(normal, seed, _S_X, ec.t * ec.c_in).reshape(ec.t, ec.c_in)
    o = np.array(sorted(ec.outliers), dtype=np.int32)
    if o.size:
        x[:, o] *= np.float32(50.0)
    for r in ec.max_in_outlier_rows:
        x[r, o[0]] = np.float32(4096.0)
    for r in ec.zero_rows:
        x[r, :] = 0.0
    w = (_chunked(normal, seed, _S_W, ec.c_in * ec.c_out) * np.float32(0.02)).reshape(ec.c_in, ec.c_out)
    dy = (_chunked(normal, seed, _S_DY, ec.t * ec.c_out) * np.float32(2.0 ** -6)).reshape(ec.t, ec.c_out)
    for r in ec.zero_rows:
        dy[r, :] = 0.0
    r_ = ec.lora_rank
    a = (normal(seed, _S_A, ec.c_in * r_) / np.sqrt(ec.c_in)).astype(np.float32).reshape(ec.c_in, r_)
    b = (normal(seed, _S_B, r_ * ec.c_out) * 0.02).astype(np.float32).reshape(r_, ec.c_out)
    return f32_to_bf16(x).reshape(x.shape), f32_to_bf16(dy).reshape(dy.shape), w, o, \
        f32_to_bf16(a).reshape(a.shape), f32_to_bf16(b).reshape(b.shape)
