// INT8 MFMA GEMM main kernel: operand tiles stream global -> LDS with direct-to-LDS loads (no register staging)
// through a ring of STAGES buffers, fragments are double-buffered in registers, and one barrier per 64-byte
// contraction step sits in the middle of the step so that the MFMAs of one half cover the LDS latency of the other.
// See quaff_gemm.hip for the computation; the epilogue is shared with the generic kernel.
#pragma once
#include "quaff_gemm_kernel.h"

namespace quaff {

#ifdef QUAFF_GEMM_TIMING
__device__ long long quaff_timing_out[64 * 8 * 4];
#endif
typedef __attribute__((address_space(3))) int8_t lds_i8;
typedef __attribute__((address_space(3))) i32x4 lds_i32x4;

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt = [3:0] and [15:14])
#define QUAFF_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

template <int BM, int BN, int WGM, int WGN, int STAGES>
struct DmaCfg {
    static constexpr int BK = 64;
    static constexpr int NW = WGM * WGN, NT = 64 * NW;    // wavefronts / threads per workgroup
    static constexpr int WM = BM / WGM, WN = BN / WGN;    // wavefront tile
    static constexpr int TM = WM / 32, TN = WN / 32;      // 32x32 MFMA blocks per wavefront tile
    static constexpr int A_BYTES = BM * BK, STAGE_BYTES = (BM + BN) * BK;
    static constexpr int NGROUP = (BM + BN) / 16;         // 16-row groups per stage, one direct load (1 KiB) each
    static constexpr int NLOAD = (NGROUP + NW - 1) / NW;  // direct loads per lane per stage
    static constexpr int STAGES_ = STAGES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static_assert(BM % 16 == 0 && BN % 16 == 0, "stages are filled in 16-row groups");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wavefront tile is made of 32x32 blocks");
    static_assert(STAGES >= 3 && (STAGES - 2) * NLOAD < 64, "ring depth / vmcnt range");
};

// Tile order.  Workgroups are dealt to the eight XCDs round-robin by the hardware and every XCD has its own L2, so
// the tile grid is cut into XM x XN = 8 rectangular regions, one per XCD: the operand panels an XCD touches are
// then as few as possible.  Returns false for surplus workgroups of a region that is smaller than the largest one.
struct TileMap {
    int tiles_m, tiles_n, xm, xn, rm, rn;   // region grid xm x xn, region size rm x rn (ceil)
};
__device__ __forceinline__ bool tile_of_block(const TileMap& t, int bid, int& tm, int& tn) {
    const int xcd = bid & 7, local = bid >> 3;
    const int rx = xcd / t.xn, ry = xcd % t.xn;
    const int lm = local / t.rn, ln = local % t.rn;
    tm = rx * t.rm + lm;
    tn = ry * t.rn + ln;
    return lm < t.rm && tm < t.tiles_m && tn < t.tiles_n;
}

// The main loop.  `dma` and `rd` both point at the LDS ring; they are separate restrict-qualified parameters so that
// the compiler does not serialise every LDS read behind all outstanding direct loads - the ordering between a
// stage's loads and its reads is enforced here with explicit vmcnt waits and barriers.
template <class C>
__device__ __forceinline__ void gemm_mainloop_dma(const int8_t* __restrict__ gA, const int8_t* __restrict__ gB,
                                                  const uint32_t (&voff)[C::NLOAD], int KT,
                                                  lds_i8* __restrict__ dma, const lds_i8* __restrict__ rd, int wave,
                                                  int a_frag_off, int b_frag_off, i32x16 (&acc)[C::TM][C::TN]) {
    constexpr int TM = C::TM, TN = C::TN, NLOAD = C::NLOAD, STAGES = C::STAGES_;

    auto issue = [&](int tile, int stage) {
#ifdef QUAFF_TILED_PROBE
        const int64_t k0 = (int64_t)tile * 1024;
#else
        const int64_t k0 = (int64_t)tile * C::BK;
#endif
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            // group q of the stage: A rows first, then B rows.  A wavefront whose last slot falls past the end repeats
            // its previous group (same bytes to the same place), so every wavefront issues NLOAD loads per stage
            int q = j * C::NW + wave;
            if (q >= C::NGROUP) q -= C::NW;
            const bool isA = q < C::A_BYTES / 1024;
            const int8_t* src = (isA ? gA : gB) + k0 + voff[j];
            lds_i8* dst = dma + stage * C::STAGE_BYTES + q * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
    };
    auto read_frags = [&](int stage, int ks, i32x4 (&fa)[TM], i32x4 (&fb)[TN]) {
        const lds_i8* base = rd + stage * C::STAGE_BYTES;
        const int x = ks * 32;   // second half of the 64-byte row: chunk index ^ 2
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const lds_i32x4*)(base + ((a_frag_off + i * 2048) ^ x));
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *(const lds_i32x4*)(base + C::A_BYTES + ((b_frag_off + j * 2048) ^ x));
    };
    auto mfmas = [&](const i32x4 (&fa)[TM], const i32x4 (&fb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };
    // issue order inside a half step: one LDS read (and at most one direct load), then a share of the MFMAs
    constexpr int MFMA_PER_READ = (TM * TN) / (TM + TN) > 0 ? (TM * TN) / (TM + TN) : 1;

#ifdef QUAFF_GEMM_TIMING
    long long quaff_timing[2] = {0, 0};
    long long tstart_ = __builtin_amdgcn_s_memtime();
    long long wstart_ = wall_clock64();
#endif
    // prologue: fill the ring (tiles beyond the last are clamped to it: harmless rewrites of a free stage)
#pragma unroll
    for (int s = 0; s < STAGES; ++s) issue(s < KT ? s : KT - 1, s);
    QUAFF_WAIT_VMCNT((STAGES - 1) * NLOAD);
    __builtin_amdgcn_s_barrier();

    i32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    read_frags(0, 0, fa0, fb0);
#ifdef QUAFF_ABL_NOLDS
    read_frags(0, 1, fa1, fb1);
#endif
    int stage = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const int next = (stage + 1 == STAGES) ? 0 : stage + 1;
        // first half: fragments of the second 32 bytes arrive while the first 32 are multiplied
#ifndef QUAFF_ABL_NOLDS
        read_frags(stage, 1, fa1, fb1);
#endif
        mfmas(fa0, fb0);
#pragma unroll
        for (int u = 0; u < TM + TN; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_READ, 0);
        }
        // every wavefront has now read all of `stage`; tile kt+1 must have landed for everybody
#ifdef QUAFF_GEMM_TIMING
        long long t0_ = __builtin_amdgcn_s_memtime();
#endif
#ifndef QUAFF_ABL_NOSYNC
        QUAFF_WAIT_VMCNT((STAGES - 2) * NLOAD);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#endif
#ifdef QUAFF_GEMM_TIMING
        long long t1_ = __builtin_amdgcn_s_memtime();
#endif
#ifndef QUAFF_ABL_NOSYNC
        __builtin_amdgcn_s_barrier();
#endif
        asm volatile("" ::: "memory");
#ifdef QUAFF_GEMM_TIMING
        long long t2_ = __builtin_amdgcn_s_memtime();
        quaff_timing[0] += t1_ - t0_;
        quaff_timing[1] += t2_ - t1_;
#endif
#ifndef QUAFF_ABL_NODMA
        {
            int t = kt + STAGES;
            issue(t < KT ? t : KT - 1, stage);
        }
#endif
#ifndef QUAFF_ABL_NOLDS
        read_frags(next, 0, fa0, fb0);
#endif
        mfmas(fa1, fb1);
#pragma unroll
        for (int u = 0; u < TM + TN; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (u < NLOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_READ, 0);
        }
        stage = next;
    }
    QUAFF_WAIT_VMCNT(0);
#ifdef QUAFF_GEMM_TIMING
    if ((threadIdx.x & 63) == 0 && blockIdx.x < 64) {
        long long tend_ = __builtin_amdgcn_s_memtime();
        long long* o = quaff_timing_out + (blockIdx.x * 8 + (threadIdx.x >> 6)) * 4;
        o[0] = quaff_timing[0]; o[1] = wall_clock64() - wstart_; o[2] = tend_ - tstart_; o[3] = KT;
    }
#endif
}

// Variant of the main loop that consumes TWO 64-byte contraction steps per barrier (ring of four stages): half as
// many workgroup barriers and counter waits per MFMA.  KT must be even.
template <class C>
__device__ __forceinline__ void gemm_mainloop_dma2(const int8_t* __restrict__ gA, const int8_t* __restrict__ gB,
                                                   const uint32_t (&voff)[C::NLOAD], int KT,
                                                   lds_i8* __restrict__ dma, const lds_i8* __restrict__ rd, int wave,
                                                   int a_frag_off, int b_frag_off, i32x16 (&acc)[C::TM][C::TN]) {
    constexpr int TM = C::TM, TN = C::TN, NLOAD = C::NLOAD;
    static_assert(C::STAGES_ == 4, "two steps per barrier need a ring of four stages");
    auto issue = [&](int tile, int stage) {
        const int64_t k0 = (int64_t)tile * C::BK;
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            int q = j * C::NW + wave;
            if (q >= C::NGROUP) q -= C::NW;
            const bool isA = q < C::A_BYTES / 1024;
            const int8_t* src = (isA ? gA : gB) + k0 + voff[j];
            lds_i8* dst = dma + stage * C::STAGE_BYTES + q * 1024;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
    };
    auto read_frags = [&](int stage, int ks, i32x4 (&fa)[TM], i32x4 (&fb)[TN]) {
        const lds_i8* base = rd + stage * C::STAGE_BYTES;
        const int x = ks * 32;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const lds_i32x4*)(base + ((a_frag_off + i * 2048) ^ x));
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = *(const lds_i32x4*)(base + C::A_BYTES + ((b_frag_off + j * 2048) ^ x));
    };
    auto mfmas = [&](const i32x4 (&fa)[TM], const i32x4 (&fb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };
    constexpr int MFMA_PER_READ = (TM * TN) / (TM + TN) > 0 ? (TM * TN) / (TM + TN) : 1;
    auto order_reads = [&](bool with_loads) {
#pragma unroll
        for (int u = 0; u < TM + TN; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (with_loads && u < 2 * NLOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_READ, 0);
        }
    };

#pragma unroll
    for (int s = 0; s < 4; ++s) issue(s < KT ? s : KT - 1, s);
    QUAFF_WAIT_VMCNT(2 * NLOAD);
    __builtin_amdgcn_s_barrier();

    i32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    read_frags(0, 0, fa0, fb0);
    int s0 = 0;                                   // stage of the first tile of the pair
    for (int kt = 0; kt < KT; kt += 2) {
        const int s1 = s0 + 1, s2 = (s0 + 2) & 3;
        read_frags(s0, 1, fa1, fb1);
        mfmas(fa0, fb0);
        order_reads(false);
        read_frags(s1, 0, fa0, fb0);
        mfmas(fa1, fb1);
        order_reads(false);
        read_frags(s1, 1, fa1, fb1);
        mfmas(fa0, fb0);
        order_reads(false);
        // both stages of the pair have been read by everyone after this barrier; the next pair must have landed
        QUAFF_WAIT_VMCNT(0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        {
            int t0 = kt + 4, t1 = kt + 5;
            issue(t0 < KT ? t0 : KT - 1, s0);
            issue(t1 < KT ? t1 : KT - 1, s1);
        }
        read_frags(s2, 0, fa0, fb0);
        mfmas(fa1, fb1);
        order_reads(true);
        s0 = s2;
    }
    QUAFF_WAIT_VMCNT(0);
}

template <int BM, int BN, int WGM, int WGN, int STAGES, bool DUMP, int MINB = 1, int PAIR = 0>
__global__ void __launch_bounds__(64 * WGM * WGN, MINB)
gemm_i8_dma_kernel(const GemmArgs g, const TileMap tmap) {
    using C = DmaCfg<BM, BN, WGM, WGN, STAGES>;
    extern __shared__ __attribute__((aligned(1024))) int8_t lds_raw[];
    lds_i8* lds = (lds_i8*)lds_raw;

    int tile_m, tile_n;
    if (!tile_of_block(tmap, blockIdx.x, tile_m, tile_n)) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

    // loader: a direct load fills 16 rows x 64 bytes of a stage (A rows first, then B rows); lane -> (row = lane / 4,
    // slot = lane % 4) and the slot holds global chunk slot ^ ((row / 4) & 3), the swizzle the fragment reads undo
    uint32_t voff[C::NLOAD];
    {
        const int r = lane >> 2, chunk = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
        for (int j = 0; j < C::NLOAD; ++j) {
            int q = j * C::NW + wave;
            if (q >= C::NGROUP) q -= C::NW;
            const bool isA = q < BM / 16;
            int local = (isA ? q : q - BM / 16) * 16 + r;
            int64_t row = (isA ? m0 : n0) + local;
            int64_t lim = (isA ? g.M : g.N) - 1;
            row = row < lim ? row : lim;                        // clamp: rows past the edge are never stored
#ifdef QUAFF_TILED_PROBE
            voff[j] = (uint32_t)((((isA ? m0 : n0) / 16 + (isA ? q : q - BM / 16)) % ((isA ? g.M : g.N) / 16)) * (g.K * 16) + lane * 16);
#else
            voff[j] = (uint32_t)(row * (isA ? g.lda : g.ldb) + chunk * 16);
#endif
        }
    }
    const int frag = l32 * 64 + ((lhi ^ ((l32 >> 2) & 3)) * 16);
    const int a_frag_off = wm * C::WM * 64 + frag, b_frag_off = wn * C::WN * 64 + frag;

    i32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    if constexpr (PAIR)
        gemm_mainloop_dma2<C>(g.A, g.B, voff, (int)(g.K / C::BK), lds, lds, wave, a_frag_off, b_frag_off, acc);
    else
        gemm_mainloop_dma<C>(g.A, g.B, voff, (int)(g.K / C::BK), lds, lds, wave, a_frag_off, b_frag_off, acc);

#ifdef QUAFF_GEMM_TIMING
    long long te0_ = __builtin_amdgcn_s_memtime();
#endif
    gemm_epilogue<C::TM, C::TN, DUMP>(g, acc, m0 + wm * C::WM, n0 + wn * C::WN, l32, lhi);
#ifdef QUAFF_GEMM_TIMING
    if ((threadIdx.x & 63) == 0 && blockIdx.x < 64) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        quaff_timing_out[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 4 + 3] = __builtin_amdgcn_s_memtime() - te0_;
    }
#endif
}

// host side: choose the XCD region grid for a tile grid
inline TileMap make_tile_map(int tiles_m, int tiles_n) {
    TileMap best{tiles_m, tiles_n, 1, 8, tiles_m, (tiles_n + 7) / 8};
    long best_cost = -1;
    const int xms[4] = {1, 2, 4, 8};
    for (int xm : xms) {
        int xn = 8 / xm;
        int rm = (tiles_m + xm - 1) / xm, rn = (tiles_n + xn - 1) / xn;
        // cost: padded work first (surplus workgroups idle), then operand panels touched per XCD
        long cost = (long)rm * rn * 1000 + rm + rn;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = TileMap{tiles_m, tiles_n, xm, xn, rm, rn}; }
    }
    return best;
}

}  // namespace quaff
