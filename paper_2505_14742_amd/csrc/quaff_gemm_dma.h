// INT8 MFMA GEMM main kernel: operand tiles stream global -> LDS with direct-to-LDS loads (no register staging)
// through a ring of buffers and fragments are double-buffered in registers.  Two main loops: 64-byte stages (one
// barrier per 64-byte contraction step, in the middle of the step so that the MFMAs of one half cover the LDS latency
// of the other) and, for contractions that are a multiple of 128, wide stages of 128 contraction bytes per row (one
// barrier per two steps, whole cache lines per direct load); the wide loop also reads the B operand as [K x N] from
// the packed weight codes for the input-gradient product.  The epilogue stages its operands through the idle ring.
// See quaff_gemm.hip for the computation.
#pragma once
#include "quaff_gemm_kernel.h"
#include <type_traits>


namespace quaff {

typedef __attribute__((address_space(3))) int8_t lds_i8;
typedef __attribute__((address_space(3))) i32x4 lds_i32x4;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;
typedef __attribute__((address_space(3))) float lds_f32;

// One direct-to-LDS load: 64 lanes x 16 bytes from per-lane global addresses to the 1 KiB of LDS that starts at `dst`
// (the same for all lanes).  Issued as inline assembly on purpose: behind the compiler's own builtin every later wait
// for an LDS read becomes a wait for ALL outstanding LDS reads (its counter model treats the load as a flat access that
// may return out of order), which stalls a wavefront for a full LDS latency at the top of every contraction sub-step;
// behind this form the waits are exact (lgkmcnt(2..6)).  The loads' own completion is tracked by hand anyway
// (QUAFF_WAIT_VMCNT + barrier).  M0 holds the LDS address; the compiler keeps nothing in M0 across statements here.
// ASM = false keeps the builtin: with exact waits the tile with one wavefront per SIMD is 2-6 % slower, the tiles that
// issue their MFMAs first (their reads have landed by the time of the wait anyway) are unchanged, and the 8-wavefront
// 256x128 tile is 3-6 % faster (all measured).
// (M0 is named as clobbered although the compiler calls it reserved: a kernel that takes this form issues every
// direct load this way, so nothing of the compiler's lives in M0.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
template <bool ASM>
__device__ __forceinline__ void dma_load_16(const void* src, __attribute__((address_space(3))) int8_t* dst) {
    if constexpr (ASM) {
        const uint32_t d = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst);
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(d) : "memory", "m0");
    } else {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    }
}
// 64 lanes x 4 bytes to the 256 bytes of LDS that start at `dst`
template <bool ASM>
__device__ __forceinline__ void dma_load_4(const void* src, __attribute__((address_space(3))) int8_t* dst) {
    if constexpr (ASM) {
        const uint32_t d = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst);
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(src), "s"(d) : "memory", "m0");
    } else {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                         (__attribute__((address_space(3))) void*)dst, 4, 0, 0);
    }
}
#pragma clang diagnostic pop

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt = [3:0] and [15:14])
#define QUAFF_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))

// B operand read as [K x N] from the packed weight codes (N = c_in contiguous within a 16-byte chunk) instead of
// contraction-contiguous.  A stage then holds 128 contraction rows x BN columns, and the MFMA fragment (16
// contraction bytes of one column per lane) is gathered with the transposing LDS read ds_read_b64_tr_b8: in every
// group of 16 lanes, lane i receives byte (i & 7) of the 8-byte pieces addressed by lanes 2 j + (i >> 3), j = 0..7.
// Lane 2 j + p of a group therefore addresses contraction row j, column piece p, and two such reads give a lane its
// 16 contraction bytes.  A read touches 8 rows x 32 bytes; the layouts below put these in different banks.
//   BN a multiple of 64: column-group major, [BN / 64][128 rows][64 bytes].  A direct load (1 KiB) then fills 16 rows
//     of one 64-column group, which are 8 whole 128-byte lines of the packed codes.  The two 32-byte halves of a row
//     swap places in rows 4..7 of every 8.
//   otherwise (288): row major, [128 rows][BN bytes], no swizzle needed (288 = 32 mod 256).
template <int BN>
struct BtStage {
    static constexpr bool GROUPED = BN % 64 == 0;
    static constexpr int ROW_STRIDE = GROUPED ? 64 : BN;
    static_assert(GROUPED || BN % 256 == 32, "row-major stage rows must rotate through the banks by themselves");
    // which (contraction row, first column) the 16-byte LDS slot number `slot` of the stage's B part holds
    __device__ static __forceinline__ void slot_source(int slot, int& krow, int& col) {
        if (GROUPED) {
            const int cg = slot >> 9, ch = slot & 3;
            krow = (slot >> 2) & 127;
            col = cg * 64 + (((ch >> 1) ^ ((krow >> 2) & 1)) * 32) + (ch & 1) * 16;
        } else {
            krow = slot / (BN / 16);
            col = (slot % (BN / 16)) * 16;
        }
    }
    // byte offset, inside the B part, of the 8-byte piece a lane addresses for the 32-column block number c32:
    // lane = 16 grp + 2 jj + piece; contraction row (grp >> 1) * 16 + jj of the 32-row sub-step, + 8 for the second read
    __device__ static __forceinline__ int piece_offset(int lane, int c32) {
        const int grp = lane >> 4, jj = (lane & 15) >> 1, piece = lane & 1;
        const int krow = (grp >> 1) * 16 + jj, in32 = (grp & 1) * 16 + piece * 8;
        if (GROUPED) return (c32 >> 1) * 8192 + krow * 64 + (((c32 & 1) ^ ((jj >> 2) & 1)) * 32) + in32;
        return krow * BN + c32 * 32 + in32;
    }
};

template <int BM, int BN, int WGM, int WGN, int STAGES>
struct DmaCfg {
    static constexpr int BK = 64, BM_ = BM, BN_ = BN;
    static constexpr int NW = WGM * WGN, NT = 64 * NW;    // wavefronts / threads per workgroup
    static constexpr int WM = BM / WGM, WN = BN / WGN;    // wavefront tile
    static constexpr int TM = WM / 32, TN = WN / 32;      // 32x32 MFMA blocks per wavefront tile
    static constexpr int A_BYTES = BM * BK, STAGE_BYTES = (BM + BN) * BK;
    static constexpr int NGROUP = (BM + BN) / 16;         // 16-row groups per stage, one direct load (1 KiB) each
    static constexpr int NLOAD = (NGROUP + NW - 1) / NW;  // direct loads per lane per stage
    static constexpr int STAGES_ = STAGES;
    static constexpr bool WAVE_SCALAR = NW >= 8 && TM * TN <= 6;
    // Issue order inside a 32-byte contraction sub-step of the wide-stage loop.  Where two or three wavefronts share
    // a SIMD, the MFMAs go first and the LDS reads of the next sub-step follow the first half of them, so that the
    // wait at the top of the next sub-step finds every read landed (-1..-8 % measured).  With one wavefront per SIMD
    // (or only four MFMAs per sub-step) reads and MFMAs alternate one by one instead (bunching the reads, in any of
    // three patterns tried, costs 5-15 % there; that tile is bound by the delivery of its operands into LDS, about
    // 53 bytes per clock and compute unit at the full MFMA rate against about 40 that the direct-load path sustains,
    // not by LDS reads).
    static constexpr bool MFMA_FIRST = NW >= 8 && TM * TN >= 6;
    static constexpr bool DMA_ASM = NW >= 8 && !MFMA_FIRST;      // see dma_load_16: only the 256x128 tile gains (3-6 %)
    // wide-stage variant (gemm_mainloop_dma128): 128 contraction bytes per row, one direct load fills 8 rows
    static constexpr int WSTAGE_BYTES = (BM + BN) * 128, A_WBYTES = BM * 128;
    static constexpr int NGROUP_W = (BM + BN) / 8, NLOAD_W = (NGROUP_W + NW - 1) / NW;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    // epilogue staging (gemm_epilogue_staged): one 64-byte-per-row plane per int8 / bf16 operand below EPI_LIMIT,
    // the fp32 row and column scales in the last SCALE_BYTES of the allocation
    static constexpr int K2_PLANES_BYTES = (BM + BN) * 64;                    // A2 and B2, 64 contraction bytes
    static constexpr int LORA_PLANES_BYTES = (2 * kLoraParts * BM + BN) * 64; // T hi/lo of every part and L, 32 columns
    static constexpr int BN_PAD = (BN + 63) / 64 * 64;
    static constexpr int SCALE_BYTES = ((BM + 2 * BN_PAD) * 4 + 1023) / 1024 * 1024;
    static constexpr int LDS_ALLOC = LDS_BYTES >= LORA_PLANES_BYTES + SCALE_BYTES ? LDS_BYTES : LORA_PLANES_BYTES + SCALE_BYTES;
    static constexpr int EPI_LIMIT = LDS_ALLOC - SCALE_BYTES;
    static_assert(BM % 64 == 0, "row scales are staged 64 at a time");
};

// Tile order.  Workgroups are dealt to the eight XCDs round-robin by the hardware and every XCD has its own L2, so
// the tile grid is cut into XM x XN = 8 rectangular regions, one per XCD: the operand panels an XCD touches are
// then as few as possible.  The launch grid is (8 GM, rn, ceil(rm / GM)): workgroups are numbered x fastest, so
// blockIdx.x % 8 is the XCD, and an XCD receives its tiles in the order: GM consecutive tile rows of tile column 0,
// the same rows of column 1, ... - no integer division in the kernel.  The 32 (or 64) tiles an XCD works on at the same
// time are then a block of GM rows by a few columns instead of a strip of one row: with more tiles than compute
// units the operand panels of the concurrent tiles are what the 4 MB L2 has to hold while the contraction advances
// (a 16384 x 13824 x 5120 product fetched 4.6 GB past its L2s with GM = 1: every tile row swept all 35 MB of its
// XCD's B region).  Returns false for surplus workgroups (a region smaller than the largest one, rows past rm).
struct TileMap {
    int tiles_m, tiles_n, xm, xn, rm, rn;   // region grid xm x xn (powers of two), region size rm x rn (ceil)
    int xn_log2;
    int gm;                                 // tile rows per group (power of two)
};
__device__ __forceinline__ bool tile_of_block(const TileMap& t, int bx, int by, int bz, int& tm, int& tn) {
    const int xcd = bx & 7, lm = bz * t.gm + (bx >> 3), ln = by;
    const int rx = xcd >> t.xn_log2, ry = xcd & (t.xn - 1);
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
                                                  int a_frag_off, int b_frag_off, int b_step,
                                                  i32x16 (&acc)[C::TM][C::TN]) {
    constexpr int TM = C::TM, TN = C::TN, NLOAD = C::NLOAD, STAGES = C::STAGES_;

    auto issue = [&](int tile, int stage) {
        const int64_t k0 = (int64_t)tile * C::BK, kb = (int64_t)tile * b_step;   // b_step: bytes of B per stage
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            // group q of the stage: A rows first, then B rows.  A wavefront whose last slot falls past the end repeats
            // its previous group (same bytes to the same place), so every wavefront issues NLOAD loads per stage
            int q = j * C::NW + wave;
            if (q >= C::NGROUP) q -= C::NW;
            const bool isA = q < C::A_BYTES / 1024;
            const int8_t* src = (isA ? gA + k0 : gB + kb) + voff[j];
            lds_i8* dst = dma + stage * C::STAGE_BYTES + q * 1024;
            dma_load_16<C::DMA_ASM>(src, dst);
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

    // prologue: fill the ring (tiles beyond the last are clamped to it: harmless rewrites of a free stage)
#pragma unroll
    for (int s = 0; s < STAGES; ++s) issue(s < KT ? s : KT - 1, s);
    QUAFF_WAIT_VMCNT((STAGES - 1) * NLOAD);
    __builtin_amdgcn_s_barrier();

    i32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    read_frags(0, 0, fa0, fb0);
    int stage = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const int next = (stage + 1 == STAGES) ? 0 : stage + 1;
        // first half: fragments of the second 32 bytes arrive while the first 32 are multiplied
        read_frags(stage, 1, fa1, fb1);
        mfmas(fa0, fb0);
#pragma unroll
        for (int u = 0; u < TM + TN; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_READ, 0);
        }
        // every wavefront has now read all of `stage`; tile kt+1 must have landed for everybody
        QUAFF_WAIT_VMCNT((STAGES - 2) * NLOAD);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        {
            int t = kt + STAGES;
            issue(t < KT ? t : KT - 1, stage);
        }
        read_frags(next, 0, fa0, fb0);
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
}

// Wide-stage variant: the ring holds two stages of 128 contraction bytes per row (the same LDS as four 64-byte stages),
// so that a direct load fetches 128-byte row segments - whole cache lines - instead of 64-byte ones, and one barrier
// serves two 64-byte contraction steps.  Row r of a stage is 128 bytes, its 16-byte chunk c sits in slot
// c ^ ((r >> 1) & 7): fragment reads (32 rows x one chunk per half wavefront) are then bank-conflict free.
// K must be a multiple of 128.
// BT: B is read as [K x N] from the packed weight codes (see BtStage); b_off[j] is then this lane's byte offset of the
// 8-byte piece it addresses for column block j in the first 32-row sub-step of a stage.
template <class C, bool BT = false>
__device__ __forceinline__ void gemm_mainloop_dma128(const int8_t* __restrict__ gA, const int8_t* __restrict__ gB,
                                                     const uint32_t (&voff)[C::NLOAD_W], int KT,
                                                     lds_i8* __restrict__ dma, const lds_i8* __restrict__ rd, int wave,
                                                     int a_frag_off, const int (&b_off)[C::TN], int64_t b_step,
                                                     i32x16 (&acc)[C::TM][C::TN]) {
    constexpr int TM = C::TM, TN = C::TN, NLOAD = C::NLOAD_W;   // b_step: bytes between consecutive stages of B
    auto issue = [&](int tile, int stage) {
        const int8_t* const pa = gA + (int64_t)tile * 128;
        const int8_t* const pb = gB + tile * b_step;
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            int q = j * C::NW + wave;
            if (q >= C::NGROUP_W) q -= C::NW;
            const bool isA = q < C::BM_ / 8;
            const int8_t* src = (isA ? pa : pb) + voff[j];
            lds_i8* dst = dma + stage * C::WSTAGE_BYTES + q * 1024;
            dma_load_16<C::DMA_ASM>(src, dst);
        }
    };
    auto read_frags = [&](int stage, int ks, i32x4 (&fa)[TM], i32x4 (&fb)[TN]) {
        const lds_i8* base = rd + stage * C::WSTAGE_BYTES;
        const int x = ks * 32;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *(const lds_i32x4*)(base + ((a_frag_off + i * 4096) ^ x));
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (BT) {
                constexpr int RS = BtStage<C::BN_>::ROW_STRIDE;
                const lds_i8* pb = base + C::A_WBYTES + b_off[j] + ks * 32 * RS;
                const i32x2 lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)pb);
                const i32x2 hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)(pb + 8 * RS));
                fb[j] = (i32x4){lo[0], lo[1], hi[0], hi[1]};
            } else {
                fb[j] = *(const lds_i32x4*)(base + C::A_WBYTES + ((b_off[0] + j * 4096) ^ x));
            }
        }
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
        if constexpr (C::MFMA_FIRST) {
        // MFMA first: the reads of the next sub-step go out behind the first MFMAs and none is issued near the end,
        // so the wait at the top of the next sub-step finds them landed.  Direct loads follow the reads.
        constexpr int R = BT ? TM + 2 * TN : TM + TN, MF = TM * TN, U = MF / 2 > 0 ? MF / 2 : 1, V = MF - U;
#pragma unroll
        for (int u = 0; u < MF; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (u < U) {
                const int cnt = R * (u + 1) / U - R * u / U;
                if (cnt == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                else if (cnt == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                else if (cnt == 3) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
                else if (cnt == 4) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            } else if (with_loads) {
                const int v = u - U, cl = NLOAD * (v + 1) / V - NLOAD * v / V;
                if (cl == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                else if (cl == 2) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
                else if (cl == 3) __builtin_amdgcn_sched_group_barrier(0x020, 3, 0);
                else if (cl == 4) __builtin_amdgcn_sched_group_barrier(0x020, 4, 0);
                else if (cl >= 5) __builtin_amdgcn_sched_group_barrier(0x020, 5, 0);
            }
        }
        return;
        }
#pragma unroll
        for (int u = 0; u < TM + TN; ++u) {
            if (BT && u >= TM) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // a B fragment is two reads
            else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            if (with_loads && u < NLOAD) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, MFMA_PER_READ, 0);
        }
    };
    constexpr int NS = C::STAGES_ / 2;            // wide stages in the ring
    static_assert(NS >= 2 && (NS - 1) * NLOAD < 64, "ring depth / vmcnt range");
#pragma unroll
    for (int s = 0; s < NS; ++s) issue(s < KT ? s : KT - 1, s);
    QUAFF_WAIT_VMCNT((NS - 1) * NLOAD);
    __builtin_amdgcn_s_barrier();

    i32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    read_frags(0, 0, fa0, fb0);
    int s = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const int next = s + 1 == NS ? 0 : s + 1;
        read_frags(s, 1, fa1, fb1);
        mfmas(fa0, fb0);
        order_reads(false);
        read_frags(s, 2, fa0, fb0);
        mfmas(fa1, fb1);
        order_reads(false);
        read_frags(s, 3, fa1, fb1);
        mfmas(fa0, fb0);
        order_reads(false);
        // this stage has been read by everyone after the barrier; the next one must have landed
        QUAFF_WAIT_VMCNT((NS - 2) * NLOAD);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // (the compiler orders every LDS read of a region after the direct loads that precede it in the source)
        if constexpr (C::MFMA_FIRST) read_frags(next, 0, fa0, fb0);
        {
            int t = kt + NS;
            issue(t < KT ? t : KT - 1, s);
        }
        if constexpr (!C::MFMA_FIRST) read_frags(next, 0, fa0, fb0);
        mfmas(fa1, fb1);
        order_reads(true);
        s = next;
    }
    QUAFF_WAIT_VMCNT(0);
}

// Epilogue of the fast kernel.  The operands of the short second product (A2, B2) and of the low-rank term (T, L)
// are first copied into the now idle LDS ring with direct loads - one memory round trip for the whole workgroup
// instead of one per 32x32 block - in the same 64-byte-row, XOR-swizzled layout as the main loop's stages.
// A whole tile whose staged operands all fit at once (r <= 32) is then finished block by block: acc2 = A2 B2^T
// (int32, exact), the block becomes  row_scale * (acc * cs + acc2 * cs2)  in fp32, the low-rank products are added
// and the block is stored while the next one computes (the epilogue is bound by instruction issue: about five vector
// instructions and a store per output element).  Edge tiles, r > 32 and operand sets that have to take turns in LDS
// run the same steps as three phases over all blocks:
//   phase A  acc2 and the conversion, per block
//   phase B  the low-rank products accumulate onto the fp32 blocks, 32 columns of r per staging round
//   phase C  stores (all loads precede all stores: they share one in-order counter)
// ACCUM adds what C already holds.  The caller guarantees (K2 / 64) * K2_PLANES_BYTES <= EPI_LIMIT.
template <class C, bool ACCUM, bool OUT16 = false>
__device__ __forceinline__ void gemm_epilogue_staged(const GemmArgs& g, i32x16 (&acc)[C::TM][C::TN],
                                                     lds_i8* __restrict__ dma, const lds_i8* __restrict__ rd,
                                                     int64_t m0, int64_t n0, int wm, int wn, int wave, int lane,
                                                     bool active = true) {
    // active = false (wavefront-uniform): this wavefront takes part in the staging loads and the barriers but has no
    // block of its own to finish (split contraction: the partner workgroup finishes it)
    constexpr int TM = C::TM, TN = C::TN, BM = C::BM_, BN = C::BN_;
    constexpr int PLANE_A = BM * 64;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int nk = g.K2 / 64, nl = (g.r + 31) / 32;
    const int k2_bytes = nk * C::K2_PLANES_BYTES;
    const bool overlap = k2_bytes + C::LORA_PLANES_BYTES <= C::EPI_LIMIT;   // both operand sets fit side by side
    const int lora_off = overlap ? k2_bytes : 0;
    const int64_t row0 = m0 + wm * C::WM, col0 = n0 + wn * C::WN;

    // loader: as in the main loop, one direct load fills 16 rows x 64 bytes; lane -> (row, swizzled 16-byte chunk).
    // A source plane is `nrows` rows, `stride` bytes apart, from the tile's first row (`first`, the same for every
    // lane: the address is a scalar base plus a 32-bit lane offset); rows past the edge of the matrix repeat the last
    // valid one (`last`: never stored).
    const int ld_r = lane >> 2, ld_chunk = (lane & 3) ^ ((lane >> 4) & 3);
    const int last_a = (int)((g.M - 1 - m0) < (int64_t)(BM - 1) ? (g.M - 1 - m0) : (int64_t)(BM - 1));
    const int last_b = (int)((g.N - 1 - n0) < (int64_t)(BN - 1) ? (g.N - 1 - n0) : (int64_t)(BN - 1));
    auto fill = [&](int lds_off, int nrows, const void* first, int last, uint32_t stride, uint32_t col_byte) {
        for (int q = wave; q < nrows / 16; q += C::NW) {
            const int local = q * 16 + ld_r;
            const uint32_t off = (uint32_t)(local < last ? local : last) * stride + col_byte;
            dma_load_16<C::DMA_ASM>(static_cast<const char*>(first) + off, dma + lds_off + q * 1024);
        }
    };
    auto issue_k2 = [&]() {
        for (int kk = 0; kk < nk; ++kk) {
            const int off = kk * C::K2_PLANES_BYTES;
            const uint32_t kb = (uint32_t)(kk * 64 + ld_chunk * 16);
            fill(off, BM, g.A2 + m0 * g.K2, last_a, (uint32_t)g.K2, kb);
            fill(off + PLANE_A, BN, g.B2 + n0 * g.K2, last_b, (uint32_t)g.K2, kb);
        }
    };
    auto issue_lora = [&](int lc) {
        // columns [32 lc, 32 lc + 32) of r; a chunk past r repeats chunk 0 (it is never multiplied)
        const uint32_t pc = (uint32_t)(lc * 32 + (lc * 32 + ld_chunk * 8 < g.r ? ld_chunk * 8 : 0)) * 2;
        const uint32_t rb = (uint32_t)g.r * 2;
#pragma unroll
        for (int part = 0; part < kLoraParts; ++part) {
            const int64_t po = ((int64_t)part * g.M + m0) * g.r;
            fill(lora_off + (2 * part) * PLANE_A, BM, g.T_hi + po, last_a, rb, pc);
            fill(lora_off + (2 * part + 1) * PLANE_A, BM, g.T_lo + po, last_a, rb, pc);
        }
        fill(lora_off + 2 * kLoraParts * PLANE_A, BN, g.L + n0 * g.r, last_b, rb, pc);
    };
    auto landed = [&]() {
        QUAFF_WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // fragment of the 32-row block that starts at plane row `base` (a multiple of 32): this lane's row, chunk c
    auto frag = [&](int plane_off, int base, int c) {
        return *(const lds_i32x4*)(rd + plane_off + (base + l32) * 64 + ((c ^ ((l32 >> 2) & 3)) * 16));
    };

    // every wavefront has finished its main-loop reads and its own direct loads before the ring is reused
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue_k2();
    if (overlap && nl > 0) issue_lora(0);

    // scales: 64 floats per direct load into the planes rs [BM], cs [BN_PAD], cs2 [BN_PAD]
    {
        constexpr int NA = BM / 64, NB = C::BN_PAD / 64;
        for (int q = wave; q < NA + 2 * NB; q += C::NW) {
            const float* first;
            int local, last;
            if (q < NA) {
                first = g.row_scale + m0;
                local = q * 64 + lane;
                last = last_a;
            } else {
                const float* base = q - NA < NB ? g.col_scale : g.col_scale2;
                if (base == nullptr) continue;
                first = base + n0;
                local = (q - NA < NB ? q - NA : q - NA - NB) * 64 + lane;
                last = last_b;
            }
            dma_load_4<C::DMA_ASM>(reinterpret_cast<const char*>(first) + (uint32_t)(local < last ? local : last) * 4,
                                   dma + C::EPI_LIMIT + q * 256);
        }
    }
    const lds_i8* rs_plane = rd + C::EPI_LIMIT;
    const lds_i8* cs_plane = rs_plane + BM * 4;
    const lds_i8* cs2_plane = cs_plane + C::BN_PAD * 4;
    const bool has_cs = g.col_scale != nullptr, has_cs2 = nk > 0;
    landed();

    // fp32 store of one 32x32 block (this lane: 16 rows of one column).  The block's first element is the same for
    // every lane, so the row offsets are scalar: a stored row costs one 64-bit add of a scalar to the lane's address
    // instead of a multiply-add chain per row and lane.
    const uint32_t store_voff = (uint32_t)(((int64_t)lhi * 4 * g.ldc + l32) * 4);   // ldc < 2^27, checked by the caller
    typedef __attribute__((address_space(1))) char gchar;
    typedef __attribute__((address_space(1))) float gfloat;
    auto block_base = [&](int i, int j) {
        const uint64_t first = reinterpret_cast<uint64_t>(g.C + (row0 + i * 32) * g.ldc + col0 + j * 32);
        return (gchar*)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(first >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)first));
    };
    auto store_block_full = [&](int i, int j, const i32x16& bits) {
        gchar* base = block_base(i, j);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            gfloat* dst = (gfloat*)(base + (int64_t)((v >> 2) * 8 + (v & 3)) * g.ldc * 4 + store_voff);
            // a relaxed system-scope atomic store is a plain store with write-through cache policy: the output
            // streams to memory while the epilogue runs instead of staying behind as dirty L2 lines that the end
            // of the kernel has to write back (measured: 1-2 us less per launch)
            __hip_atomic_store(dst, __int_as_float(bits[v]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    };
    auto store_block = [&](int i, int j, const i32x16& bits) {
        const int64_t ib = row0 + i * 32, jb = col0 + j * 32;
        if (ib + 32 <= g.M && jb + 32 <= g.N) {
            store_block_full(i, j, bits);
        } else {
            gchar* base = block_base(i, j);
            const int64_t col = jb + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int64_t row = ib + (v >> 2) * 8 + lhi * 4 + (v & 3);
                if (row < g.M && col < g.N)
                    *(gfloat*)(base + (int64_t)((v >> 2) * 8 + (v & 3)) * g.ldc * 4 + store_voff) = __int_as_float(bits[v]);
            }
        }
    };

    // ---- bf16 form of the last phase (a lambda, so that each path above ends in its own copy of it)
    // two fp32 blocks values of neighbouring columns -> one word of two bf16 (RNE): lanes 2q and 2q + 1 swap half of
    // their 16 rows; word p of a lane is row (v >> 2) * 8 + lhi * 4 + (v & 3), v = 2p + (lane & 1), columns 2q, 2q + 1
    auto pack16 = [&](const i32x16& bits, int p) -> uint32_t {
        const bool odd = l32 & 1;
        auto rne = [](int b) { uint32_t u = (uint32_t)b; return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16; };
        const int even_row = bits[2 * p], odd_row = bits[2 * p + 1];
        const int mine_keep = odd ? odd_row : even_row;
        const int mine_send = odd ? even_row : odd_row;
        const int got = __builtin_amdgcn_mov_dpp(mine_send, 0xB1, 0xF, 0xF, true);   // quad_perm [1, 0, 3, 2]: lane ^ 1
        const uint32_t lo = rne(odd ? got : mine_keep), hi = rne(odd ? mine_keep : got);
        return lo | (hi << 16);
    };
    auto out16_phase = [&]() {
        // bf16 output (round to nearest even).  A 32x32 block is only 64 bytes wide in bf16, so the wavefront's
        // 32 x WN strip is first assembled in a private piece of the idle LDS ring (neighbouring lanes swap half of
        // their rows so that a lane writes two adjacent columns as one 32-bit word) and then leaves as 16-byte
        // stores that cover whole WN * 2-byte row segments.
        constexpr int ROWB = C::WN * 2, STRIP = 32 * ROWB, CPR = C::WN / 8;   // bytes per row / strip, 16-byte chunks per row
        static_assert(C::NW * STRIP <= C::LDS_BYTES, "output strips must fit the ring");
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();            // every wavefront is done reading the staged operands
        asm volatile("" ::: "memory");
        lds_i8* strip_w = dma + wave * STRIP;
        const lds_i8* strip_r = rd + wave * STRIP;
        const bool odd = l32 & 1;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t ib = row0 + i * 32;
            if (ib >= g.M) continue;             // uniform over the wavefront
#pragma unroll
            for (int j = 0; j < TN; ++j) {
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const uint32_t word = pack16(acc[i][j], p);
                    const int v = 2 * p + (odd ? 1 : 0);
                    const int row = (v >> 2) * 8 + lhi * 4 + (v & 3);
                    *(__attribute__((address_space(3))) uint32_t*)(strip_w + row * ROWB + (j * 32 + (l32 & ~1)) * 2) = word;
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int it = 0; it < (32 * CPR + 63) / 64; ++it) {
                const int q = it * 64 + lane;
                const int row = q / CPR, c16 = q % CPR;
                if (q < 32 * CPR) {
                    const i32x4 val = *(const lds_i32x4*)(strip_r + row * ROWB + c16 * 16);
                    const int64_t grow = ib + row, gcol = col0 + c16 * 8;
                    if (grow < g.M && gcol < g.N) *reinterpret_cast<i32x4*>(g.C16 + grow * g.ldc + gcol) = val;
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the strip is reused by the next block row
        }
    };

    // (bf16 output keeps the phases below - the output strips need the registers - with the arithmetic of the form
    // an fp32 launch takes on the same tile, so that it is that launch's result rounded)
    constexpr bool PIPE = C::NW <= 8 && TM * TN <= 6;
    const bool one_pass = overlap && nl <= 1 && m0 + BM <= g.M && n0 + BN <= g.N;
    if (!OUT16 && one_pass) {
        // ---- the usual case (a whole tile, every staged operand fits side by side, r <= 32): one pass per 32x32
        // block, whose stores leave while the next block computes.  Where the registers allow a second block in
        // flight (at most 96 accumulator registers and two wavefronts per SIMD), the correction and low-rank products of
        // the next block - the latter accumulated from zero, so that neither depends on the conversion arithmetic -
        // are issued before the vector instructions of this block and run under them.  The other tile shapes take
        // the blocks one by one (correction product, conversion, low-rank product onto the result): there the other
        // wavefronts of the SIMD fill the gaps.  The scheduling barrier after each block bounds the live registers.
        constexpr int L_PLANE = 2 * kLoraParts * PLANE_A;
        constexpr int NB = TM * TN;
        // this lane's column scales (a missing scale is 1 or 0); the pipelined form reads them once for its TN
        // block columns, ahead of the loop, so that no block waits for them
        auto read_cs = [&](int j) { return has_cs ? *(const lds_f32*)(cs_plane + (wn * C::WN + j * 32 + l32) * 4) : 1.0f; };
        auto read_cs2 = [&](int j) { return has_cs2 ? *(const lds_f32*)(cs2_plane + (wn * C::WN + j * 32 + l32) * 4) : 0.0f; };
        float col_cs[PIPE ? TN : 1], col_cs2[PIPE ? TN : 1];
        // acc2 = A2 B2^T of the block, nk >= 1 (the first MFMA takes a constant zero as its addend: no register clearing)
        // SIMPLE (the pipelined form's straight-line variant): one outlier slice, r = 16 - no loops, no branches
        auto block_k2 = [&](int i, int j, i32x16& acc2, auto simple) {
            const i32x16 zero = {};
            acc2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(frag(0, wm * C::WM + i * 32, lhi),
                                                         frag(PLANE_A, wn * C::WN + j * 32, lhi), zero, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(frag(0, wm * C::WM + i * 32, 2 + lhi),
                                                         frag(PLANE_A, wn * C::WN + j * 32, 2 + lhi), acc2, 0, 0, 0);
            for (int kk = 1; !decltype(simple)::value && kk < nk; ++kk) {
                const int off = kk * C::K2_PLANES_BYTES;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
                    acc2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(frag(off, wm * C::WM + i * 32, ks * 2 + lhi),
                                                                 frag(off + PLANE_A, wn * C::WN + j * 32, ks * 2 + lhi),
                                                                 acc2, 0, 0, 0);
            }
        };
        // c (+)= T L^T of the block; FROM_ZERO: c is the product alone (r >= 16: the first MFMA's addend is a constant)
        auto block_lora = [&](int i, int j, f32x16& c, auto from_zero, auto simple) {
            constexpr bool FROM_ZERO = decltype(from_zero)::value;
            constexpr bool SIMPLE = decltype(simple)::value;
            if (!FROM_ZERO && nl == 0) return;
#pragma unroll
            for (int h = 0; h < (SIMPLE ? 1 : 2); ++h) {           // 16 columns of r per MFMA
                if (h > 0 && h * 16 >= g.r) continue;
                const bf16x8 lb = __builtin_bit_cast(bf16x8, frag(lora_off + L_PLANE, wn * C::WN + j * 32, h * 2 + lhi));
#pragma unroll
                for (int pl = 0; pl < 2 * kLoraParts; ++pl) {
                    const bf16x8 tf =
                        __builtin_bit_cast(bf16x8, frag(lora_off + pl * PLANE_A, wm * C::WM + i * 32, h * 2 + lhi));
                    if (FROM_ZERO && h == 0 && pl == 0) {
                        const f32x16 zero = {};
                        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf, lb, zero, 0, 0, 0);
                    } else {
                        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf, lb, c, 0, 0, 0);
                    }
                }
            }
        };
        // c = row_scale * (acc * cs + acc2 * cs2) [+ c];  MODE 2: both column scales, 1: cs only, 0: neither
        // (a missing scale is 1 or 0 in the phases below: the same bits, more instructions)
        auto block_dequant = [&](int i, int j, const f32x4 (&rs)[4], const i32x16& acc2, f32x16& c, auto add, auto mode) {
            constexpr bool ADD = decltype(add)::value;
            constexpr int MODE = decltype(mode)::value;
            const float cs = PIPE ? col_cs[PIPE ? j : 0] : read_cs(j), cs2 = PIPE ? col_cs2[PIPE ? j : 0] : read_cs2(j);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float a = (float)acc[i][j][v];
                const float inner = MODE == 2 ? __builtin_fmaf(a, cs, (float)acc2[v] * cs2) : MODE == 1 ? a * cs : a;
                const float r = rs[v >> 2][v & 3];
                c[v] = ADD ? __builtin_fmaf(r, inner, c[v]) : r * inner;
            }
        };
        auto block_prev = [&](int i, int j, f32x16& c) {   // what C holds, as store_block addresses it
            const gchar* base = block_base(i, j);
#pragma unroll
            for (int v = 0; v < 16; ++v)
                c[v] = *(const gfloat*)(base + (int64_t)((v >> 2) * 8 + (v & 3)) * g.ldc * 4 + store_voff);
        };
        auto block_out = [&](int i, int j, const f32x16& c) { store_block_full(i, j, __builtin_bit_cast(i32x16, c)); };
        i32x16 acc2[PIPE ? 2 : 1];
        f32x16 low[PIPE ? 2 : 1];
        f32x4 rs[4];   // this lane's 16 output rows of a block are 4 runs of 4 consecutive rows
        auto block_ahead = [&](int b, int buf, auto mode, auto simple) {   // the MFMA work of block b
            if constexpr (decltype(mode)::value == 2) block_k2(b / TN, b % TN, acc2[buf], simple);   // (nk >= 1)
            if (decltype(simple)::value || nl > 0) {
                block_lora(b / TN, b % TN, low[buf], std::true_type{}, simple);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) low[buf][v] = 0.0f;
            }
        };
        auto run = [&](auto mode, auto simple) {
            constexpr int MODE = decltype(mode)::value;
            constexpr bool SIMPLE = decltype(simple)::value;
            if constexpr (PIPE) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (MODE >= 1) col_cs[j] = read_cs(j);
                    if constexpr (MODE == 2) col_cs2[j] = read_cs2(j);
                }
                block_ahead(0, 0, mode, simple);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int i = b / TN, j = b % TN;
                if (j == 0 || !PIPE) {   // (read per block where registers are short)
#pragma unroll
                    for (int vg = 0; vg < 4; ++vg)
                        rs[vg] = *(const lds_f32x4*)(rs_plane + (wm * C::WM + i * 32 + vg * 8 + lhi * 4) * 4);
                }
                if constexpr (PIPE) {
                    if (b + 1 < NB) block_ahead(b + 1, (b + 1) & 1, mode, simple);
                    f32x16& c = low[b & 1];
                    if constexpr (ACCUM) {
                        f32x16 prev;
                        block_prev(i, j, prev);
#pragma unroll
                        for (int v = 0; v < 16; ++v) c[v] += prev[v];
                    }
                    block_dequant(i, j, rs, acc2[b & 1], c, std::true_type{}, mode);
                    block_out(i, j, c);
                } else {
                    f32x16& c = low[0];
                    if constexpr (MODE == 2) block_k2(i, j, acc2[0], std::false_type{});   // (nk >= 1)
                    if constexpr (ACCUM) block_prev(i, j, c);
                    block_dequant(i, j, rs, acc2[0], c, std::integral_constant<bool, ACCUM>{}, mode);
                    block_lora(i, j, c, std::false_type{}, std::false_type{});
                    block_out(i, j, c);
                }
                if constexpr (PIPE && SIMPLE) {
                    // Issue order of the straight-line variant: the LDS reads of the next block, a first run of this
                    // block's vector instructions over their latency, then one MFMA of the next block (each depends
                    // on the one before) after every further run, the stores last.
                    if (b + 1 < NB) {
                        constexpr int NM = (MODE == 2 ? 2 : 0) + 2 * kLoraParts;      // MFMAs of a block
                        constexpr int NV = 16 * (MODE == 2 ? 5 : MODE == 1 ? 3 : 2) + 16; // vector instructions, about
                        constexpr int RUN = NV / (NM + 1);
                        __builtin_amdgcn_sched_group_barrier(0x100, (MODE == 2 ? 4 : 0) + 1 + 2 * kLoraParts, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, RUN, 0);
#pragma unroll
                        for (int u = 0; u < NM; ++u) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x002, RUN, 0);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        const bool simple = PIPE && nl == 1 && g.r == 16 && nk <= 1;
        auto run_mode = [&](auto mode) {
            if (simple) run(mode, std::true_type{});
            else run(mode, std::false_type{});
        };
        if (!active) return;            // (no barrier follows on this path)
        if (has_cs2) run_mode(std::integral_constant<int, 2>{});
        else if (has_cs) run_mode(std::integral_constant<int, 1>{});
        else run_mode(std::integral_constant<int, 0>{});
        return;
    }
    {
        // bf16 output of a tile whose fp32 form is the pipelined one-pass form: the low-rank product is summed from
        // zero and joins  row_scale * inner  in one fused multiply-add (phase A leaves `inner` in the block)
        const bool low_first = OUT16 && PIPE && one_pass && nl == 1;
        // ---- phase A
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (row0 + i * 32 >= g.M || !active) continue;
            f32x4 rs[4];   // this lane's 16 output rows of the block are 4 runs of 4 consecutive rows
#pragma unroll
            for (int vg = 0; vg < 4; ++vg)
                rs[vg] = *(const lds_f32x4*)(rs_plane + (wm * C::WM + i * 32 + vg * 8 + lhi * 4) * 4);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (col0 + j * 32 >= g.N) continue;
                const int lcol = wn * C::WN + j * 32 + l32;
                const float cs = has_cs ? *(const lds_f32*)(cs_plane + lcol * 4) : 1.0f;
                const float cs2 = has_cs2 ? *(const lds_f32*)(cs2_plane + lcol * 4) : 0.0f;
                i32x16 acc2;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[v] = 0;
                for (int kk = 0; kk < nk; ++kk) {
                    const int off = kk * C::K2_PLANES_BYTES;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
                        acc2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(frag(off, wm * C::WM + i * 32, ks * 2 + lhi),
                                                                     frag(off + PLANE_A, wn * C::WN + j * 32, ks * 2 + lhi),
                                                                     acc2, 0, 0, 0);
                }
                float prev[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) prev[v] = 0.0f;
                if constexpr (ACCUM) {
                    // this lane's 16 output elements of the block, as phase C addresses them (clamped: never stored)
                    const int64_t ib = row0 + i * 32, col = col0 + j * 32 + l32;
                    const int64_t cc = col < g.N ? col : g.N - 1;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int64_t row = ib + (v >> 2) * 8 + lhi * 4 + (v & 3);
                        prev[v] = g.C[(row < g.M ? row : g.M - 1) * g.ldc + cc];
                    }
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float inner = __builtin_fmaf((float)acc[i][j][v], cs, (float)acc2[v] * cs2);
                    acc[i][j][v] = __float_as_int(low_first ? inner : rs[v >> 2][v & 3] * inner + prev[v]);
                }
            }
        }

        // ---- phase B
        for (int lc = 0; lc < nl; ++lc) {
            if (!(overlap && lc == 0)) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();          // everybody has read what the next loads overwrite
                asm volatile("" ::: "memory");
                issue_lora(lc);
                landed();
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (row0 + i * 32 >= g.M || !active) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (col0 + j * 32 >= g.N) continue;
                    const f32x16 inner = __builtin_bit_cast(f32x16, acc[i][j]);
                    f32x16 c = inner;
                    if (low_first) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) c[v] = 0.0f;
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h) {           // 16 columns of r per MFMA
                        if (lc * 32 + h * 16 >= g.r) continue;
                        const bf16x8 lb = __builtin_bit_cast(
                            bf16x8, frag(lora_off + 2 * kLoraParts * PLANE_A, wn * C::WN + j * 32, h * 2 + lhi));
#pragma unroll
                        for (int pl = 0; pl < 2 * kLoraParts; ++pl)
                            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8, frag(lora_off + pl * PLANE_A, wm * C::WM + i * 32, h * 2 + lhi)),
                                lb, c, 0, 0, 0);
                    }
                    if (low_first) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int row = wm * C::WM + i * 32 + (v >> 2) * 8 + lhi * 4 + (v & 3);
                            c[v] = __builtin_fmaf(*(const lds_f32*)(rs_plane + row * 4), inner[v], c[v]);
                        }
                    }
                    acc[i][j] = __builtin_bit_cast(i32x16, c);
                }
            }
        }
    }

    // ---- phase C
    if constexpr (OUT16) {
        out16_phase();
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if (row0 + i * 32 >= g.M || col0 + j * 32 >= g.N || !active) continue;
            store_block(i, j, acc[i][j]);
        }
    }
}

// Contraction split over the two workgroups of a tile (KSPLIT = 2).  The "giver" (second half of the contraction)
// writes its int32 accumulators, register image by register image, into the exchange buffer and raises the tile's
// flag; the "taker" (first half) adds them to its own and runs the epilogue: the sums are integers, so the result is
// the unsplit product bit for bit.  The hand-over relies on the two workgroups sharing an L2, which the launch grid
// arranges (same XCD) but the hardware does not promise: the giver records the XCD it ran on, and a taker on another
// one - or one whose bounded wait runs out - computes the second half itself instead.  The flag is exchanged, never
// just written: whoever finds the other's mark resets the word to zero, so a finished launch always leaves zeros.
constexpr unsigned long long kSplitFull = 0x5146474956450000ull;        // | XCD of the giver
constexpr unsigned long long kSplitAbandoned = 0x5146414241440000ull;
__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg(((4 - 1) << 11) | 20) & 15u; }

template <int BM, int BN, int WGM, int WGN, int STAGES, bool DUMP, int MINB = 1, int PAIR = 0, bool STAGED = false,
          bool ACCUM = false, bool OUT16 = false, bool BT = false, int KSPLIT = 1>
__global__ void __launch_bounds__(64 * WGM * WGN, MINB)
gemm_i8_dma_kernel(const GemmArgs g, const TileMap tmap) {
    using C = DmaCfg<BM, BN, WGM, WGN, STAGES>;
    extern __shared__ __attribute__((aligned(1024))) int8_t lds_raw[];
    lds_i8* lds = (lds_i8*)lds_raw;
    static_assert(KSPLIT == 1 || (KSPLIT == 2 && PAIR == 2), "the split exists for the wide-stage main loop");

    int tile_m, tile_n;
    // (split: the two workgroups of a tile are neighbours in y, so they carry the same blockIdx.x = XCD)
    const int kh = KSPLIT == 2 ? (int)(blockIdx.y & 1) : 0;
    if (!tile_of_block(tmap, blockIdx.x, KSPLIT == 2 ? blockIdx.y >> 1 : blockIdx.y, blockIdx.z, tile_m, tile_n)) return;

    const int tid = threadIdx.x, lane = tid & 63;
    // The wavefront number is uniform; telling the compiler so moves the loader's address selects to scalar code,
    // which is faster where several wavefronts share a SIMD and slower where one wavefront has it to itself (measured).
    const int wave = C::WAVE_SCALAR ? __builtin_amdgcn_readfirstlane(tid >> 6) : tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

    // loader: a direct load fills 16 rows x 64 bytes of a stage (A rows first, then B rows); lane -> (row = lane / 4,
    // slot = lane % 4) and the slot holds global chunk slot ^ ((row / 4) & 3), the swizzle the fragment reads undo
    if constexpr (PAIR == 2) {
        // wide stages: a direct load fills 8 rows x 128 bytes; lane -> (row = lane / 8, slot = lane % 8) and the slot
        // holds global chunk slot ^ ((row >> 1) & 7)
        uint32_t voffw[C::NLOAD_W];
#pragma unroll
        for (int j = 0; j < C::NLOAD_W; ++j) {
            int q = j * C::NW + wave;
            if (q >= C::NGROUP_W) q -= C::NW;
            const bool isA = q < BM / 8;
            const int local = (isA ? q : q - BM / 8) * 8 + (lane >> 3);
            const int chunk = (lane & 7) ^ ((local >> 1) & 7);
            int64_t row = (isA ? m0 : n0) + local;
            int64_t lim = (isA ? g.M : g.N) - 1;
            row = row < lim ? row : lim;
            voffw[j] = (uint32_t)(row * (isA ? g.lda : g.ldb) + chunk * 16);
            if (!BT && !isA && g.b_layout == kPackedNK) voffw[j] = (uint32_t)weight_code_offset(row, chunk * 16, g.ldb);
            if (BT && !isA) {
                // B stored [K x N]: the stage's B part is 128 contraction rows of BN bytes; this lane fills the
                // 16-byte slot number (q - BM / 8) * 64 + lane of it
                int krow, lcol;
                BtStage<BN>::slot_source((q - BM / 8) * 64 + lane, krow, lcol);
                int64_t col = n0 + lcol;
                col = col < g.N - 16 ? col : g.N - 16;      // clamp: columns past the edge are never stored
                voffw[j] = (uint32_t)weight_code_offset(krow, col, g.ldb);
            }
        }
        const int64_t b_step = BT ? 128 * g.ldb : g.b_layout == kPackedNK ? 256 : 128;
        const int fragw = l32 * 128 + ((lhi ^ ((l32 >> 1) & 7)) * 16);
        int b_off[C::TN];
#pragma unroll
        for (int j = 0; j < C::TN; ++j) {
            if constexpr (BT) {
                b_off[j] = BtStage<BN>::piece_offset(lane, wn * C::WN / 32 + j);
            } else {
                b_off[j] = wn * C::WN * 128 + fragw + j * 4096;
            }
        }
        i32x16 accw[C::TM][C::TN];
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) accw[i][j][v] = 0;
        const int KT = (int)(g.K / 128) / KSPLIT;
        const int a_frag = wm * C::WM * 128 + fragw;
        gemm_mainloop_dma128<C, BT>(g.A + (int64_t)kh * KT * 128, g.B + kh * KT * b_step, voffw, KT, lds, lds, wave, a_frag,
                                    b_off, b_step, accw);
        bool active = true;                                  // does this wavefront finish (dequantise, store) its block
        if constexpr (KSPLIT == 2) {
            // Workgroup kh finishes the tile's row half kh: its wavefronts of the other half ("givers") ship their
            // accumulators to the partner workgroup, its wavefronts of row half kh ("takers") add what the partner's
            // same-numbered wavefronts ship.  Thread tid of one workgroup writes slot tid, thread tid of the other
            // reads it: piece q of a thread at [q][tid], so that every store and load covers whole lines.
            constexpr int NV = C::TM * C::TN * 4;          // 16-byte pieces of a lane's accumulators
            const int64_t tile_id = (int64_t)tile_m * tmap.tiles_n + tile_n;
            // (the two flags of a tile sit 128 bytes apart, each in a line of its own)
            unsigned long long* flags = reinterpret_cast<unsigned long long*>(g.split_scratch) + tile_id * 32;
            i32x4* xb = reinterpret_cast<i32x4*>(static_cast<char*>(g.split_scratch) +
                                                 (size_t)tmap.tiles_m * tmap.tiles_n * 256) +
                        tile_id * NV * C::NT + tid;
            const bool giver = (wm >= WGM / 2) == (kh == 0);
            active = !giver;
            if (giver) {
#pragma unroll
                for (int i = 0; i < C::TM; ++i)
#pragma unroll
                    for (int j = 0; j < C::TN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            xb[((i * C::TN + j) * 4 + q) * C::NT] = (i32x4){accw[i][j][4 * q], accw[i][j][4 * q + 1],
                                                                             accw[i][j][4 * q + 2], accw[i][j][4 * q + 3]};
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's pieces have reached the L2
            }
            __syncthreads();     // all givers of this workgroup have written; nobody reads the ring any more
            if (tid == 0) {
                // raise this workgroup's flag ...
                const unsigned long long old = __hip_atomic_exchange(flags + 16 * kh, kSplitFull | xcc_id(), __ATOMIC_RELAXED,
                                                                     __HIP_MEMORY_SCOPE_AGENT);
                if (old == kSplitAbandoned)     // (the partner stopped waiting and does the work itself)
                    __hip_atomic_store(flags + 16 * kh, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                // ... and wait, for a bounded time, for the partner's
                unsigned long long* theirs = flags + 16 * (1 - kh);
                const long long t0 = (long long)wall_clock64();
                unsigned long long w;
                int take = 0;
                for (;;) {
                    w = __hip_atomic_load(theirs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((w & ~15ull) == kSplitFull) break;
                    if ((long long)wall_clock64() - t0 >= g.split_wait_ticks) {
                        w = __hip_atomic_exchange(theirs, kSplitAbandoned, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
                if ((w & ~15ull) == kSplitFull) {
                    take = (unsigned)(w & 15ull) == xcc_id();
                    if (!take) __hip_atomic_store(theirs, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                *reinterpret_cast<volatile int*>(lds_raw) = take;
            }
            __syncthreads();
            const int take = *reinterpret_cast<volatile int*>(lds_raw);
            __syncthreads();
            if (take) {
                if (active) {
#pragma unroll
                    for (int i = 0; i < C::TM; ++i)
#pragma unroll
                        for (int j = 0; j < C::TN; ++j)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const i32x4 v = xb[((i * C::TN + j) * 4 + q) * C::NT];
#pragma unroll
                                for (int e = 0; e < 4; ++e) accw[i][j][4 * q + e] += v[e];
                            }
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                }
                __syncthreads();                 // all pieces read: the partner's flag goes back to zero
                if (tid == 0) __hip_atomic_store(flags + 16 * (1 - kh), 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                // the other half of the contraction, computed here (the givers' sums are not used again)
                gemm_mainloop_dma128<C, BT>(g.A + (int64_t)(1 - kh) * KT * 128, g.B + (1 - kh) * KT * b_step, voffw, KT,
                                            lds, lds, wave, a_frag, b_off, b_step, accw);
            }
        }
        if constexpr (STAGED && !DUMP)
            gemm_epilogue_staged<C, ACCUM, OUT16>(g, accw, lds, lds, m0, n0, wm, wn, wave, lane, active);
        else
            gemm_epilogue<C::TM, C::TN, DUMP>(g, accw, m0 + wm * C::WM, n0 + wn * C::WN, l32, lhi);
        return;
    }
    static_assert(!BT || PAIR == 2, "the [K x N] B layout exists for the wide-stage main loop only");
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
            voff[j] = (uint32_t)(row * (isA ? g.lda : g.ldb) + chunk * 16);
            if (!isA && g.b_layout == kPackedNK) voff[j] = (uint32_t)weight_code_offset(row, chunk * 16, g.ldb);
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

    gemm_mainloop_dma<C>(g.A, g.B, voff, (int)(g.K / C::BK), lds, lds, wave, a_frag_off, b_frag_off,
                         g.b_layout == kPackedNK ? 128 : 64, acc);

    if constexpr (STAGED && !DUMP)
        gemm_epilogue_staged<C, ACCUM, OUT16>(g, acc, lds, lds, m0, n0, wm, wn, wave, lane);
    else
        gemm_epilogue<C::TM, C::TN, DUMP>(g, acc, m0 + wm * C::WM, n0 + wn * C::WN, l32, lhi);
}

// host side: choose the XCD region grid for a grid of bm x bn tiles.  Padded work first (a surplus workgroup idles a
// compute unit for a whole pass), then the operand rows an XCD has to fetch into its own L2: rm * bm rows of A plus
// rn * bn rows of B, every one K bytes long.  (Eight L2s that share nothing cannot fetch less than the sum of these
// over the XCDs: 78.6 MB for a 2048 x 9216 x 3072 product in 256 x 288 tiles, against 34.6 MB of operands.)
inline TileMap make_tile_map(int tiles_m, int tiles_n, int bm, int bn, int wgs_per_cu) {
    TileMap best{tiles_m, tiles_n, 1, 8, tiles_m, (tiles_n + 7) / 8, 3, 1};
    long best_cost = -1;
    const int xms[4] = {1, 2, 4, 8};
    for (int xm : xms) {
        int xn = 8 / xm;
        int rm = (tiles_m + xm - 1) / xm, rn = (tiles_n + xn - 1) / xn;
        long cost = (long)rm * rn * 1000000 + (long)rm * bm + (long)rn * bn;
        const int xn_log2 = xn == 1 ? 0 : xn == 2 ? 1 : xn == 4 ? 2 : 3;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = TileMap{tiles_m, tiles_n, xm, xn, rm, rn, xn_log2, 1}; }
    }
    // tile rows per group: the block of concurrent tiles (32 compute units per XCD) with the fewest operand rows
    const int conc = 32 * wgs_per_cu;
    if (best.rm * best.rn > conc) {
        long gcost = -1;
        for (int gm = 1; gm <= 16 && gm <= best.rm; gm *= 2) {
            // concurrent tiles: `cols` columns of as many whole groups as it takes
            const int cols = (conc + gm - 1) / gm < best.rn ? (conc + gm - 1) / gm : best.rn;
            const int groups = (conc + gm * cols - 1) / (gm * cols);
            const long cst = (long)gm * groups * bm + (long)cols * bn;
            if (gcost < 0 || cst < gcost) { gcost = cst; best.gm = gm; }
        }
    }
    return best;
}

}  // namespace quaff
