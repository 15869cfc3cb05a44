// INT8 MFMA GEMM with int32 accumulation and a fused dequantising epilogue (Eq. 9 of the paper) that also
// adds the rank-r LoRA term.  The same kernels serve the forward product (contraction over c_in) and the
// input-gradient product (contraction over c_out).  A is contraction-contiguous; B is either a plain
// contraction-contiguous [N x K] matrix or the packed weight codes (one copy, quaff_internal.h), read as [N x K] by
// the forward product and as [K x N], through transposing LDS reads, by the input-gradient product.
//
//   C[i, j] = row_scale[i] * ( acc1[i, j] * col_scale[j] + acc2[i, j] * col_scale2[j] ) + sum_p T[i, p] L[j, p]
//   acc1 = A B^T   (K long, the hot loop),   acc2 = A2 B2^T   (K2 = padded outlier count, done in the epilogue)
//
// Two kernels share the epilogue:
//   gemm_i8_dma_kernel  the fast path (contraction a multiple of 64): direct-to-LDS operand streaming through a ring
//                       of stages, v_mfma_i32_32x32x32_i8, XCD-aware tile order (quaff_gemm_dma.h);
//   gemm_i8_kernel      register-staged fallback for contractions that are not a multiple of 64 (128 for the
//                       [K x N] reading) (quaff_gemm_kernel.h).
#include "quaff_gemm_dma.h"

namespace quaff {

template <int BM, int BN, int BK, int WGM, int WGN>
static hipError_t launch_generic(const GemmArgs& g, bool dump, hipStream_t stream) {
    int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
    size_t lds = 2 * (size_t)(BM + BN) * BK;
    dim3 grid((unsigned)(tiles_m * tiles_n));
    const bool bt = g.b_layout == kPackedKN;
    auto k = dump ? (bt ? gemm_i8_kernel<BM, BN, BK, WGM, WGN, true, true> : gemm_i8_kernel<BM, BN, BK, WGM, WGN, true, false>)
                  : (bt ? gemm_i8_kernel<BM, BN, BK, WGM, WGN, false, true> : gemm_i8_kernel<BM, BN, BK, WGM, WGN, false, false>);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k, grid, dim3(64 * WGM * WGN), lds, stream, g, tiles_n);
    return hipGetLastError();
}

// BT: B is read as [K x N] from the packed weight codes (wide-stage main loop only)
template <int BM, int BN, int WGM, int WGN, int STAGES, int MINB, int PAIR = 0, bool BT = false, int KSPLIT = 1>
static hipError_t launch_dma(const GemmArgs& g, bool dump, hipStream_t stream) {
    using C = DmaCfg<BM, BN, WGM, WGN, STAGES>;
    int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
    TileMap tm = make_tile_map(tiles_m, tiles_n, BM, BN, MINB);
#ifdef QUAFF_FORCE_GM
    tm.gm = QUAFF_FORCE_GM < tm.rm ? QUAFF_FORCE_GM : 1;
#endif
    // x % 8 = XCD, x / 8 = tile row inside a group of gm, y = tile column, z = group; a split contraction doubles y
    // (the two halves of a tile are neighbours)
    const int groups = (tm.rm + tm.gm - 1) / tm.gm;
    dim3 grid(8 * (unsigned)tm.gm, (unsigned)tm.rn * KSPLIT, (unsigned)groups), block(C::NT);
    if (tm.rn * KSPLIT > 65535 || groups > 65535) return hipErrorInvalidValue;
    if constexpr (KSPLIT == 2) {
        if (dump || g.C16 || g.accumulate || (int64_t)(g.K2 / 64) * C::K2_PLANES_BYTES > C::EPI_LIMIT)
            return hipErrorInvalidValue;
        auto k = gemm_i8_dma_kernel<BM, BN, WGM, WGN, STAGES, false, MINB, PAIR, true, false, false, BT, 2>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_ALLOC);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, block, C::LDS_ALLOC, stream, g, tm);
        return hipGetLastError();
    } else if (dump) {
        auto k = gemm_i8_dma_kernel<BM, BN, WGM, WGN, STAGES, true, MINB, PAIR, false, false, false, BT>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, block, C::LDS_BYTES, stream, g, tm);
    } else if ((int64_t)(g.K2 / 64) * C::K2_PLANES_BYTES <= C::EPI_LIMIT) {
        // the epilogue operands are staged through the idle LDS ring
        auto k = g.C16          ? gemm_i8_dma_kernel<BM, BN, WGM, WGN, STAGES, false, MINB, PAIR, true, false, true, BT>
                 : g.accumulate ? gemm_i8_dma_kernel<BM, BN, WGM, WGN, STAGES, false, MINB, PAIR, true, true, false, BT>
                                : gemm_i8_dma_kernel<BM, BN, WGM, WGN, STAGES, false, MINB, PAIR, true, false, false, BT>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_ALLOC);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, block, C::LDS_ALLOC, stream, g, tm);
    } else {
        return hipErrorInvalidValue;   // launch_gemm splits such a product into two launches
    }
    return hipGetLastError();
}

namespace {
// Tile shapes of the fast path.  `spc` = workgroups that fit on one compute unit at once (LDS and registers);
// `ineff` = measured cost per MAC relative to the 256x256 shape on a large problem.
struct TileChoice { int bm, bn, spc; double ineff; };
constexpr TileChoice kChoices[4] = {
    {256, 256, 1, 1.00},   // 8 wavefronts, 128x64 each
    {256, 288, 1, 1.03},   // 12 wavefronts, 64x96 each: 2048 x 9216 outputs are exactly 256 such tiles
    {256, 128, 1, 1.18},   // 8 wavefronts, 64x64 each (its wide-stage ring leaves room for one workgroup per unit)
    {128, 192, 2, 1.20},   // 4 wavefronts, 64x96 each: 2048 x 3072 outputs are exactly 256 such tiles
};

// Estimated time of a tile shape on 256 compute units: full rounds of spc tiles per unit, then the remainder at one
// tile per unit per pass.  The shape that wastes the fewest compute-unit passes wins.
int choose_tile(int64_t M, int64_t N) {
    int best = 0;
    double best_cost = -1.0;
    for (int c = 0; c < 4; ++c) {
        const TileChoice& t = kChoices[c];
        int64_t tiles = ((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
        int64_t slots = 256 * t.spc;
        int64_t full = tiles / slots, rem = tiles % slots;
        double passes = (double)full * t.spc + (double)((rem + 255) / 256);
        double cost = passes * t.bm * t.bn * t.ineff;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = c; }
    }
    return best;
}
}  // namespace

static hipError_t launch_gemm_one(const GemmArgs& g, bool dump_acc, hipStream_t stream);

// A product whose output is at most 128 tiles of 256 x 192 (a 2048 x 3072 output is exactly 128) with a long
// contraction runs as two workgroups per tile, each over half of the contraction: 30 % fewer operand bytes per
// multiply-add than one 128 x 192 tile per compute unit, whose main loop is bound by the delivery of operands from L2
// into LDS.  The price is one more trip of the output's worth of int32 sums through the L2 (written, read, and
// written back when the kernel ends): measured on 2048 x 3072 outputs, the split loses at K = 3072, breaks even at
// K = 9216 (66.7 against 67.2 us) and wins at K = 16384 (103 against 111 us).
#ifndef QUAFF_SPLIT_MIN_K
#define QUAFF_SPLIT_MIN_K 12288
#endif
static bool split_applies(int64_t M, int64_t N, int64_t K) {
    const int64_t tiles = ((M + 255) / 256) * ((N + 191) / 192);
    return K % 256 == 0 && K >= QUAFF_SPLIT_MIN_K && tiles > 64 && tiles <= 128;
}
size_t gemm_split_bytes(int64_t M, int64_t N, int64_t K) {
    if (!split_applies(M, N, K)) return 0;
    const size_t tiles = (size_t)((M + 255) / 256) * (size_t)((N + 191) / 192);
    return tiles * 256 + tiles * 512 * 96 * 4;   // two flags per tile in lines of their own, then 96 accumulators of 512 threads
}

// the direct-to-LDS loader addresses an operand with 32-bit offsets from its tile's first row
static bool fast_path_ok(const GemmArgs& g) {
    const int64_t lim32 = (int64_t)1 << 32;
    if (g.K % 64 != 0 || g.M * g.lda >= lim32) return false;
    if (g.b_layout == kPackedKN) return g.K % 128 == 0 && 130 * g.ldb < lim32;   // 128 contraction rows per stage
    return (g.N + 2) * g.ldb < lim32;
}


hipError_t launch_gemm(const GemmArgs& g, bool dump_acc, hipStream_t stream) {
    ProfScope prof(K_GEMM, stream);
    // A second product too wide for the epilogue's LDS staging (more than two to four 64-wide outlier slices,
    // depending on the tile shape) runs as a launch of its own that writes row_scale * acc2 * col_scale2, and the
    // main product then accumulates onto it: one extra write and read of the output instead of a slow epilogue.
    const bool main_fast = fast_path_ok(g);
    // bf16 output exists in the fast kernel's single-launch form only
    if (g.C16 && (!main_fast || g.K2 > 128 || dump_acc)) return hipErrorNotSupported;
    if (!dump_acc && g.K2 > 128 && main_fast) {
        GemmArgs c2{};
        c2.A = g.A2; c2.lda = g.K2; c2.B = g.B2; c2.ldb = g.K2;
        c2.M = g.M; c2.N = g.N; c2.K = g.K2;
        c2.row_scale = g.row_scale; c2.col_scale = g.col_scale2;
        c2.C = g.C; c2.ldc = g.ldc;
        hipError_t e = launch_gemm_one(c2, false, stream);
        if (e != hipSuccess) return e;
        GemmArgs m = g;
        m.K2 = 0; m.A2 = nullptr; m.B2 = nullptr; m.col_scale2 = nullptr;
        m.accumulate = 1;
        return launch_gemm_one(m, false, stream);
    }
    return launch_gemm_one(g, dump_acc, stream);
}

hipError_t launch_gemm_one(const GemmArgs& g, bool dump_acc, hipStream_t stream) {
    if (!fast_path_ok(g)) return launch_generic<128, 128, 64, 2, 2>(g, dump_acc, stream);
    if (g.split_scratch && !dump_acc && !g.C16 && !g.accumulate && g.K2 <= 128 && split_applies(g.M, g.N, g.K)) {
        if (g.b_layout == kPackedKN) return launch_dma<256, 192, 4, 2, 4, 1, 2, true, 2>(g, false, stream);
        return launch_dma<256, 192, 4, 2, 4, 1, 2, false, 2>(g, false, stream);
    }
    // The 128 x 192 tile with at most one tile per compute unit takes a ring of three wide stages (120 KB of LDS: one
    // workgroup per unit): the operands of the stage after next are then in flight too, which is what a product whose
    // operands come from HBM rather than from the Infinity Cache needs (measured back to back on operand sets that
    // rotate through more than the cache holds: o_proj forward 36.2 -> 30.5 us, qkv dX 79.2 -> 69.8, 8192 -> 3072
    // forward 74.1 -> 61.7; on cached operands the two rings are level, 29.4 / 65.6 / 60.1 us).  It is compiled for
    // the register budget of two workgroups per unit like the two-stage form (with the whole file to itself the
    // compiler's schedule is 2 - 8 % slower).  With more tiles than units two workgroups per unit overlap each
    // other's epilogues instead, which needs the smaller ring.
    const bool one_round = ((g.M + 127) / 128) * ((g.N + 191) / 192) <= 256;
    if (g.b_layout == kPackedKN) {
        switch (choose_tile(g.M, g.N)) {
            case 0: return launch_dma<256, 256, 2, 4, 4, 1, 2, true>(g, dump_acc, stream);
            case 1: return launch_dma<256, 288, 4, 3, 4, 1, 2, true>(g, dump_acc, stream);
            case 2: return launch_dma<256, 128, 4, 2, 4, 1, 2, true>(g, dump_acc, stream);
            default: return one_round ? launch_dma<128, 192, 2, 2, 6, 2, 2, true>(g, dump_acc, stream)
                                      : launch_dma<128, 192, 2, 2, 4, 2, 2, true>(g, dump_acc, stream);
        }
    }
    // contractions that are a multiple of 128 run the wide-stage main loop (128-byte row segments per direct load)
    const bool wide = g.K % 128 == 0;
    switch (choose_tile(g.M, g.N)) {
        case 0: return wide ? launch_dma<256, 256, 2, 4, 4, 1, 2>(g, dump_acc, stream)
                            : launch_dma<256, 256, 2, 4, 3, 1>(g, dump_acc, stream);
        case 1: return wide ? launch_dma<256, 288, 4, 3, 4, 1, 2>(g, dump_acc, stream)
                            : launch_dma<256, 288, 4, 3, 3, 1>(g, dump_acc, stream);
        case 2: return wide ? launch_dma<256, 128, 4, 2, 4, 1, 2>(g, dump_acc, stream)
                            : launch_dma<256, 128, 4, 2, 3, 1>(g, dump_acc, stream);
        default: return wide ? (one_round ? launch_dma<128, 192, 2, 2, 6, 2, 2>(g, dump_acc, stream)
                                          : launch_dma<128, 192, 2, 2, 4, 2, 2>(g, dump_acc, stream))
                             : launch_dma<128, 192, 2, 2, 4, 2>(g, dump_acc, stream);
    }
}

}  // namespace quaff
