// INT8 MFMA GEMM kernel template (see quaff_gemm.hip for the description of the computation).
#pragma once
#include "quaff_internal.h"

namespace quaff {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int BK>
__device__ __forceinline__ int lds_chunk_offset(int row, int chunk) {
    // BK = 64: four chunks per row, rotate by (row / 4) & 3.  BK = 128: eight chunks, rotate by (row / 2) & 7.
    constexpr int CH = BK / 16;
    int sw = (BK == 64) ? ((row >> 2) & 3) : ((row >> 1) & 7);
    return row * BK + ((chunk ^ sw) & (CH - 1)) * 16;
}

// Epilogue shared by the GEMM kernels, for the wavefront tile whose first element is (row0, col0).
// Phase 1 (loads and arithmetic only): for every 32x32 accumulator block, the short second product and the
// low-rank term are formed with a few extra MFMAs and the dequantised fp32 value replaces the int32 accumulator
// in place.  Phase 2 (stores only): the blocks are written out.  Keeping every load ahead of every store matters:
// loads and stores share one in-order counter, so a load issued after a store would wait for that store to drain.
template <int TM, int TN, bool DUMP>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, i32x16 (&acc)[TM][TN], int64_t row0, int64_t col0,
                                              int l32, int lhi) {
    if (DUMP) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t ib = row0 + i * 32;
            const int64_t frag_row = ib + l32 < g.M ? ib + l32 : g.M - 1;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t jb = col0 + j * 32, col = jb + l32;
                const int64_t ccol = col < g.N ? col : g.N - 1;
                if (ib >= g.M || jb >= g.N) continue;
                i32x16 acc2;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[v] = 0;
                for (int kk = 0; kk < g.K2; kk += 32) {
                    i32x4 a = *reinterpret_cast<const i32x4*>(g.A2 + frag_row * g.K2 + kk + lhi * 16);
                    i32x4 b = *reinterpret_cast<const i32x4*>(g.B2 + ccol * g.K2 + kk + lhi * 16);
                    acc2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc2, 0, 0, 0);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int64_t row = ib + (v >> 2) * 8 + lhi * 4 + (v & 3);
                    if (row < g.M && col < g.N) {
                        g.acc1[row * g.N + col] = acc[i][j][v];
                        if (g.acc2) g.acc2[row * g.N + col] = acc2[v];
                    }
                }
            }
        }
        return;
    }

    // ---- phase 1
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t ib = row0 + i * 32;
        if (ib >= g.M) continue;
        const int64_t frag_row = ib + l32 < g.M ? ib + l32 : g.M - 1;   // clamped: rows past the edge are not stored
        float rs[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int64_t row = ib + (v >> 2) * 8 + lhi * 4 + (v & 3);
            rs[v] = g.row_scale[row < g.M ? row : g.M - 1];
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t jb = col0 + j * 32;
            if (jb >= g.N) continue;
            const int64_t ccol = jb + l32 < g.N ? jb + l32 : g.N - 1;
            i32x16 acc2;
            f32x16 lo;
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc2[v] = 0; lo[v] = 0.0f; }
            for (int kk = 0; kk < g.K2; kk += 32) {
                i32x4 a = *reinterpret_cast<const i32x4*>(g.A2 + frag_row * g.K2 + kk + lhi * 16);
                i32x4 b = *reinterpret_cast<const i32x4*>(g.B2 + ccol * g.K2 + kk + lhi * 16);
                acc2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc2, 0, 0, 0);
            }
            for (int pp = 0; pp < g.r; pp += 16) {
                i32x4 lb = *reinterpret_cast<const i32x4*>(g.L + ccol * g.r + pp + lhi * 8);
#pragma unroll
                for (int part = 0; part < kLoraParts; ++part) {
                    const int64_t po = (int64_t)part * g.M * g.r;
                    i32x4 th = *reinterpret_cast<const i32x4*>(g.T_hi + po + frag_row * g.r + pp + lhi * 8);
                    i32x4 tl = *reinterpret_cast<const i32x4*>(g.T_lo + po + frag_row * g.r + pp + lhi * 8);
                    lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, th),
                                                                 __builtin_bit_cast(bf16x8, lb), lo, 0, 0, 0);
                    lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tl),
                                                                 __builtin_bit_cast(bf16x8, lb), lo, 0, 0, 0);
                }
            }
            const float cs = g.col_scale ? g.col_scale[ccol] : 1.0f;
            const float cs2 = g.K2 > 0 ? g.col_scale2[ccol] : 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float inner = __builtin_fmaf((float)acc[i][j][v], cs, (float)acc2[v] * cs2);
                acc[i][j][v] = __float_as_int(__builtin_fmaf(rs[v], inner, lo[v]));
            }
        }
    }
    // ---- phase 2
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t ib = row0 + i * 32;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t jb = col0 + j * 32, col = jb + l32;
            if (ib >= g.M || jb >= g.N) continue;
            float* out = g.C + (ib + lhi * 4) * g.ldc + col;
            if (ib + 32 <= g.M && jb + 32 <= g.N) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    out[((v >> 2) * 8 + (v & 3)) * g.ldc] = __int_as_float(acc[i][j][v]);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int64_t row = ib + (v >> 2) * 8 + lhi * 4 + (v & 3);
                    if (row < g.M && col < g.N) out[((v >> 2) * 8 + (v & 3)) * g.ldc] = __int_as_float(acc[i][j][v]);
                }
            }
        }
    }
}

typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) i32x2 lds_i32x2;

// BT: B is read as [K x N] from the packed weight codes; its tile is staged row-major [BK][BN] and the fragments are
// gathered with transposing LDS reads (see BtStage in quaff_gemm_dma.h for the lane mapping).
template <int BM, int BN, int BK, int WGM, int WGN, bool DUMP, bool BT = false>
__global__ void __launch_bounds__(64 * WGM * WGN)
gemm_i8_kernel(const GemmArgs g, int tiles_n) {
    constexpr int NT = 64 * WGM * WGN;            // threads per workgroup
    constexpr int WM = BM / WGM, WN = BN / WGN;   // wavefront tile
    constexpr int TM = WM / 32, TN = WN / 32;     // 32x32 MFMA blocks per wavefront tile
    constexpr int CH = BK / 16;                   // 16-byte chunks per staged row
    constexpr int A_LOADS = BM * CH / NT, B_LOADS = BN * CH / NT;
    static_assert(BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "tile shape");
    static_assert((BM * CH) % NT == 0 && (BN * CH) % NT == 0, "loader mapping");
    static_assert(A_LOADS >= 1 && B_LOADS >= 1, "tile too small for the loader threads");

    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    int8_t* As = lds;                      // [2][BM * BK]
    int8_t* Bs = lds + 2 * BM * BK;        // [2][BN * BK]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * BM;
    const int64_t n0 = (int64_t)(blockIdx.x % tiles_n) * BN;

    // loader mapping: thread -> (row, chunk) pairs, CH consecutive threads cover one staged row
    const int ld_chunk = tid % CH, ld_row = tid / CH;
    constexpr int ROWS_PER_PASS = NT / CH;

    i32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    i32x4 pa[A_LOADS], pb[B_LOADS];
    auto fetch = [&](int64_t k0) {
        const int64_t k = k0 + ld_chunk * 16;
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p) {
            int64_t row = m0 + ld_row + p * ROWS_PER_PASS;
            pa[p] = (i32x4){0, 0, 0, 0};
            if (row < g.M && k < g.K) pa[p] = *reinterpret_cast<const i32x4*>(g.A + row * g.lda + k);
        }
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            pb[p] = (i32x4){0, 0, 0, 0};
            if constexpr (BT) {
                const int idx = tid + p * NT;                     // 16-byte piece of the [BK][BN] tile
                const int64_t kr = k0 + idx / (BN / 16), col = n0 + (idx % (BN / 16)) * 16;
                if (kr < g.K && col < g.N)
                    pb[p] = *reinterpret_cast<const i32x4*>(g.B + weight_code_offset(kr, col, g.ldb));
            } else {
                int64_t row = n0 + ld_row + p * ROWS_PER_PASS;
                if (row < g.N && k < g.K)
                    pb[p] = *reinterpret_cast<const i32x4*>(
                        g.B + (g.b_layout == kPackedNK ? weight_code_offset(row, k, g.ldb) : row * g.ldb + k));
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p)
            *reinterpret_cast<i32x4*>(As + buf * BM * BK + lds_chunk_offset<BK>(ld_row + p * ROWS_PER_PASS, ld_chunk)) = pa[p];
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p) {
            if constexpr (BT)
                *reinterpret_cast<i32x4*>(Bs + buf * BN * BK + (tid + p * NT) * 16) = pb[p];
            else
                *reinterpret_cast<i32x4*>(Bs + buf * BN * BK + lds_chunk_offset<BK>(ld_row + p * ROWS_PER_PASS, ld_chunk)) = pb[p];
        }
    };
    // BT: this lane's 8-byte piece of the transposing read (lane = 16 grp + 2 jj + piece), first column block
    const int bt_off = (((lane >> 4) >> 1) * 16 + ((lane & 15) >> 1)) * BN + wn * WN + ((lane >> 4) & 1) * 16 + (lane & 1) * 8;

    const int KT = (int)((g.K + BK - 1) / BK);
    fetch(0);
    stage(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) fetch((int64_t)(kt + 1) * BK);
        const int8_t* at = As + buf * BM * BK;
        const int8_t* bt = Bs + buf * BN * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            i32x4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const i32x4*>(at + lds_chunk_offset<BK>(wm * WM + i * 32 + l32, ks * 2 + lhi));
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if constexpr (BT) {
                    const int8_t* pp = bt + bt_off + j * 32 + ks * 32 * BN;
                    const i32x2 lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)pp);
                    const i32x2 hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2*)(pp + 8 * BN));
                    fb[j] = (i32x4){lo[0], lo[1], hi[0], hi[1]};
                } else {
                    fb[j] = *reinterpret_cast<const i32x4*>(bt + lds_chunk_offset<BK>(wn * WN + j * 32 + l32, ks * 2 + lhi));
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) stage(buf ^ 1);
        __syncthreads();
    }

    gemm_epilogue<TM, TN, DUMP>(g, acc, m0 + wm * WM, n0 + wn * WN, l32, lhi);
}

}  // namespace quaff
