// INT8 MFMA GEMM with int32 accumulation and a fused dequantising epilogue (Eq. 9 of the paper) that also
// adds the rank-r LoRA term.  The same kernel serves the forward product (contraction over c_in) and the
// input-gradient product (contraction over c_out): both operands arrive contraction-contiguous.
//
//   C[i, j] = row_scale[i] * ( acc1[i, j] * col_scale[j] + acc2[i, j] * col_scale2[j] ) + sum_p T[i, p] L[j, p]
//   acc1 = A B^T   (K long, the hot loop),   acc2 = A2 B2^T   (K2 = padded outlier count, done in the epilogue)
//
// Work decomposition: 256 threads (four wavefronts) per BM x BN output tile; v_mfma_i32_32x32x32_i8 with 16
// contraction bytes per lane; operand tiles are staged through LDS in BK-byte rows whose 16-byte chunks are
// XOR-swizzled by row so that both the staging writes and the fragment reads (ds_read_b128) are conflict-free.
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

template <int BM, int BN, int BK, int WGM, int WGN, bool DUMP>
__global__ void __launch_bounds__(256)
gemm_i8_kernel(const GemmArgs g, int tiles_n) {
    constexpr int WM = BM / WGM, WN = BN / WGN;   // wavefront tile
    constexpr int TM = WM / 32, TN = WN / 32;     // 32x32 MFMA blocks per wavefront tile
    constexpr int CH = BK / 16;                   // 16-byte chunks per staged row
    constexpr int A_LOADS = BM * CH / 256, B_LOADS = BN * CH / 256;
    static_assert(WGM * WGN == 4 && BM % (32 * WGM) == 0 && BN % (32 * WGN) == 0, "tile shape");
    static_assert(A_LOADS >= 1 && B_LOADS >= 1, "tile too small for 256 loader threads");

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
    constexpr int ROWS_PER_PASS = 256 / CH;

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
            int64_t row = n0 + ld_row + p * ROWS_PER_PASS;
            pb[p] = (i32x4){0, 0, 0, 0};
            if (row < g.N && k < g.K) pb[p] = *reinterpret_cast<const i32x4*>(g.B + row * g.ldb + k);
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < A_LOADS; ++p)
            *reinterpret_cast<i32x4*>(As + buf * BM * BK + lds_chunk_offset<BK>(ld_row + p * ROWS_PER_PASS, ld_chunk)) = pa[p];
#pragma unroll
        for (int p = 0; p < B_LOADS; ++p)
            *reinterpret_cast<i32x4*>(Bs + buf * BN * BK + lds_chunk_offset<BK>(ld_row + p * ROWS_PER_PASS, ld_chunk)) = pb[p];
    };

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
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const i32x4*>(bt + lds_chunk_offset<BK>(wn * WN + j * 32 + l32, ks * 2 + lhi));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) stage(buf ^ 1);
        __syncthreads();
    }

    // ---------------- epilogue, one 32x32 block at a time
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int64_t ib = m0 + wm * WM + i * 32;           // first row of the block
        const int64_t frag_row = ib + l32;                   // row this lane supplies as an MFMA operand
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t jb = n0 + wn * WN + j * 32;
            const int64_t col = jb + l32;                    // column of this lane's accumulator elements
            if (ib >= g.M || jb >= g.N) continue;
            i32x16 acc2;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc2[v] = 0;
            for (int kk = 0; kk < g.K2; kk += 32) {
                i32x4 a = (i32x4){0, 0, 0, 0}, b = (i32x4){0, 0, 0, 0};
                if (frag_row < g.M) a = *reinterpret_cast<const i32x4*>(g.A2 + frag_row * g.K2 + kk + lhi * 16);
                if (col < g.N) b = *reinterpret_cast<const i32x4*>(g.B2 + col * g.K2 + kk + lhi * 16);
                acc2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc2, 0, 0, 0);
            }
            if (DUMP) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int64_t row = ib + (v >> 2) * 8 + lhi * 4 + (v & 3);
                    if (row < g.M && col < g.N) {
                        g.acc1[row * g.N + col] = acc[i][j][v];
                        if (g.acc2) g.acc2[row * g.N + col] = acc2[v];
                    }
                }
                continue;
            }
            f32x16 lo;
#pragma unroll
            for (int v = 0; v < 16; ++v) lo[v] = 0.0f;
            for (int pp = 0; pp < g.r; pp += 16) {
                i32x4 th = (i32x4){0, 0, 0, 0}, tl = (i32x4){0, 0, 0, 0}, lb = (i32x4){0, 0, 0, 0};
                if (frag_row < g.M) {
                    th = *reinterpret_cast<const i32x4*>(g.T_hi + frag_row * g.r + pp + lhi * 8);
                    tl = *reinterpret_cast<const i32x4*>(g.T_lo + frag_row * g.r + pp + lhi * 8);
                }
                if (col < g.N) lb = *reinterpret_cast<const i32x4*>(g.L + col * g.r + pp + lhi * 8);
                lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, th),
                                                             __builtin_bit_cast(bf16x8, lb), lo, 0, 0, 0);
                lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tl),
                                                             __builtin_bit_cast(bf16x8, lb), lo, 0, 0, 0);
            }
            if (col < g.N) {
                const float cs = g.col_scale ? g.col_scale[col] : 1.0f;
                const float cs2 = g.K2 > 0 ? g.col_scale2[col] : 0.0f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    int64_t row = ib + (v >> 2) * 8 + lhi * 4 + (v & 3);
                    if (row < g.M) {
                        float inner = __builtin_fmaf((float)acc[i][j][v], cs, (float)acc2[v] * cs2);
                        g.C[row * g.ldc + col] = __builtin_fmaf(g.row_scale[row], inner, lo[v]);
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int BK, int WGM, int WGN>
static hipError_t launch_cfg(const GemmArgs& g, bool dump, hipStream_t stream) {
    int tiles_m = (int)((g.M + BM - 1) / BM), tiles_n = (int)((g.N + BN - 1) / BN);
    size_t lds = 2 * (size_t)(BM + BN) * BK;
    dim3 grid((unsigned)(tiles_m * tiles_n));
    if (dump) {
        auto k = gemm_i8_kernel<BM, BN, BK, WGM, WGN, true>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(256), lds, stream, g, tiles_n);
    } else {
        auto k = gemm_i8_kernel<BM, BN, BK, WGM, WGN, false>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, dim3(256), lds, stream, g, tiles_n);
    }
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& g, bool dump_acc, hipStream_t stream) {
    ProfScope prof(K_GEMM, stream);
    // large tiles when they still give every compute unit work, smaller ones otherwise
    int64_t big_tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big_tiles >= 200) return launch_cfg<256, 256, 64, 2, 2>(g, dump_acc, stream);
    return launch_cfg<128, 128, 64, 2, 2>(g, dump_acc, stream);
}

}  // namespace quaff
