// LoRA down-projection for the adapter branch of the quantized linear layer (rank r, no dropout; the paper's
// App. "Model and experimental settings"):  T = scale * X L  with X [t x c] bf16 and L the rank-r factor.
// Forward: X is the layer input and L = A [c_in x r].  Backward: X is dY and L = B^T, given as B [r x c_out].
//
// HBM-bound skinny product (reads X once).  bf16 MFMA 16x16x32 with fp32 accumulation; a workgroup owns 16 rows,
// its eight wavefronts take interleaved 32-wide contraction steps and are summed in a fixed order, so the result
// is deterministic.  When L is stored [c x r] the MFMA needs it transposed: each wavefront stages its own
// 32 x r slice through a private piece of LDS (coalesced 16-byte loads in, 2-byte scatter, 16-byte fragment out).
// T is handed to the GEMM epilogue as a bf16 pair (hi + lo, 16 significant bits) so that the up-projection can
// also run on the bf16 MFMA without losing the fp32 accumulation's accuracy.  Extra workgroups of the same launch
// write the transposed copy of the other factor that the epilogue reads contraction-contiguous.
#include "quaff_lora_body.h"

namespace quaff {

// R16 = r / 16 column blocks of T.  L_RC: L is [r x c] (contraction-contiguous) else [c x r].
// Up to r = 32 the kernel is held to 64 registers (8 wavefronts per SIMD): its 16-wavefront workgroups then fit on
// a compute unit beside a workgroup of the input-gradient product, which the one-call backward step runs them next to.
template <int R16, bool L_RC>
__global__ void __launch_bounds__(64 * kLoraWaves, R16 <= 2 ? 8 : 4)
lora_down_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const uint16_t* __restrict__ L,
                 float scale, uint16_t* __restrict__ T_hi, uint16_t* __restrict__ T_lo, int row_blocks,
                 const uint16_t* __restrict__ tr_src, uint16_t* __restrict__ tr_dst, int64_t tr_rows, int64_t tr_cols) {
    lora_down_body<R16, L_RC, L_RC ? lora_row_groups(R16) : 1>(blockIdx.x, blockIdx.y, gridDim.x, X, t, c, ldx, L, scale,
                                                                T_hi, T_lo, row_blocks, tr_src, tr_dst, tr_rows, tr_cols);
}

// Two rank-16 down-projections of matrices with the same number of rows in one launch: blockIdx.z = 0 multiplies X0 by
// a contraction-contiguous factor L0 [r x c0], blockIdx.z = 1 multiplies X1 by L1 [c1 x r].
struct LoraPairArgs {
    const uint16_t* X[2]; int c[2]; int64_t ldx[2]; const uint16_t* L[2]; uint16_t* T_hi[2]; uint16_t* T_lo[2];
    int64_t t; float scale; int row_blocks;
};
__global__ void __launch_bounds__(64 * kLoraWaves, 8)
lora_down_pair_kernel(LoraPairArgs a) {
    if (blockIdx.z == 0)
        lora_down_body<1, true>(blockIdx.x, blockIdx.y, gridDim.x, a.X[0], a.t, a.c[0], a.ldx[0], a.L[0], a.scale, a.T_hi[0],
                                a.T_lo[0], a.row_blocks, nullptr, nullptr, 0, 0);
    else
        lora_down_body<1, false>(blockIdx.x, blockIdx.y, gridDim.x, a.X[1], a.t, a.c[1], a.ldx[1], a.L[1], a.scale, a.T_hi[1],
                                 a.T_lo[1], a.row_blocks, nullptr, nullptr, 0, 0);
}

template <bool L_RC>
static void dispatch(int R16, dim3 grid, hipStream_t stream, const uint16_t* X, int64_t t, int c, int64_t ldx,
                     const uint16_t* L, float scale, uint16_t* T_hi, uint16_t* T_lo, int row_blocks,
                     const uint16_t* tr_src, uint16_t* tr_dst, int64_t tr_rows, int64_t tr_cols) {
#define QUAFF_LORA(N)                                                                                              \
    case N:                                                                                                        \
        hipLaunchKernelGGL((lora_down_kernel<N, L_RC>), grid, dim3(64 * kLoraWaves), 0, stream, X, t, c, ldx, L,   \
                           scale, T_hi, T_lo, row_blocks, tr_src, tr_dst, tr_rows, tr_cols);                       \
        break;
    switch (R16) {
        QUAFF_LORA(1) QUAFF_LORA(2) QUAFF_LORA(3) QUAFF_LORA(4)
    }
#undef QUAFF_LORA
}

// dst [cols x rows] <- src [rows x cols] (bf16), consecutive threads write consecutive addresses
__global__ void __launch_bounds__(256)
transpose_bf16_kernel(const uint16_t* __restrict__ src, int64_t rows, int64_t cols, uint16_t* __restrict__ dst) {
    const int64_t total = rows * cols;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t col = e / rows, row = e % rows;
        dst[e] = src[row * cols + col];
    }
}

hipError_t launch_transpose_bf16(const uint16_t* src, int64_t rows, int64_t cols, uint16_t* dst, hipStream_t stream) {
    int64_t blocks = (rows * cols + 255) / 256;
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)(blocks < 1024 ? blocks : 1024)), dim3(256), 0, stream, src,
                       rows, cols, dst);
    return hipGetLastError();
}

hipError_t launch_lora_down(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const uint16_t* L, bool L_is_r_by_c,
                            int32_t r, float scale, uint16_t* T_hi, uint16_t* T_lo, const uint16_t* tr_src,
                            uint16_t* tr_dst, int64_t tr_rows, int64_t tr_cols, hipStream_t stream,
                            uint16_t* Lt_scratch) {
    ProfScope prof(K_LORA, stream);
    if (lora_stream_applies(r, t, c, 0))
        return launch_lora_stream(X, t, c, ldx, L, L_is_r_by_c, scale, T_hi, T_lo, tr_src, tr_dst, tr_rows, tr_cols,
                                  nullptr, 0, nullptr, nullptr, nullptr, stream);
    if (!L_is_r_by_c && Lt_scratch && lora_prefers_transposed(r, t)) {
        // a [c x r] factor of rank 32 or more is transposed once (r x c, contraction-contiguous) instead of slice by
        // slice through LDS inside the product: one small launch more, a several times faster product
        hipError_t e = launch_transpose_bf16(L, c, r, Lt_scratch, stream);
        if (e != hipSuccess) return e;
        L = Lt_scratch;
        L_is_r_by_c = true;
    }
    const int rows = L_is_r_by_c ? lora_rows_per_block(r) : 16;      // rows per workgroup
    int row_blocks = (int)((t + rows - 1) / rows);
    int tr_blocks = 0;
    if (tr_src) {
        int64_t b = (tr_rows * tr_cols + 2047) / 2048;
        tr_blocks = (int)(b < 128 ? (b > 0 ? b : 1) : 128);
    }
    dim3 grid(row_blocks + tr_blocks, kLoraParts);
    if (L_is_r_by_c)
        dispatch<true>(r / 16, grid, stream, X, t, (int)c, ldx, L, scale, T_hi, T_lo, row_blocks, tr_src, tr_dst,
                       tr_rows, tr_cols);
    else
        dispatch<false>(r / 16, grid, stream, X, t, (int)c, ldx, L, scale, T_hi, T_lo, row_blocks, tr_src, tr_dst,
                        tr_rows, tr_cols);
    return hipGetLastError();
}

hipError_t launch_lora_down_pair(const uint16_t* dY, int64_t lddy, int64_t c_out, const uint16_t* B, uint16_t* T1_hi,
                                 uint16_t* T1_lo, const uint16_t* X, int64_t ldx, int64_t c_in, const uint16_t* A,
                                 uint16_t* T2_hi, uint16_t* T2_lo, int64_t t, int32_t r, float scale,
                                 uint16_t* At_scratch, hipStream_t stream) {
    if (r != 16 || lora_stream_applies(r, t, c_out, 0) || lora_stream_applies(r, t, c_in, 0)) {
        hipError_t e = launch_lora_down(dY, t, c_out, lddy, B, true, r, scale, T1_hi, T1_lo, nullptr, nullptr, 0, 0,
                                        stream);
        if (e != hipSuccess) return e;
        return launch_lora_down(X, t, c_in, ldx, A, false, r, scale, T2_hi, T2_lo, nullptr, nullptr, 0, 0, stream,
                                At_scratch);
    }
    ProfScope prof(K_LORA, stream);
    const int row_blocks = (int)((t + 15) / 16);
    LoraPairArgs a{{dY, X}, {(int)c_out, (int)c_in}, {lddy, ldx}, {B, A}, {T1_hi, T2_hi}, {T1_lo, T2_lo},
                   t, scale, row_blocks};
    hipLaunchKernelGGL(lora_down_pair_kernel, dim3(row_blocks, kLoraParts, 2), dim3(64 * kLoraWaves), 0, stream, a);
    return hipGetLastError();
}

}  // namespace quaff
