// First launch of the fused forward step: the outlier-column abs-max (Eq. 8) and the LoRA down-projection X A both
// only read X and neither fills the chip, so they share one launch: the first workgroups take the down-projection
// (and the transposed copy of B for the GEMM epilogue), the rest the abs-max slabs.
#include "quaff_lora_body.h"
#include "quaff_scale_body.h"

namespace quaff {

template <int R16, bool L_RC>
__global__ void __launch_bounds__(64 * kLoraWaves)
colmax_lora_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const int32_t* __restrict__ O, int n,
                   uint32_t* __restrict__ part, const float* __restrict__ s_O, float* __restrict__ s_prev, int nslab,
                   const uint16_t* __restrict__ L, float scale, uint16_t* __restrict__ T_hi,
                   uint16_t* __restrict__ T_lo, int row_blocks, int lora_nbx, const uint16_t* __restrict__ tr_src,
                   uint16_t* __restrict__ tr_dst, int64_t tr_rows, int64_t tr_cols) {
    __shared__ uint32_t wred[16 * kLoraWaves];
    const int lora_blocks = lora_nbx * kLoraParts;
    if ((int)blockIdx.x < lora_blocks)
        lora_down_body<R16, L_RC, L_RC ? lora_row_groups(R16) : 1>(blockIdx.x % lora_nbx, blockIdx.x / lora_nbx, lora_nbx, X,
                                                                    t, c, ldx, L, scale, T_hi, T_lo, row_blocks, tr_src,
                                                                    tr_dst, tr_rows, tr_cols);
    else
        colmax_outlier_body<64 * kLoraWaves>(blockIdx.x - lora_blocks, nslab, wred, X, t, ldx, O, n, part, s_O, s_prev);
}

// part [nslab x n] and s_prev as launch_scale_update lays them out; A is [c x r], B [r x c_out] -> Bt [c_out x r]
hipError_t launch_colmax_lora(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const int32_t* O, int32_t n,
                              uint32_t* part, const float* s_O, float* s_prev, int nslab, const uint16_t* A, int32_t r,
                              float scale, uint16_t* T_hi, uint16_t* T_lo, const uint16_t* B, uint16_t* Bt,
                              int64_t c_out, hipStream_t stream, uint16_t* At_scratch) {
    ProfScope prof(K_COLMAX_LORA, stream);
    if (lora_stream_applies(r, t, c, n) && nslab == lora_stream_row_groups(t))
        return launch_lora_stream(X, t, c, ldx, A, false, scale, T_hi, T_lo, B, Bt, (int64_t)r, c_out, O, n, part, s_O,
                                  s_prev, stream);
    const bool transposed = At_scratch && lora_prefers_transposed(r, t);
    if (transposed) {
        hipError_t e = launch_transpose_bf16(A, c, r, At_scratch, stream);
        if (e != hipSuccess) return e;
        A = At_scratch;
    }
    const int rows = transposed ? lora_rows_per_block(r) : 16;        // rows per down-projection workgroup
    const int row_blocks = (int)((t + rows - 1) / rows);
    int64_t b = ((int64_t)r * c_out + 2047) / 2048;
    const int tr_blocks = (int)(b < 128 ? (b > 0 ? b : 1) : 128);
    const int lora_nbx = row_blocks + tr_blocks;
    dim3 grid((unsigned)(lora_nbx * kLoraParts + nslab));
#define QUAFF_CL(N)                                                                                                   \
    case N:                                                                                                           \
        if (transposed)                                                                                               \
            hipLaunchKernelGGL((colmax_lora_kernel<N, true>), grid, dim3(64 * kLoraWaves), 0,      \
                               stream, X, t, (int)c, ldx, O, n, part, s_O, s_prev, nslab, A, scale, T_hi, T_lo,       \
                               row_blocks, lora_nbx, B, Bt, (int64_t)r, c_out);                                       \
        else                                                                                                          \
            hipLaunchKernelGGL((colmax_lora_kernel<N, false>), grid, dim3(64 * kLoraWaves), 0,     \
                               stream, X, t, (int)c, ldx, O, n, part, s_O, s_prev, nslab, A, scale, T_hi, T_lo,       \
                               row_blocks, lora_nbx, B, Bt, (int64_t)r, c_out);                                       \
        break;
    switch (r / 16) {
        QUAFF_CL(1) QUAFF_CL(2) QUAFF_CL(3) QUAFF_CL(4)
    }
#undef QUAFF_CL
    return hipGetLastError();
}

}  // namespace quaff
