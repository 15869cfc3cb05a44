// Fused column scaling and per-token INT8 quantization (Eq. 5 then Eq. 1 of the paper, one step size per token).
//
// HBM-bound: 2 bytes read and 1 byte written per element.  A row is read once into registers (eight bf16 per
// 16-byte load), the row maximum is taken with a wavefront reduction, and the codes leave as packed 8-byte
// stores.  Rows up to 64*8*NV elements are handled by one wavefront (four rows per workgroup); longer rows
// by a whole workgroup; anything longer than that by a two-pass fallback that re-reads the row.
#include "quaff_quant_body.h"

namespace quaff {


// TPR threads cooperate on one row (64 = a wavefront, 256 = the workgroup); each holds NV vectors of 8 elements.
template <int TPR, int NV>
__global__ void __launch_bounds__(256)
quant_rows_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const float* __restrict__ cs,
                  const int32_t* __restrict__ O, int n, int n_pad, int8_t* __restrict__ Xq, float* __restrict__ delta,
                  int8_t* __restrict__ xq_O) {
    quant_rows_body<256, TPR, NV>(blockIdx.x, X, t, c, ldx, cs, O, n, n_pad, Xq, delta, xq_O);
}

// Fallback for very long rows: one workgroup per row, two passes over the row.
__global__ void __launch_bounds__(256)
quant_rows_twopass_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const float* __restrict__ cs,
                          const int32_t* __restrict__ O, int n, int n_pad, int8_t* __restrict__ Xq,
                          float* __restrict__ delta, int8_t* __restrict__ xq_O) {
    __shared__ float red[4];
    const int64_t row = blockIdx.x;
    const uint16_t* xrow = X + row * ldx;
    float m = 0.0f;
    for (int col = threadIdx.x * 8; col < c; col += 256 * 8) {
        float v[8];
        widen_scale(*reinterpret_cast<const u32x4*>(xrow + col), cs, col, v);
#pragma unroll
        for (int u = 0; u < 8; ++u) m = fmaxf(m, fabsf(v[u]));
    }
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float d, cc;
    rtn_steps(m, d, cc);
    if (threadIdx.x == 0) delta[row] = d;
    int8_t* qrow = Xq + row * (int64_t)c;
    for (int col = threadIdx.x * 8; col < c; col += 256 * 8) {
        float v[8];
        widen_scale(*reinterpret_cast<const u32x4*>(xrow + col), cs, col, v);
        *reinterpret_cast<u32x2*>(qrow + col) = pack_codes(v, cc);
    }
    if (xq_O) write_outlier_codes(xrow, cs, O, n, n_pad, cc, xq_O + row * (int64_t)n_pad, threadIdx.x, 256);
}

template <int TPR, int NV>
static void launch_rows(const uint16_t* X, int64_t t, int c, int64_t ldx, const float* cs, const int32_t* O, int n,
                        int n_pad, int8_t* Xq, float* delta, int8_t* xq_O, hipStream_t stream) {
    constexpr int RPB = 256 / TPR;
    hipLaunchKernelGGL((quant_rows_kernel<TPR, NV>), dim3((unsigned)((t + RPB - 1) / RPB)), dim3(256), 0, stream, X, t,
                       c, ldx, cs, O, n, n_pad, Xq, delta, xq_O);
}

hipError_t launch_quant_act(const uint16_t* X, int64_t t, int64_t c64, int64_t ldx, const float* cs, const int32_t* O,
                            int32_t n, int8_t* Xq, float* delta, int8_t* xq_O, hipStream_t stream) {
    ProfScope prof(K_QUANT, stream);
    const int c = (int)c64;
    const int n_pad = (n + kPadK - 1) / kPadK * kPadK;
    const int vec = (c + 7) / 8;   // 16-byte vectors per row
#define QUAFF_ROWS(TPR, NV) launch_rows<TPR, NV>(X, t, c, ldx, cs, O, n, n_pad, Xq, delta, xq_O, stream)
    if (vec <= 64 * 1) QUAFF_ROWS(64, 1);
    else if (vec <= 64 * 2) QUAFF_ROWS(64, 2);
    else if (vec <= 64 * 4) QUAFF_ROWS(64, 4);
    else if (vec <= 64 * 6) QUAFF_ROWS(64, 6);
    else if (vec <= 64 * 8) QUAFF_ROWS(64, 8);
    else if (vec <= 256 * 3) QUAFF_ROWS(256, 3);
    else if (vec <= 256 * 4) QUAFF_ROWS(256, 4);
    else if (vec <= 256 * 6) QUAFF_ROWS(256, 6);
    else if (vec <= 256 * 8) QUAFF_ROWS(256, 8);
    else
        hipLaunchKernelGGL(quant_rows_twopass_kernel, dim3((unsigned)t), dim3(256), 0, stream, X, t, c, ldx, cs, O, n,
                           n_pad, Xq, delta, xq_O);
#undef QUAFF_ROWS
    return hipGetLastError();
}

}  // namespace quaff
