// Offline weight preprocessing (Sec. 3.3 of the paper, first paragraph): per-output-channel Eq. 1 on the
// frozen W, the packed copy of the codes (one byte per weight, read by both products), and the retained
// full-precision rows W_O.
// Runs once per layer and is not on the per-step path, so it is written for clarity.
#include "quaff_internal.h"

namespace quaff {

constexpr int kSlab = 64;   // rows of W per partial column maximum

__global__ void __launch_bounds__(256)
colmax_partial_kernel(const float* __restrict__ W, int64_t c_in, int64_t c_out, int64_t ldw, float* __restrict__ part) {
    int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= c_out) return;
    int64_t k0 = (int64_t)blockIdx.y * kSlab;
    int64_t k1 = k0 + kSlab < c_in ? k0 + kSlab : c_in;
    float m = 0.0f;
    for (int64_t k = k0; k < k1; ++k) m = fmaxf(m, fabsf(W[k * ldw + j]));
    part[(int64_t)blockIdx.y * c_out + j] = m;
}

__global__ void __launch_bounds__(256)
colmax_final_kernel(const float* __restrict__ part, int nslab, int64_t c_out, float* __restrict__ delta_w,
                    float* __restrict__ recip) {
    int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= c_out) return;
    float m = 0.0f;
    for (int s = 0; s < nslab; ++s) m = fmaxf(m, part[(int64_t)s * c_out + j]);
    float d, c;
    rtn_steps(m, d, c);
    delta_w[j] = d;
    recip[j] = c;
}

__global__ void __launch_bounds__(256)
weight_codes_kernel(const float* __restrict__ W, int64_t c_in, int64_t c_out, int64_t ldw,
                    const float* __restrict__ recip, int8_t* __restrict__ Wp, int64_t cpad,
                    int8_t* __restrict__ Wq_plain) {
    int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= c_out) return;
    float c = recip[j];
    for (int64_t k = blockIdx.y; k < c_in; k += gridDim.y) {
        int8_t q = (int8_t)rtn_code(W[k * ldw + j], c);
        Wp[weight_code_offset(j, k, cpad)] = q;
        if (Wq_plain) Wq_plain[k * c_out + j] = q;
    }
}

__global__ void __launch_bounds__(256)
outlier_rows_kernel(const float* __restrict__ W, int64_t c_out, int64_t ldw, const int32_t* __restrict__ O,
                    float* __restrict__ W_O, float* __restrict__ wmax_O) {
    __shared__ float red[4];
    int k = blockIdx.x;
    const float* src = W + (int64_t)O[k] * ldw;
    float m = 0.0f;
    for (int64_t j = threadIdx.x; j < c_out; j += 256) {
        float w = src[j];
        W_O[(int64_t)k * c_out + j] = w;
        m = fmaxf(m, fabsf(w));
    }
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) wmax_O[k] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

hipError_t launch_prepare_weight(const float* W, int64_t c_in, int64_t c_out, int64_t ldw, const int32_t* O, int32_t n,
                                 int8_t* Wp, float* delta_w, float* W_O, float* wmax_O, int8_t* Wq_plain,
                                 float* ws, hipStream_t stream) {
    ProfScope prof(K_PREPARE, stream);
    int nslab = (int)((c_in + kSlab - 1) / kSlab);
    float* part = ws;                               // [nslab x c_out]
    float* recip = ws + (int64_t)nslab * c_out;     // [c_out]
    dim3 gx((unsigned)((c_out + 255) / 256));
    hipLaunchKernelGGL(colmax_partial_kernel, dim3(gx.x, nslab), dim3(256), 0, stream, W, c_in, c_out, ldw, part);   // nslab <= 65535 is checked by the caller
    hipLaunchKernelGGL(colmax_final_kernel, gx, dim3(256), 0, stream, part, nslab, c_out, delta_w, recip);
    hipLaunchKernelGGL(weight_codes_kernel, dim3(gx.x, (unsigned)(c_in < 65535 ? c_in : 65535)), dim3(256), 0, stream, W, c_in, c_out, ldw,
                       recip, Wp, packed_weight_cpad(c_in), Wq_plain);
    if (n > 0)
        hipLaunchKernelGGL(outlier_rows_kernel, dim3(n), dim3(256), 0, stream, W, c_out, ldw, O, W_O, wmax_O);
    return hipGetLastError();
}

}  // namespace quaff
