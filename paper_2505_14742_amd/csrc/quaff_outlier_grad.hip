// Full-precision input gradient on the outlier channels.  The paper keeps the outlier rows W_O of the frozen weight
// in full precision (Sec. 3.3) and the scaling factors cancel in the true gradient (Eq. 3), so for k in O
//     dX[i, O_k] = sum_j dY[i, j] W_O[k, j] + scale * sum_p (sum_j dY[i, j] B[p, j]) A[O_k, p]
// can replace the quantized product on exactly the columns where quantization error concentrates.  Both terms are
// one skinny product of dY with the effective rows  Weff[k, :] = W_O[k, :] + scale * A[O_k, :] B  (fp32), taken
// with the LoRA down-projection kernel on a bf16 hi/lo split of Weff (32 outlier channels per pass: rows 0..31 of the
// stacked factor hold the hi halves, rows 32..63 the lo halves), followed by a scatter into dX.
#include "quaff_internal.h"

namespace quaff {

__device__ __forceinline__ uint32_t og_f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// L [64 x c_out] bf16 for the group of outliers g0 .. g0 + 31 (rows past n are zero)
__global__ void __launch_bounds__(256)
outlier_weff_kernel(const float* __restrict__ W_O, const int32_t* __restrict__ O, int n, int g0, int64_t c_out,
                    const uint16_t* __restrict__ lora_A, const uint16_t* __restrict__ lora_B, int r, float scale,
                    uint16_t* __restrict__ L) {
    const int kk = blockIdx.y;                         // 0..31
    const int k = g0 + kk;
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < c_out; j += (int64_t)gridDim.x * 256) {
        float w = 0.0f;
        if (k < n) {
            float l = 0.0f;
            const uint16_t* a = lora_A + (int64_t)O[k] * r;
            for (int p = 0; p < r; ++p)
                l = __builtin_fmaf(bf16_bits_to_f32(a[p]), bf16_bits_to_f32(lora_B[(int64_t)p * c_out + j]), l);
            w = __builtin_fmaf(scale, l, W_O[(int64_t)k * c_out + j]);
        }
        const uint32_t hi = og_f32_to_bf16_rne(w);
        L[(int64_t)kk * c_out + j] = (uint16_t)hi;
        L[(int64_t)(32 + kk) * c_out + j] = (uint16_t)og_f32_to_bf16_rne(w - __uint_as_float(hi << 16));
    }
}

// dX[i, O_k] = sum over parts and hi/lo of T[i, kk] + T[i, 32 + kk],  k = g0 + kk
__global__ void __launch_bounds__(256)
outlier_scatter_kernel(const uint16_t* __restrict__ T_hi, const uint16_t* __restrict__ T_lo, int64_t t,
                       const int32_t* __restrict__ O, int n, int g0, float* __restrict__ dX, int64_t lddx) {
    const int64_t total = t * 32;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t i = e >> 5;
        const int kk = (int)(e & 31), k = g0 + kk;
        if (k >= n) continue;
        float v = 0.0f;
#pragma unroll
        for (int part = 0; part < kLoraParts; ++part) {
            const int64_t o = ((int64_t)part * t + i) * 64;
            v += bf16_bits_to_f32(T_hi[o + kk]) + bf16_bits_to_f32(T_lo[o + kk]);
            v += bf16_bits_to_f32(T_hi[o + 32 + kk]) + bf16_bits_to_f32(T_lo[o + 32 + kk]);
        }
        dX[i * lddx + O[k]] = v;
    }
}

hipError_t launch_outlier_grad(const uint16_t* dY, int64_t t, int64_t lddy, int64_t c_out, const int32_t* O, int32_t n,
                               const float* W_O, const uint16_t* lora_A, const uint16_t* lora_B, int32_t r, float scale,
                               float* dX, int64_t lddx, uint16_t* L, uint16_t* T_hi, uint16_t* T_lo,
                               hipStream_t stream) {
    for (int g0 = 0; g0 < n; g0 += 32) {
        {
            ProfScope prof(K_OUTLIER_GRAD, stream);
            int64_t bx = (c_out + 255) / 256;
            hipLaunchKernelGGL(outlier_weff_kernel, dim3((unsigned)(bx < 64 ? bx : 64), 32), dim3(256), 0, stream, W_O,
                               O, n, g0, c_out, lora_A, lora_B, r, scale, L);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        hipError_t e = launch_lora_down(dY, t, c_out, lddy, L, true, 64, 1.0f, T_hi, T_lo, nullptr, nullptr, 0, 0, stream);
        if (e != hipSuccess) return e;
        ProfScope prof(K_OUTLIER_GRAD, stream);
        int64_t blocks = (t * 32 + 255) / 256;
        hipLaunchKernelGGL(outlier_scatter_kernel, dim3((unsigned)(blocks < 2048 ? blocks : 2048)), dim3(256), 0, stream,
                           T_hi, T_lo, t, O, n, g0, dX, lddx);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace quaff
