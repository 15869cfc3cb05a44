// Second launch of the fused forward step.  The per-token quantizer of X needs the new scaling factors only on the
// outlier columns, and those follow from the abs-max slabs by a few hundred flops (Eq. 8, Eq. 7): instead of
// waiting for a launch that publishes them, every quantizing workgroup derives them itself while its row loads are
// in flight, into an LDS copy of the column scales.  The requantization of what = (s_O - 1) W_O (Eq. 5, Eq. 9) runs
// in the first workgroups of the same launch; workgroup 0 publishes s, 1/s and cmax exactly as the stand-alone
// kernel does.  Both roles evaluate the same device function, so the factors agree bit for bit.
#include "quaff_quant_body.h"
#include "quaff_scale_body.h"

namespace quaff {

constexpr int kWqBatch = 16;   // partial maxima per thread and round trip: 256 x 16 = 4096 cover the usual slab counts

template <int TPR, int NV>
__global__ void __launch_bounds__(256)
what_quant_kernel(const uint32_t* __restrict__ part, int nslab, int n, int n_pad, const float* __restrict__ wmax_O,
                  const float* __restrict__ s_prev, float gamma, const int32_t* __restrict__ O, float* __restrict__ s_O,
                  float* colscale, float* __restrict__ cmax_out, const float* __restrict__ W_O, int64_t c_out,
                  int8_t* __restrict__ what_int, float* __restrict__ delta_what, int what_blocks,
                  const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, int8_t* __restrict__ Xq,
                  float* __restrict__ delta, int8_t* __restrict__ xq_O) {
    extern __shared__ float dyn[];
    if ((int)blockIdx.x < what_blocks) {
        momentum_what_body<256, kWqBatch>(blockIdx.x, dyn, part, nslab, n, n_pad, wmax_O, s_prev, gamma, O, s_O, colscale,
                                          cmax_out, W_O, c_out, what_int, delta_what);
        return;
    }
    // quantizing workgroup: dyn = column scales [c], then n words for the reduction of the slabs
    auto prologue = [&]() {
        typedef float f32x4_ __attribute__((ext_vector_type(4)));
        uint32_t* smax = reinterpret_cast<uint32_t*>(dyn + c);
        for (int k = threadIdx.x; k < n; k += 256) smax[k] = 0u;
        // the caller's column scales (1 outside O by contract, but copied rather than assumed)
        for (int i = threadIdx.x * 4; i < c; i += 1024)
            *reinterpret_cast<f32x4_*>(dyn + i) = *reinterpret_cast<const f32x4_*>(colscale + i);
        __syncthreads();
        const int total = nslab * n;
        for (int e0 = threadIdx.x; e0 < total; e0 += kWqBatch * 256) {
            uint32_t v[kWqBatch];
#pragma unroll
            for (int u = 0; u < kWqBatch; ++u) {
                int e = e0 + u * 256;
                v[u] = part[e < total ? e : total - 1];
            }
#pragma unroll
            for (int u = 0; u < kWqBatch; ++u) {
                int e = e0 + u * 256;
                if (e < total) atomicMax(&smax[e % n], v[u]);
            }
        }
        __syncthreads();
        for (int k = threadIdx.x; k < n; k += 256) {
            float s = momentum_scale(__uint_as_float(smax[k]), wmax_O[k], s_prev[k], gamma);
            dyn[O[k]] = __fdiv_rn(1.0f, s);
        }
        __syncthreads();
    };
    quant_rows_body<256, TPR, NV, const lds_float*, decltype(prologue)>(
        blockIdx.x - what_blocks, X, t, c, ldx, (const lds_float*)dyn, O, n, n_pad, Xq, delta, xq_O, prologue);
}

template <int TPR, int NV>
static void launch_wq(dim3 grid, size_t lds, hipStream_t stream, const uint32_t* part, int nslab, int n, int n_pad,
                      const float* wmax_O, const float* s_prev, float gamma, const int32_t* O, float* s_O,
                      float* colscale, float* cmax_out, const float* W_O, int64_t c_out, int8_t* what_int,
                      float* delta_what, int what_blocks, const uint16_t* X, int64_t t, int c, int64_t ldx, int8_t* Xq,
                      float* delta, int8_t* xq_O) {
    hipLaunchKernelGGL((what_quant_kernel<TPR, NV>), grid, dim3(256), lds, stream, part, nslab, n, n_pad, wmax_O, s_prev,
                       gamma, O, s_O, colscale, cmax_out, W_O, c_out, what_int, delta_what, what_blocks, X, t, c, ldx,
                       Xq, delta, xq_O);
}

// Returns false (nothing enqueued) for shapes this launch does not cover.
bool launch_what_quant(const uint32_t* part, int nslab, int32_t n, const float* wmax_O, const float* s_prev, float gamma,
                       const int32_t* O, float* s_O, float* colscale, float* cmax_out, const float* W_O, int64_t c_out,
                       int8_t* what_int, float* delta_what, const uint16_t* X, int64_t t, int64_t c64, int64_t ldx,
                       int8_t* Xq, float* delta, int8_t* xq_O, hipStream_t stream, hipError_t* err) {
    const int c = (int)c64;
    const int vec = (c + 7) / 8;
    const size_t lds = ((size_t)c + 2 * (size_t)n) * sizeof(float);
    if (n < 1 || n > 64 || vec > 256 * 8 || lds > 64 * 1024) return false;
    ProfScope prof(K_WHAT_QUANT, stream);
    const int n_pad = (n + kPadK - 1) / kPadK * kPadK;
    const int what_blocks = (int)((c_out + 255) / 256);
#define QUAFF_WQ(TPR, NV)                                                                                              \
    launch_wq<TPR, NV>(dim3((unsigned)(what_blocks + (t + 256 / TPR - 1) / (256 / TPR))), lds, stream, part, nslab, n,  \
                       n_pad, wmax_O, s_prev, gamma, O, s_O, colscale, cmax_out, W_O, c_out, what_int, delta_what,      \
                       what_blocks, X, t, c, ldx, Xq, delta, xq_O)
    if (vec <= 64 * 1) QUAFF_WQ(64, 1);
    else if (vec <= 64 * 2) QUAFF_WQ(64, 2);
    else if (vec <= 64 * 4) QUAFF_WQ(64, 4);
    else if (vec <= 64 * 6) QUAFF_WQ(64, 6);
    else if (vec <= 64 * 8) QUAFF_WQ(64, 8);
    else if (vec <= 256 * 3) QUAFF_WQ(256, 3);
    else if (vec <= 256 * 4) QUAFF_WQ(256, 4);
    else if (vec <= 256 * 6) QUAFF_WQ(256, 6);
    else QUAFF_WQ(256, 8);
#undef QUAFF_WQ
    *err = hipGetLastError();
    return true;
}

}  // namespace quaff
