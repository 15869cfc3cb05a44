// Device code of the outlier-column abs-max (Eq. 8 of the paper, max_i |X[i, O_k]|), shared by its stand-alone launch
// and by the launch that runs it next to the LoRA down-projection.
#pragma once
#include "quaff_internal.h"

namespace quaff {

constexpr int kRowsPerSlab = 16;
constexpr int kMaxSlabs = 128;

// part[slab][k] = max over the slab's rows of |X[row, O_k]|; slab s owns row groups s, s + nslab, ...
// Work of workgroup `block` of `nslab` (all NT threads take part); smax is n words of LDS.
template <int NT>
__device__ __forceinline__ void colmax_outlier_body(int block, int nslab, uint32_t* smax, const uint16_t* __restrict__ X,
                                                    int64_t t, int64_t ldx, const int32_t* __restrict__ O, int n,
                                                    uint32_t* __restrict__ part, const float* __restrict__ s_O,
                                                    float* __restrict__ s_prev) {
    for (int k = threadIdx.x; k < n; k += NT) smax[k] = 0u;
    if (block == 0)
        for (int k = threadIdx.x; k < n; k += NT) s_prev[k] = s_O[k];
    __syncthreads();
    const int per_group = kRowsPerSlab * n;
    for (int64_t r0 = (int64_t)block * kRowsPerSlab; r0 < t; r0 += (int64_t)nslab * kRowsPerSlab) {
        for (int e0 = threadIdx.x; e0 < per_group; e0 += 4 * NT) {   // four independent gathers in flight per thread
            uint32_t mag[4];
            int kk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int e = e0 + u * NT;
                int ec = e < per_group ? e : per_group - 1;
                int r = ec / n;
                kk[u] = ec - r * n;
                int64_t row = r0 + r < t ? r0 + r : t - 1;
                mag[u] = ((uint32_t)X[row * ldx + O[kk[u]]] & 0x7FFFu) << 16;   // |x| as fp32 bits
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (e0 + u * NT < per_group) atomicMax(&smax[kk[u]], mag[u]);
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < n; k += NT) part[(int64_t)block * n + k] = smax[k];
}

}  // namespace quaff
