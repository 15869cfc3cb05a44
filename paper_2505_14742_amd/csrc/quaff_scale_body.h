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

// Eq. 7 with Eq. 8 for one outlier channel, in fp32 with one rounding per operation
__device__ __forceinline__ float momentum_scale(float cmax, float wmax, float s_prev, float gamma) {
    float beta = 1.0f;
    if (wmax > 0.0f) beta = fmaxf(1.0f, __builtin_sqrtf(__fdiv_rn(cmax, wmax)));                 // Eq. 8
    return __fadd_rn(__fmul_rn(gamma, s_prev), __fmul_rn(__fsub_rn(1.0f, gamma), beta));       // Eq. 7
}

// Work of workgroup `block` (NT threads, one output channel of what each): reduce the partial maxima, evaluate
// Eq. 8 / Eq. 7 for all outlier channels (workgroup 0 publishes s, 1/s and cmax), requantize what.  sm1 is 2 n words
// of LDS; PB partial maxima are loaded per thread before the first is used.
template <int NT, int PB>
__device__ __forceinline__ void momentum_what_body(int block, float* sm1, const uint32_t* __restrict__ part, int nslab,
                                                   int n, int n_pad, const float* __restrict__ wmax_O,
                                                   const float* __restrict__ s_prev, float gamma,
                                                   const int32_t* __restrict__ O, float* __restrict__ s_O,
                                                   float* __restrict__ colscale, float* __restrict__ cmax_out,
                                                   const float* __restrict__ W_O, int64_t c_out,
                                                   int8_t* __restrict__ what_int, float* __restrict__ delta_what) {
    uint32_t* smax = reinterpret_cast<uint32_t*>(sm1 + n);         // [n]
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int64_t j = (int64_t)block * NT + threadIdx.x;
    const int64_t jc = j < c_out ? j : c_out - 1;
    const bool small = n <= 64;
    // Every global load that does not depend on the reduction is issued first, so that the kernel pays about one
    // memory round trip instead of three: this thread's column of W_O (n <= 64: kept in registers), its share of the
    // partial maxima, and the per-outlier constants.
    float w[64];
    if (small) {
#pragma unroll
        for (int k = 0; k < 64; ++k) w[k] = W_O[(int64_t)(k < n ? k : n - 1) * c_out + jc];
    }
    const int kk = threadIdx.x < n ? threadIdx.x : n - 1;          // outlier handled by this thread (first pass)
    const float wmax0 = wmax_O[kk], sprev0 = s_prev[kk];
    const int o0 = O[kk];
    for (int k = threadIdx.x; k < n; k += NT) smax[k] = 0u;
    __syncthreads();
    const int total = nslab * n;
    for (int e0 = threadIdx.x; e0 < total; e0 += PB * NT) {   // one round trip for up to 4096 partials
        uint32_t v[PB];
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            int e = e0 + u * NT;
            v[u] = part[e < total ? e : total - 1];
        }
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            int e = e0 + u * NT;
            if (e < total) atomicMax(&smax[e % n], v[u]);
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < n; k += NT) {
        const bool first = k == (int)threadIdx.x;
        float cmax = __uint_as_float(smax[k]);
        float s = momentum_scale(cmax, first ? wmax0 : wmax_O[k], first ? sprev0 : s_prev[k], gamma);
        sm1[k] = __fsub_rn(s, 1.0f);
        if (block == 0) {
            s_O[k] = s;
            colscale[first ? o0 : O[k]] = __fdiv_rn(1.0f, s);
            if (cmax_out) cmax_out[k] = cmax;
        }
    }
    __syncthreads();
    if (j >= c_out) return;
    // what[k, j] for this output channel (Eq. 5), quantized per output channel (Eq. 1)
    u32x4* dst = reinterpret_cast<u32x4*>(what_int + j * n_pad);
    float d, c;
    if (small) {
        float m = 0.0f;
#pragma unroll
        for (int k = 0; k < 64; ++k) {
            w[k] = k < n ? __fmul_rn(sm1[k < n ? k : n - 1], w[k]) : 0.0f;
            m = fmaxf(m, fabsf(w[k]));
        }
        rtn_steps(m, d, c);
#pragma unroll
        for (int k16 = 0; k16 < 64; k16 += 16) {
            u32x4 q4 = (u32x4){0, 0, 0, 0};
#pragma unroll
            for (int u = 0; u < 16; ++u) q4[u >> 2] |= (uint32_t)(rtn_code(w[k16 + u], c) & 0xFF) << (8 * (u & 3));
            dst[k16 >> 4] = q4;
        }
    } else {
        float m = 0.0f;
        for (int k = 0; k < n; ++k) m = fmaxf(m, fabsf(__fmul_rn(sm1[k], W_O[(int64_t)k * c_out + j])));
        rtn_steps(m, d, c);
        for (int k16 = 0; k16 < n_pad; k16 += 16) {
            u32x4 q4 = (u32x4){0, 0, 0, 0};
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                int k = k16 + u;
                int q = 0;
                if (k < n) q = rtn_code(__fmul_rn(sm1[k], W_O[(int64_t)k * c_out + j]), c);
                q4[u >> 2] |= (uint32_t)(q & 0xFF) << (8 * (u & 3));
            }
            dst[k16 >> 4] = q4;
        }
    }
    delta_what[j] = d;
}

}  // namespace quaff
