// Device code of the outlier-column abs-max (Eq. 8 of the paper, max_i |X[i, O_k]|), shared by its stand-alone launch
// and by the launch that runs it next to the LoRA down-projection.
#pragma once
#include "quaff_internal.h"

namespace quaff {

constexpr int kRowsPerSlab = 16;
constexpr int kMaxSlabs = 128;

// part[slab][k] = max over the slab's rows of |X[row, O_k]|; slab s owns the 16-row groups s, s + nslab, ...
// Work of workgroup `block` of `nslab` (all NT threads take part).  Sixteen outlier columns are handled per pass:
// thread (slot = tid / 16, kk = tid % 16) walks rows slot, slot + NT / 16, ... of the slab's groups for column kk of the
// pass - sixteen neighbouring lanes read sixteen (often neighbouring) columns of one row - and keeps a running maximum
// in a register, four gathers in flight.  The maxima of a wavefront's four row slots are combined with wavefront
// shuffles and the wavefronts' results through a small LDS array (plain stores, one barrier): no atomics.
// wred is 16 * NT / 64 words of LDS.
template <int NT>
__device__ __forceinline__ void colmax_outlier_body(int block, int nslab, uint32_t* wred, const uint16_t* __restrict__ X,
                                                    int64_t t, int64_t ldx, const int32_t* __restrict__ O, int n,
                                                    uint32_t* __restrict__ part, const float* __restrict__ s_O,
                                                    float* __restrict__ s_prev) {
    constexpr int SLOTS = NT / 16, NWAVE = NT / 64;
    static_assert(SLOTS % kRowsPerSlab == 0, "the row slots of a pass cover whole 16-row groups");
    if (block == 0)
        for (int k = threadIdx.x; k < n; k += NT) s_prev[k] = s_O[k];
    const int kk = threadIdx.x & 15, slot = threadIdx.x >> 4;
    // row of this thread in its first pass over the slab's groups, and the distance between passes: the slab's
    // groups are 16 rows every nslab * 16 rows; the SLOTS row slots of a pass cover SLOTS / 16 of them
    constexpr int GPP = SLOTS / kRowsPerSlab;     // groups per pass
    const int64_t group_stride = (int64_t)nslab * kRowsPerSlab;
    for (int k0 = 0; k0 < n; k0 += 16) {
        const int k = k0 + kk < n ? k0 + kk : n - 1;
        const int64_t col = O[k];
        uint32_t mx = 0;
        const int64_t first = ((int64_t)block + (int64_t)(slot / kRowsPerSlab) * nslab) * kRowsPerSlab + slot % kRowsPerSlab;
        const int64_t step = group_stride * GPP;
        for (int64_t row = first; row < t; row += 4 * step) {
            uint32_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t r = row + u * step;
                v[u] = (uint32_t)X[(r < t ? r : t - 1) * ldx + col] & 0x7FFFu;   // (a repeated row changes no maximum)
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) mx = v[u] > mx ? v[u] : mx;
        }
        // the four row slots of a wavefront, then the wavefronts
        mx = max(mx, (uint32_t)__shfl_xor((int)mx, 16, 64));
        mx = max(mx, (uint32_t)__shfl_xor((int)mx, 32, 64));
        if ((threadIdx.x & 63) < 16) wred[(threadIdx.x >> 6) * 16 + kk] = mx;
        __syncthreads();
        if (threadIdx.x < 16 && k0 + kk < n) {
            uint32_t m = 0;
#pragma unroll
            for (int w = 0; w < NWAVE; ++w) m = max(m, wred[w * 16 + kk]);
            part[(int64_t)block * n + k0 + kk] = m << 16;                              // |x| as fp32 bits
        }
        __syncthreads();
    }
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
