// Targeted momentum scaling (Eq. 7, Eq. 8 of the paper) and the dynamic outlier weights
// what = (s_O - 1) W_O with their per-output-channel quantization (Eq. 5, Eq. 9).
//
// Two launches:
//   colmax_outlier_kernel   partial column maxima of |X[:, O]| per slab of rows (a strided 2-byte gather: the
//                           traffic is one DRAM sector per (row, outlier) whatever the kernel does; register maxima
//                           combined with wavefront shuffles), and a copy
//                           of the previous scales so that the in-place update below has no read/write race;
//   momentum_what_kernel    every block reduces the partial maxima and evaluates Eq. 8 / Eq. 7 for all outlier
//                           channels (a few hundred flops, cheaper than another launch); block 0 publishes s,
//                           1/s and cmax; then each thread requantizes one output channel of what.
// Maxima of non-negative floats are taken on their bit patterns (same order as unsigned integers), which is exact
// and independent of the order in which they are combined.
#include "quaff_scale_body.h"
#include <mutex>

namespace quaff {

// Scratch of quaff_scale_update_static (callers that cannot allocate): the partial column maxima [slabs x n] and the
// copy of the previous scales [n] that the workspace of quaff_scale_update otherwise holds.  One copy per device, held
// until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the
// address that call returns.
constexpr int kStaticMaxOutliers = 1024;
static __device__ __align__(256) __attribute__((used)) float scratch[(size_t)(kMaxSlabs + 1) * kStaticMaxOutliers];

int scale_update_static_max_outliers() { return kStaticMaxOutliers; }

hipError_t scale_update_static_scratch(float** ptr) {
    static std::mutex mu;
    static float* per_device[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!per_device[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // this device's copy of the array
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = static_cast<float*>(p);
    }
    *ptr = per_device[dev];
    return hipSuccess;
}

constexpr int kWhatThreads = 128;   // output channels per workgroup of momentum_what_kernel
constexpr int kPartBatch = 32;     // partial maxima loaded per thread before the first is used

int scale_update_blocks(int64_t t) {
    int64_t b = (t + kRowsPerSlab - 1) / kRowsPerSlab;
    return (int)(b < kMaxSlabs ? b : kMaxSlabs);
}

__global__ void __launch_bounds__(256)
colmax_outlier_kernel(const uint16_t* __restrict__ X, int64_t t, int64_t ldx, const int32_t* __restrict__ O, int n,
                      uint32_t* __restrict__ part, const float* __restrict__ s_O, float* __restrict__ s_prev) {
    __shared__ uint32_t wred[16 * 256 / 64];
    colmax_outlier_body<256>(blockIdx.x, gridDim.x, wred, X, t, ldx, O, n, part, s_O, s_prev);
}

__global__ void __launch_bounds__(kWhatThreads)
momentum_what_kernel(const uint32_t* __restrict__ part, int nslab, int n, int n_pad, const float* __restrict__ wmax_O,
                     const float* __restrict__ s_prev, float gamma, const int32_t* __restrict__ O,
                     float* __restrict__ s_O, float* __restrict__ colscale, float* __restrict__ cmax_out,
                     const float* __restrict__ W_O, int64_t c_out, int8_t* __restrict__ what_int,
                     float* __restrict__ delta_what) {
    extern __shared__ float sm1[];                                  // [n] : s_k - 1, then [n] maxima
    momentum_what_body<kWhatThreads, kPartBatch>(blockIdx.x, sm1, part, nslab, n, n_pad, wmax_O, s_prev, gamma, O, s_O,
                                                 colscale, cmax_out, W_O, c_out, what_int, delta_what);
}

// Dense variant of the column abs-max for outlier sets that touch most 64-byte segments of a row anyway (the
// paper's 4 % - 10 % budgets): every column of a 2048-column chunk is reduced over the slab's rows with coalesced
// 16-byte loads (bf16 magnitudes compare as integers), then the chunk's outlier columns are picked out of LDS.
__global__ void __launch_bounds__(256)
colmax_dense_kernel(const uint16_t* __restrict__ X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* __restrict__ O,
                    int n, uint32_t* __restrict__ part, const float* __restrict__ s_O, float* __restrict__ s_prev,
                    int rows_per_slab) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    __shared__ uint16_t cm[2048];
    __shared__ int krange[2];
    const int chunk0 = blockIdx.x * 2048, slab = blockIdx.y;
    if (blockIdx.x == 0 && slab == 0)
        for (int k = threadIdx.x; k < n; k += 256) s_prev[k] = s_O[k];
    if (threadIdx.x < 2) {
        // first outlier index >= chunk0 (thread 0) and >= chunk0 + 2048 (thread 1): O is sorted
        const int target = chunk0 + 2048 * (int)threadIdx.x;
        int lo = 0, hi = n;
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (O[mid] < target) lo = mid + 1; else hi = mid;
        }
        krange[threadIdx.x] = lo;
    }
    const int64_t col = chunk0 + (int64_t)threadIdx.x * 8;
    const int64_t r0 = (int64_t)slab * rows_per_slab;
    const int64_t r1 = r0 + rows_per_slab < t ? r0 + rows_per_slab : t;
    uint32_t mx[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col < c_in) {
        const uint16_t* src = X + col;
        for (int64_t row = r0; row < r1; row += 4) {   // four independent loads in flight
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int64_t rr = row + u < r1 ? row + u : r1 - 1;
                v[u] = *reinterpret_cast<const u32x4*>(src + rr * ldx);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int w = 0; w < 4; ++w) {     // a repeated row changes no maximum
                    uint32_t lo = v[u][w] & 0x7FFFu, hi = (v[u][w] >> 16) & 0x7FFFu;
                    mx[2 * w] = lo > mx[2 * w] ? lo : mx[2 * w];
                    mx[2 * w + 1] = hi > mx[2 * w + 1] ? hi : mx[2 * w + 1];
                }
        }
    }
#pragma unroll
    for (int w = 0; w < 8; ++w) cm[threadIdx.x * 8 + w] = (uint16_t)mx[w];
    __syncthreads();
    for (int k = krange[0] + threadIdx.x; k < krange[1]; k += 256)
        part[(int64_t)slab * n + k] = (uint32_t)cm[O[k] - chunk0] << 16;   // |x| as fp32 bits
}

// momentum_what_kernel for more than 64 outlier channels: a workgroup owns 32 output channels and its 16 thread
// groups split the outlier range, so that the n x c_out read of W_O is spread over enough workgroups.
constexpr int kWideCh = 32, kWideGroups = 16;
__global__ void __launch_bounds__(kWideCh * kWideGroups)
momentum_what_wide_kernel(const uint32_t* __restrict__ part, int nslab, int n, int n_pad,
                          const float* __restrict__ wmax_O, const float* __restrict__ s_prev, float gamma,
                          const int32_t* __restrict__ O, float* __restrict__ s_O, float* __restrict__ colscale,
                          float* __restrict__ cmax_out, const float* __restrict__ W_O, int64_t c_out,
                          int8_t* __restrict__ what_int, float* __restrict__ delta_what) {
    constexpr int NT = kWideCh * kWideGroups;
    extern __shared__ float sm1[];                                  // [n] : s_k - 1
    uint32_t* smax = reinterpret_cast<uint32_t*>(sm1 + n);         // [n]
    float* red = sm1 + 2 * n;                                       // [kWideGroups][kWideCh]
    for (int k = threadIdx.x; k < n; k += NT) smax[k] = 0u;
    __syncthreads();
    const int total = nslab * n;
    for (int e0 = threadIdx.x; e0 < total; e0 += 16 * NT) {
        uint32_t v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            int e = e0 + u * NT;
            v[u] = part[e < total ? e : total - 1];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            int e = e0 + u * NT;
            if (e < total) atomicMax(&smax[e % n], v[u]);
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < n; k += NT) {
        float cmax = __uint_as_float(smax[k]);
        float s = momentum_scale(cmax, wmax_O[k], s_prev[k], gamma);
        sm1[k] = __fsub_rn(s, 1.0f);
        if (blockIdx.x == 0) {
            s_O[k] = s;
            colscale[O[k]] = __fdiv_rn(1.0f, s);
            if (cmax_out) cmax_out[k] = cmax;
        }
    }
    __syncthreads();
    const int jj = threadIdx.x % kWideCh, grp = threadIdx.x / kWideCh;
    const int64_t j = (int64_t)blockIdx.x * kWideCh + jj;
    const int64_t jc = j < c_out ? j : c_out - 1;
    const int per = n_pad / kWideGroups;                  // a multiple of 4 (n_pad is a multiple of 64)
    const int kb = grp * per, ke = kb + per < n ? kb + per : n;
    // pass 1: this group's share of max_k |what[k, j]|
    float m = 0.0f;
    for (int k0 = kb; k0 < ke; k0 += 8) {
        float w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) w[u] = W_O[(int64_t)(k0 + u < ke ? k0 + u : ke - 1) * c_out + jc];
#pragma unroll
        for (int u = 0; u < 8; ++u) m = fmaxf(m, fabsf(__fmul_rn(sm1[k0 + u < ke ? k0 + u : ke - 1], w[u])));
    }
    red[grp * kWideCh + jj] = m;
    __syncthreads();
    m = 0.0f;
#pragma unroll
    for (int g2 = 0; g2 < kWideGroups; ++g2) m = fmaxf(m, red[g2 * kWideCh + jj]);
    float d, c;
    rtn_steps(m, d, c);
    if (j >= c_out) return;
    if (grp == 0) delta_what[j] = d;
    // pass 2: codes of this group's range (zero beyond n), four per 32-bit store
    uint32_t* dst = reinterpret_cast<uint32_t*>(what_int + j * n_pad + kb);
    for (int k0 = kb; k0 < kb + per; k0 += 8) {
        float w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u;
            w[u] = W_O[(int64_t)(k < n ? k : n - 1) * c_out + j];
        }
        uint32_t q[2] = {0u, 0u};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = k0 + u;
            int code = 0;
            if (k < n) code = rtn_code(__fmul_rn(sm1[k], w[u]), c);
            q[u >> 2] |= (uint32_t)(code & 0xFF) << (8 * (u & 3));
        }
        dst[(k0 - kb) >> 2] = q[0];
        if (k0 + 4 < kb + per) dst[((k0 - kb) >> 2) + 1] = q[1];
    }
}

// Validity of an outlier index list (Sec. 3.3 fixes O before fine-tuning: one check per layer).  One workgroup scans
// the list; *result = 0 when O is strictly ascending and inside [0, c_in), else 1 + the first offending position.
__global__ void __launch_bounds__(256)
check_outliers_kernel(const int32_t* __restrict__ O, int n, int64_t c_in, int32_t* __restrict__ result) {
    __shared__ int first_bad;
    if (threadIdx.x == 0) first_bad = 0x7FFFFFFF;
    __syncthreads();
    int mine = 0x7FFFFFFF;
    for (int k = threadIdx.x; k < n; k += 256) {
        const int64_t v = O[k];
        const bool bad = v < 0 || v >= c_in || (k > 0 && (int64_t)O[k - 1] >= v);
        if (bad && k < mine) mine = k;
    }
    if (mine != 0x7FFFFFFF) atomicMin(&first_bad, mine);
    __syncthreads();
    if (threadIdx.x == 0) *result = first_bad == 0x7FFFFFFF ? 0 : first_bad + 1;
}

hipError_t launch_check_outliers(const int32_t* O, int32_t n, int64_t c_in, int32_t* result, hipStream_t stream) {
    hipLaunchKernelGGL(check_outliers_kernel, dim3(1), dim3(256), 0, stream, O, n, c_in, result);
    return hipGetLastError();
}

// as many slabs as the rows allow, but no more partial maxima than momentum_what_kernel reduces in one batch
int scale_update_gather_slabs(int64_t t, int32_t n) {
    int nslab = scale_update_blocks(t);
    const int one_batch = kPartBatch * kWhatThreads / n;
    const int cap = one_batch > 16 ? one_batch : 16;
    return nslab < cap ? nslab : cap;
}

hipError_t launch_scale_update(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O, int32_t n,
                               const float* W_O, const float* wmax_O, int64_t c_out, float gamma, float* s_O,
                               float* colscale, int8_t* what_int, float* delta_what, float* cmax_out, float* ws,
                               hipStream_t stream) {
    const int n_pad = (n + kPadK - 1) / kPadK * kPadK;
    uint32_t* part = reinterpret_cast<uint32_t*>(ws);   // [nslab x n]
    int nslab = scale_update_blocks(t);
    const bool dense = (int64_t)n * 64 >= c_in;          // most 64-byte segments of a row hold an outlier anyway
    if (dense) {
        // enough (chunk, slab) workgroups to fill the chip, within the slab count the workspace was sized for
        const int chunks = (int)((c_in + 2047) / 2048);
        int want = (512 + chunks - 1) / chunks;
        if (want < nslab) nslab = want;
        const int rows = (int)((t + nslab - 1) / nslab);
        nslab = (int)((t + rows - 1) / rows);
        float* s_prev = ws + (int64_t)nslab * n;
        {
            ProfScope prof(K_COLMAX, stream);
            hipLaunchKernelGGL(colmax_dense_kernel, dim3(chunks, nslab), dim3(256), 0, stream, X, t, c_in, ldx, O, n,
                               part, s_O, s_prev, rows);
        }
        return launch_momentum(part, nslab, n, n_pad, wmax_O, s_prev, gamma, O, s_O, colscale, cmax_out, W_O, c_out,
                               what_int, delta_what, stream);
    }
    nslab = scale_update_gather_slabs(t, n);
    float* s_prev = ws + (int64_t)nslab * n;            // [n]
    {
        ProfScope prof(K_COLMAX, stream);
        hipLaunchKernelGGL(colmax_outlier_kernel, dim3(nslab), dim3(256), 0, stream, X, t, ldx, O,
                           n, part, s_O, s_prev);
    }
    return launch_momentum(part, nslab, n, n_pad, wmax_O, s_prev, gamma, O, s_O, colscale, cmax_out, W_O, c_out,
                           what_int, delta_what, stream);
}

hipError_t launch_momentum(const uint32_t* part, int nslab, int n, int n_pad, const float* wmax_O,
                                  const float* s_prev, float gamma, const int32_t* O, float* s_O, float* colscale,
                                  float* cmax_out, const float* W_O, int64_t c_out, int8_t* what_int,
                                  float* delta_what, hipStream_t stream) {
    ProfScope prof(K_MOMENTUM, stream);
    if (n <= 64) {
        hipLaunchKernelGGL(momentum_what_kernel, dim3((unsigned)((c_out + kWhatThreads - 1) / kWhatThreads)),
                           dim3(kWhatThreads), 2 * n * sizeof(float), stream, part, nslab, n, n_pad, wmax_O, s_prev,
                           gamma, O, s_O, colscale, cmax_out, W_O, c_out, what_int, delta_what);
    } else {
        const size_t lds = (2 * (size_t)n + kWideCh * kWideGroups) * sizeof(float);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(momentum_what_wide_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(momentum_what_wide_kernel, dim3((unsigned)((c_out + kWideCh - 1) / kWideCh)),
                           dim3(kWideCh * kWideGroups), lds, stream, part, nslab, n, n_pad, wmax_O, s_prev, gamma, O,
                           s_O, colscale, cmax_out, W_O, c_out, what_int, delta_what);
    }
    return hipGetLastError();
}

}  // namespace quaff
