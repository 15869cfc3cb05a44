// Outlier-channel identification on calibration data (Eq. 6 of the paper, Sec. 3.3) and budgeted selection of O.
//   xi_o = number of calibration samples i with  max_rows |X^i[:, o]| > ratio * mean(|X^i|)       (ratio = 100)
// Four launches:
//   calib_sample_kernel   one workgroup per (2048-column chunk, sample, row slab): streams its rows once (HBM-bound),
//                         keeps the running column maxima in registers (bf16 magnitudes compare as integers) and
//                         the sum of magnitudes in fp64;
//   calib_count_kernel    thresholds ratio * mean per sample (fp64, chunk sums added in a fixed order), then one
//                         thread per channel counts the samples that exceed theirs;
//   calib_rank_kernel     rank of every channel in the order (xi descending, index ascending), summed over slices
//   calib_place_kernel    the first `budget` channels of that order with xi > 0, written in ascending channel order.
// The comparison that decides a count is made in fp64 on both sides of the parity test; the fp64 sum of a few
// million bf16 magnitudes is exact or within an ulp whatever the order, so a decision could only differ for a
// column maximum within 1e-15 (relative) of the threshold.
#include "quaff_internal.h"

namespace quaff {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kCalibCols = 2048;   // columns per workgroup: 256 threads x 8
constexpr int kCalibSlabs = 8;     // a sample's rows are cut into this many slabs, one workgroup each

__global__ void __launch_bounds__(256)
calib_sample_kernel(const uint16_t* __restrict__ X, int64_t ldx, int64_t c_in, int64_t t_total,
                    const int64_t* __restrict__ offsets, uint16_t* __restrict__ colmax, double* __restrict__ part_sum) {
    __shared__ double red[256];
    const int sample = blockIdx.y, nchunk = gridDim.x;
    int64_t r0 = offsets[sample], r1 = offsets[sample + 1];
    r0 = r0 < 0 ? 0 : r0;                      // offsets are the caller's: never read outside X whatever they hold
    r1 = r1 > t_total ? t_total : r1;
    {
        const int64_t per = r1 > r0 ? (r1 - r0 + kCalibSlabs - 1) / kCalibSlabs : 0;
        r0 += blockIdx.z * per;
        r1 = r0 + per < r1 ? r0 + per : r1;   // may leave this slab empty (r1 <= r0)
    }
    const int64_t unit = (int64_t)sample * kCalibSlabs + blockIdx.z;
    const int64_t col = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    const bool live = col < c_in;
    uint32_t mx[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    double sum = 0.0;
    if (live) {
        const uint16_t* src = X + col;
        for (int64_t row = r0; row < r1; row += 4) {   // four independent loads in flight
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                int64_t rr = row + u < r1 ? row + u : r1 - 1;
                v[u] = *reinterpret_cast<const u32x4*>(src + rr * ldx);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (row + u >= r1) continue;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    uint32_t lo = v[u][w] & 0x7FFFu, hi = (v[u][w] >> 16) & 0x7FFFu;
                    mx[2 * w] = lo > mx[2 * w] ? lo : mx[2 * w];
                    mx[2 * w + 1] = hi > mx[2 * w + 1] ? hi : mx[2 * w + 1];
                    sum += (double)__uint_as_float(lo << 16);
                    sum += (double)__uint_as_float(hi << 16);
                }
            }
        }
        u32x4 out;
#pragma unroll
        for (int w = 0; w < 4; ++w) out[w] = mx[2 * w] | (mx[2 * w + 1] << 16);
        *reinterpret_cast<u32x4*>(colmax + unit * c_in + col) = out;
    }
    red[threadIdx.x] = sum;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {           // fixed-order tree
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) part_sum[unit * nchunk + blockIdx.x] = red[0];
}

constexpr int kCalibTile = 2048;   // samples whose thresholds are held in LDS at a time

__global__ void __launch_bounds__(256)
calib_count_kernel(const uint16_t* __restrict__ colmax, const double* __restrict__ part_sum, int nchunk,
                   const int64_t* __restrict__ offsets, int64_t t_total, int n_samples, int64_t c_in, double ratio,
                   int32_t* __restrict__ xi, int32_t* __restrict__ rank) {
    __shared__ double thr[kCalibTile];
    const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int count = 0;
    for (int s0 = 0; s0 < n_samples; s0 += kCalibTile) {
        const int ns = n_samples - s0 < kCalibTile ? n_samples - s0 : kCalibTile;
        __syncthreads();
        for (int i = threadIdx.x; i < ns; i += 256) {
            int64_t r0 = offsets[s0 + i], r1 = offsets[s0 + i + 1];
            r0 = r0 < 0 ? 0 : r0;
            r1 = r1 > t_total ? t_total : r1;
            double sum = 0.0;
            for (int ch = 0; ch < kCalibSlabs * nchunk; ++ch) sum += part_sum[(int64_t)(s0 + i) * kCalibSlabs * nchunk + ch];
            // an empty sample flags nothing
            thr[i] = r1 > r0 ? ratio * (sum / ((double)(r1 - r0) * (double)c_in)) : __builtin_huge_val();
        }
        __syncthreads();
        if (o < c_in)
            for (int i = 0; i < ns; ++i) {
                uint32_t mb = 0;
#pragma unroll
                for (int z = 0; z < kCalibSlabs; ++z) {
                    uint32_t v = colmax[((int64_t)(s0 + i) * kCalibSlabs + z) * c_in + o];
                    mb = v > mb ? v : mb;
                }
                double m = (double)bf16_bits_to_f32(mb);
                count += m > thr[i] ? 1 : 0;
            }
    }
    if (o < c_in) {
        xi[o] = count;
        rank[o] = 0;   // accumulated by calib_rank_kernel
    }
}

// rank[o] += number of channels q in this workgroup's 2048-channel slice that precede o in the order
// (xi descending, index ascending).  One thread per channel and slice; integer atomics, so the sum is exact
// whatever the order.  rank was zeroed by calib_count_kernel.
__global__ void __launch_bounds__(256)
calib_rank_kernel(const int32_t* __restrict__ xi, int c_in, int32_t* __restrict__ rank) {
    __shared__ int32_t tile[2048];
    const int o = blockIdx.x * 256 + threadIdx.x;
    const int q0 = blockIdx.y * 2048;
    const int nq = c_in - q0 < 2048 ? c_in - q0 : 2048;
    for (int q = threadIdx.x; q < nq; q += 256) tile[q] = xi[q0 + q];
    __syncthreads();
    if (o >= c_in) return;
    const int x = xi[o];
    int r = 0;
    for (int q = 0; q < nq; ++q) {
        const int y = tile[q];
        r += (y > x || (y == x && q0 + q < o)) ? 1 : 0;
    }
    atomicAdd(&rank[o], r);
}

// Channel o is selected iff xi[o] > 0 and rank[o] < budget.  O[pos] = o for the selected channels in ascending
// order, pos = number of selected channels below o.
__global__ void __launch_bounds__(256)
calib_place_kernel(const int32_t* __restrict__ xi, const int32_t* __restrict__ rank, int budget, int c_in,
                   int32_t* __restrict__ O, int32_t* __restrict__ n_out) {
    __shared__ uint8_t tile[4096];
    const int o = blockIdx.x * 256 + threadIdx.x;
    const int last = blockIdx.x * 256 + 255 < c_in - 1 ? blockIdx.x * 256 + 255 : c_in - 1;   // highest channel here
    int pos = 0;
    for (int q0 = 0; q0 <= last; q0 += 4096) {
        const int nq = c_in - q0 < 4096 ? c_in - q0 : 4096;
        __syncthreads();
        for (int q = threadIdx.x; q < nq; q += 256) tile[q] = (xi[q0 + q] > 0 && rank[q0 + q] < budget) ? 1 : 0;
        __syncthreads();
        const int lim = o - q0 < nq ? o - q0 : nq;     // channels q0 .. min(o, q0 + nq) - 1
        for (int q = 0; q < lim; ++q) pos += tile[q];
    }
    if (o >= c_in) return;
    const int mine = (xi[o] > 0 && rank[o] < budget) ? 1 : 0;
    if (mine) O[pos] = o;
    if (o == c_in - 1) *n_out = pos + mine;
}

hipError_t launch_calibrate(const uint16_t* X, int64_t ldx, int64_t c_in, int64_t t_total, const int64_t* offsets,
                            int32_t n_samples, double ratio, int32_t budget, int32_t* xi, int32_t* O, int32_t* n_out,
                            uint16_t* colmax, double* part_sum, int32_t* rank, hipStream_t stream) {
    ProfScope prof(K_CALIB, stream);
    const int nchunk = (int)((c_in + kCalibCols - 1) / kCalibCols);
    hipLaunchKernelGGL(calib_sample_kernel, dim3(nchunk, n_samples, kCalibSlabs), dim3(256), 0, stream, X, ldx, c_in, t_total,
                       offsets, colmax, part_sum);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(calib_count_kernel, dim3((unsigned)((c_in + 255) / 256)), dim3(256), 0, stream, colmax, part_sum,
                       nchunk, offsets, t_total, n_samples, c_in, ratio, xi, rank);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (O) {
        const unsigned nb = (unsigned)((c_in + 255) / 256);
        hipLaunchKernelGGL(calib_rank_kernel, dim3(nb, (unsigned)((c_in + 2047) / 2048)), dim3(256), 0, stream, xi,
                           (int)c_in, rank);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(calib_place_kernel, dim3(nb), dim3(256), 0, stream, xi, rank, budget, (int)c_in, O, n_out);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace quaff
