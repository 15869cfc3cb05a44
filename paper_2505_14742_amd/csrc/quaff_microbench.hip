// Device micro-benchmarks used to put measured ceilings next to the published peaks that roofline fractions are
// quoted against: the sustained rate of a register-only v_mfma_i32_32x32x32_i8 loop (with constant or with
// full-range random operands - the sustained clock, and with it the rate, depends on operand toggling), and the
// bandwidth of a plain streaming copy.  Not part of the method; these calls allocate and synchronize.
#include "../../include/quaff.h"
#include "quaff_internal.h"

namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(256) mfma_rate_kernel(int iters, int random_operands, long long* out) {
    i32x4 p[8];
    for (int i = 0; i < 8; ++i)
        for (int j = 0; j < 4; ++j) {
            unsigned h = (threadIdx.x * 977u + i * 131u + j * 31u + blockIdx.x * 7u) * 2654435761u;
            h ^= h >> 13; h *= 2246822519u; h ^= h >> 16;
            p[i][j] = random_operands ? (int)h : 0x01020304;
        }
    i32x16 c[8];
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 16; ++v) c[i][v] = 0;
    long long m0 = __builtin_amdgcn_s_memtime(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(p[i], p[(i + 3) & 7], c[i], 0, 0, 0);
    }
    long long m1 = __builtin_amdgcn_s_memtime(), w1 = wall_clock64();
    int s = 0;
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 16; ++v) s += c[i][v];
    if (threadIdx.x == 0 && blockIdx.x == 0) { out[0] = m1 - m0; out[1] = w1 - w0; }
    if (s == 0x12345678) out[2] = s;   // keeps the accumulators alive
}

__global__ void __launch_bounds__(256) copy_kernel(const i32x4* __restrict__ a, i32x4* __restrict__ b, size_t n) {
    size_t i = blockIdx.x * (size_t)256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) b[i] = a[i];
}

}  // namespace

extern "C" {

int quaff_microbench_mfma_i8(int random_operands, double* tops, double* clock_mhz) {
    if (!tops || !clock_mhz) return QUAFF_ERR_NULL;
    int dev = 0, cus = 0;
    long long* d = nullptr;
    hipEvent_t e0, e1;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipMalloc(&d, 64) != hipSuccess || hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return QUAFF_ERR_HIP;
    const int iters = 20000, blocks = 2 * cus;   // two wavefronts per SIMD
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, 0, 500, random_operands, d);
    (void)hipEventRecord(e0, 0);
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(blocks), dim3(256), 0, 0, iters, random_operands, d);
    (void)hipEventRecord(e1, 0);
    float ms = 0.f;
    long long h[2] = {0, 1};
    int st = QUAFF_OK;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
        hipMemcpy(h, d, 16, hipMemcpyDeviceToHost) != hipSuccess)
        st = QUAFF_ERR_HIP;
    *tops = (double)blocks * 4 * iters * 8 * 65536.0 / (ms * 1e-3) / 1e12;
    *clock_mhz = (double)h[0] / (double)(h[1] > 0 ? h[1] : 1) * 100.0;   // shader cycles per 100 MHz tick
    (void)hipFree(d); (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return st;
}

int quaff_microbench_copy(size_t bytes, double* gbs_read_plus_write) {
    if (!gbs_read_plus_write) return QUAFF_ERR_NULL;
    if (bytes < (1u << 20) || bytes % 16 != 0) return QUAFF_ERR_SHAPE;
    i32x4 *a = nullptr, *b = nullptr;
    hipEvent_t e0, e1;
    if (hipMalloc(&a, bytes) != hipSuccess) return QUAFF_ERR_HIP;
    if (hipMalloc(&b, bytes) != hipSuccess) { (void)hipFree(a); return QUAFF_ERR_HIP; }
    (void)hipMemset(a, 1, bytes); (void)hipMemset(b, 2, bytes);
    (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    const int reps = 5;
    hipLaunchKernelGGL(copy_kernel, dim3(32768), dim3(256), 0, 0, a, b, bytes / 16);
    (void)hipEventRecord(e0, 0);
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(copy_kernel, dim3(32768), dim3(256), 0, 0, a, b, bytes / 16);
    (void)hipEventRecord(e1, 0);
    float ms = 0.f;
    int st = QUAFF_OK;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) st = QUAFF_ERR_HIP;
    *gbs_read_plus_write = 2.0 * bytes * reps / (ms * 1e-3) / 1e9;
    (void)hipFree(a); (void)hipFree(b); (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return st;
}

}  // extern "C"
