// Fused column scaling and per-token INT8 quantization (Eq. 5 then Eq. 1 of the paper, one step size per token).
//
// HBM-bound: 2 bytes read and 1 byte written per element.  A row is read once into registers (eight bf16 per
// 16-byte load), the row maximum is taken with a wavefront reduction, and the codes leave as packed 8-byte
// stores.  Rows up to 64*8*NV elements are handled by one wavefront (four rows per workgroup); longer rows
// by a whole workgroup; anything longer than that by a two-pass fallback that re-reads the row.
#include "quaff_internal.h"

namespace quaff {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// scaled fp32 values of eight consecutive bf16 elements
__device__ __forceinline__ void widen_scale(const u32x4& raw, const float* __restrict__ cs, int64_t col, float (&v)[8]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        v[2 * u] = __uint_as_float(raw[u] << 16);
        v[2 * u + 1] = __uint_as_float(raw[u] & 0xFFFF0000u);
    }
    if (cs) {
        f32x4 c0 = *reinterpret_cast<const f32x4*>(cs + col);
        f32x4 c1 = *reinterpret_cast<const f32x4*>(cs + col + 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v[u] = __fmul_rn(v[u], c0[u]);
            v[4 + u] = __fmul_rn(v[4 + u], c1[u]);
        }
    }
}

__device__ __forceinline__ u32x2 pack_codes(const float (&v)[8], float c) {
    u32x2 out;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t w = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) w |= (uint32_t)(rtn_code(v[4 * h + u], c) & 0xFF) << (8 * u);
        out[h] = w;
    }
    return out;
}

// compact copy of the outlier columns' codes: xq_O[row, k] = code(X[row, O_k]), zero beyond n
__device__ __forceinline__ void write_outlier_codes(const uint16_t* __restrict__ xrow, const float* __restrict__ cs,
                                                    const int32_t* __restrict__ O, int n, int n_pad, float c,
                                                    int8_t* __restrict__ dst, int lane, int nlanes) {
    for (int k = lane; k < n_pad; k += nlanes) {
        int q = 0;
        if (k < n) {
            int col = O[k];
            float x = bf16_bits_to_f32(xrow[col]);
            if (cs) x = __fmul_rn(x, cs[col]);
            q = rtn_code(x, c);
        }
        dst[k] = (int8_t)q;
    }
}

// TPR threads cooperate on one row (64 = a wavefront, 256 = the workgroup); each holds NV vectors of 8 elements.
template <int TPR, int NV>
__global__ void __launch_bounds__(256)
quant_rows_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const float* __restrict__ cs,
                  const int32_t* __restrict__ O, int n, int n_pad, int8_t* __restrict__ Xq, float* __restrict__ delta,
                  int8_t* __restrict__ xq_O) {
    constexpr int RPB = 256 / TPR;   // rows per workgroup
    __shared__ float red[4];
    const int lane = threadIdx.x % TPR;
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / TPR;
    const bool live = row < t;
    const uint16_t* xrow = X + (live ? row : 0) * ldx;

    u32x4 raw[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int col = (i * TPR + lane) * 8;
        raw[i] = (u32x4){0, 0, 0, 0};
        if (live && col < c) raw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xrow + col));
    }
    // the outlier columns' values are gathered now so that their (dependent) loads overlap the row loads
    constexpr int GPL = 4;                       // gathered outliers per lane in registers (TPR * GPL per row)
    float xo[GPL];
    const bool gather_regs = xq_O && n_pad <= TPR * GPL;
    if (gather_regs) {
#pragma unroll
        for (int u = 0; u < GPL; ++u) {
            int k = lane + u * TPR;
            xo[u] = 0.0f;
            if (live && k < n) {
                int col = O[k];
                float x = bf16_bits_to_f32(xrow[col]);
                xo[u] = cs ? __fmul_rn(x, cs[col]) : x;
            }
        }
    }
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int col = (i * TPR + lane) * 8;
        if (col < c) {
            float v[8];
            widen_scale(raw[i], cs, col, v);
#pragma unroll
            for (int u = 0; u < 8; ++u) m = fmaxf(m, fabsf(v[u]));
        }
    }
    m = wave_max(m);
    if (TPR == 256) {
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
        __syncthreads();
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    }
    if (!live) return;
    float d, cc;
    rtn_steps(m, d, cc);
    if (lane == 0) delta[row] = d;
    int8_t* qrow = Xq + row * (int64_t)c;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int col = (i * TPR + lane) * 8;
        if (col < c) {
            float v[8];
            widen_scale(raw[i], cs, col, v);
            *reinterpret_cast<u32x2*>(qrow + col) = pack_codes(v, cc);
        }
    }
    if (gather_regs) {
        int8_t* dst = xq_O + row * (int64_t)n_pad;
#pragma unroll
        for (int u = 0; u < GPL; ++u) {
            int k = lane + u * TPR;
            if (k < n_pad) dst[k] = (int8_t)rtn_code(xo[u], cc);   // xo = 0 beyond n: code 0
        }
    } else if (xq_O) {
        write_outlier_codes(xrow, cs, O, n, n_pad, cc, xq_O + row * (int64_t)n_pad, lane, TPR);
    }
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
