// Device code of the fused column scaling and per-token INT8 quantization (Eq. 5 then Eq. 1 of the paper), shared by
// the stand-alone quantizer launch and by the launch that runs it next to the LoRA down-projection.
#pragma once
#include "quaff_internal.h"

namespace quaff {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// The column scales may live in global memory (const float*) or in LDS (const lds_float*).
typedef __attribute__((address_space(3))) float lds_float;
template <class P> struct Vec4Of;
template <> struct Vec4Of<const float*> { typedef const f32x4* type; };
template <> struct Vec4Of<const lds_float*> { typedef const __attribute__((address_space(3))) f32x4* type; };
struct NoPrologue { __device__ __forceinline__ void operator()() const {} };
// "are there column scales at all": a global pointer may be null; an LDS copy always exists (and may legitimately
// sit at LDS offset 0, which must not be mistaken for a null pointer)
__device__ __forceinline__ bool has_scales(const float* cs) { return cs != nullptr; }
__device__ __forceinline__ bool has_scales(const lds_float*) { return true; }

// scaled fp32 values of eight consecutive bf16 elements
template <class CsPtr>
__device__ __forceinline__ void widen_scale(const u32x4& raw, CsPtr cs, int64_t col, float (&v)[8]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        v[2 * u] = __uint_as_float(raw[u] << 16);
        v[2 * u + 1] = __uint_as_float(raw[u] & 0xFFFF0000u);
    }
    if (has_scales(cs)) {
        f32x4 c0 = *(typename Vec4Of<CsPtr>::type)(cs + col);
        f32x4 c1 = *(typename Vec4Of<CsPtr>::type)(cs + col + 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v[u] = __fmul_rn(v[u], c0[u]);
            v[4 + u] = __fmul_rn(v[4 + u], c1[u]);
        }
    }
}

// Eight codes of Eq. 1, packed.  code = rne(x * c): the product is rounded once (fp32), then adding 1.5 * 2^23 rounds
// it to the nearest integer, ties to even, in the same addition - the sum is exact for |product| < 2^22 - and leaves
// that integer's two's complement in the low mantissa bits, so the low byte is the code.  No clamp is needed for
// finite inputs: |x| <= m gives |x * fl(127 / m)| < 127.5, which rounds to at most 127 (a non-finite input, outside
// the contract, yields an unspecified byte).  Three byte permutes assemble four codes into a word.
__device__ __forceinline__ u32x2 pack_codes(const float (&v)[8], float c) {
    u32x2 out;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) b[u] = __float_as_uint(__fadd_rn(__fmul_rn(v[4 * h + u], c), 12582912.0f));
        // __builtin_amdgcn_perm(hi, lo, sel): result byte i = byte sel[i] of the pair {hi: bytes 4..7, lo: bytes 0..3}
        const uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], 0x0C0C0400u);   // byte 0 of b0, byte 0 of b1, zero, zero
        const uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], 0x04000C0Cu);   // zero, zero, byte 0 of b2, byte 0 of b3
        out[h] = lo | hi;
    }
    return out;
}

// compact copy of the outlier columns' codes: xq_O[row, k] = code(X[row, O_k]), zero beyond n
template <class CsPtr>
__device__ __forceinline__ void write_outlier_codes(const uint16_t* __restrict__ xrow, CsPtr cs,
                                                    const int32_t* __restrict__ O, int n, int n_pad, float c,
                                                    int8_t* __restrict__ dst, int lane, int nlanes) {
    for (int k = lane; k < n_pad; k += nlanes) {
        int q = 0;
        if (k < n) {
            int col = O[k];
            float x = bf16_bits_to_f32(xrow[col]);
            if (has_scales(cs)) x = __fmul_rn(x, cs[col]);
            q = rtn_code(x, c);
        }
        dst[k] = (int8_t)q;
    }
}

// Work of one workgroup of NT threads whose index among the quantizing workgroups is `block`.
// TPR threads cooperate on one row (64 = a wavefront, 256 = four wavefronts); each holds NV vectors of 8 elements.
// `prologue` runs (on every thread of the workgroup; it may contain barriers) after the row loads have been issued
// and before the column scales are first read: the launch that derives the scales itself hides that work there.
template <int NT, int TPR, int NV, class CsPtr = const float*, class Prologue = NoPrologue>
__device__ __forceinline__ void quant_rows_body(int block, const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx,
                                                CsPtr cs, const int32_t* __restrict__ O, int n, int n_pad,
                                                int8_t* __restrict__ Xq, float* __restrict__ delta,
                                                int8_t* __restrict__ xq_O, Prologue prologue = Prologue()) {
    constexpr int RPB = NT / TPR;   // rows per workgroup
    __shared__ float red[NT / 64];
    const int lane = threadIdx.x % TPR;
    const int64_t row = (int64_t)block * RPB + threadIdx.x / TPR;
    const bool live = row < t;
    const uint16_t* xrow = X + (live ? row : 0) * ldx;

    u32x4 raw[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        int col = (i * TPR + lane) * 8;
        raw[i] = (u32x4){0, 0, 0, 0};
        if (live && col < c) raw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xrow + col));
    }
    prologue();
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
                xo[u] = has_scales(cs) ? __fmul_rn(x, cs[col]) : x;
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
        const int w0 = (threadIdx.x / TPR) * 4;   // the four wavefronts of this row
        m = fmaxf(fmaxf(red[w0], red[w0 + 1]), fmaxf(red[w0 + 2], red[w0 + 3]));
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

}  // namespace quaff
