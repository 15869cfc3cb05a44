// LoRA weight gradients of the adapter branch Y_l = scale (X A) B (rank r; the paper's App. "Model and experimental
// settings" puts LoRA on every linear layer, the frozen quantized weight gets no gradient):
//     dA = scale X^T (dY B^T)   [c_in x r]          dB = scale (X A)^T dY   [r x c_out]
// Both are one skinny product  G[p, j] = sum_i P[i, p] Q[i, j]  that contracts over the t tokens:
//     dB:  P = scale X A   (the forward down-projection),  Q = dY
//     dA:  P = scale dY B^T (the backward down-projection), Q = X,  result stored transposed.
// HBM-bound: Q is read once.  bf16 MFMA 16x16x32 with fp32 accumulation; P arrives as the hi/lo bf16 pairs the
// down-projection kernel writes and is first folded and transposed to [r x t] (token-contiguous, what the MFMA's
// first operand wants); the Q tile has the tokens on the slow axis, so it is staged row-major in LDS and the
// second operand's eight tokens per lane are gathered from there with 2-byte reads.  The token range is cut into
// slabs over workgroups; the slabs' partial results are summed in a fixed order by a second launch, so the result
// is deterministic.
#include "quaff_internal.h"

namespace quaff {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kGradCols = 128;       // columns of Q per workgroup (eight 16-column MFMA blocks, two per wavefront)
constexpr int kGradRowBytes = 264;   // LDS row stride: 256 bytes of data + 8, so that the four 8-row groups of a
                                     // gather fall into disjoint banks

__device__ __forceinline__ uint32_t grad_f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

void lora_grad_plan(int64_t t, int64_t c, int* nslab, int* rows_per_slab) {
    const int64_t t_pad = (t + 31) / 32 * 32;
    const int64_t chunks = (c + kGradCols - 1) / kGradCols;
    int64_t want = (512 + chunks - 1) / chunks;            // about two workgroups per compute unit
    if (want > 16) want = 16;                              // bounds the partial-result traffic
    if (want > t_pad / 32) want = t_pad / 32;
    if (want < 1) want = 1;
    int64_t rows = ((t_pad / 32 + want - 1) / want) * 32;
    *rows_per_slab = (int)rows;
    *nslab = (int)((t_pad + rows - 1) / rows);
}

// Pt_hi/Pt_lo [r x t_pad] <- sum over the parts of (T_hi + T_lo) [t x r], zero for tokens >= t.  blockIdx.y selects
// one of two independent inputs (the forward and the backward down-projection).
struct PrepArgs {
    const uint16_t* T_hi[2]; const uint16_t* T_lo[2];
    uint16_t* Pt_hi[2]; uint16_t* Pt_lo[2];
};
__global__ void __launch_bounds__(256)
lora_grad_prep_kernel(PrepArgs a, int64_t t, int64_t t_pad, int r) {
    const int which = blockIdx.y;
    const uint16_t* th = a.T_hi[which];
    const uint16_t* tl = a.T_lo[which];
    const int64_t total = t_pad * r;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t p = e / t_pad, i = e % t_pad;
        float v = 0.0f;
        if (i < t) {
#pragma unroll
            for (int part = 0; part < kLoraParts; ++part) {
                const int64_t o = (int64_t)part * t * r + i * r + p;
                v += bf16_bits_to_f32(th[o]) + bf16_bits_to_f32(tl[o]);
            }
        }
        const uint32_t hi = grad_f32_to_bf16_rne(v);
        a.Pt_hi[which][e] = (uint16_t)hi;
        a.Pt_lo[which][e] = (uint16_t)grad_f32_to_bf16_rne(v - __uint_as_float(hi << 16));
    }
}

// partial[slab][p][j] = sum over the slab's tokens i of P[i, p] Q[i, j]
// one of the two products of a launch (blockIdx.z selects it)
struct GradProblem {
    const uint16_t* Q; int64_t ldq; int c;
    const uint16_t* Pt_hi; const uint16_t* Pt_lo;
    int rows_per_slab, nslab, chunks;
    float* partial; float* out; int transposed;
};
struct GradPair { GradProblem p[2]; };

template <int R16>
__global__ void __launch_bounds__(256)
lora_grad_kernel(GradPair pair, int64_t t, int64_t t_pad) {
    constexpr int r = R16 * 16;
    const GradProblem& pb = pair.p[blockIdx.z];
    if ((int)blockIdx.x >= pb.chunks || (int)blockIdx.y >= pb.nslab) return;
    const uint16_t* __restrict__ Q = pb.Q;
    const int64_t ldq = pb.ldq;
    const int c = pb.c, rows_per_slab = pb.rows_per_slab;
    const uint16_t* __restrict__ Pt_hi = pb.Pt_hi;
    const uint16_t* __restrict__ Pt_lo = pb.Pt_lo;
    float* __restrict__ partial = pb.partial;
    __shared__ __attribute__((aligned(16))) uint8_t tile[32 * kGradRowBytes];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int c0 = blockIdx.x * kGradCols;
    const int64_t i_begin = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t i_end = i_begin + rows_per_slab < t_pad ? i_begin + rows_per_slab : t_pad;

    // loader: 32 rows x 256 bytes = 512 vectors of 16 bytes, two per thread (rows tid / 16 and tid / 16 + 16)
    const int ld_row = tid >> 4;
    int ld_col = c0 + (tid & 15) * 8;
    if (ld_col > c - 8) ld_col = c - 8;        // columns past the edge repeat valid data and are never stored
    auto load_tile = [&](int64_t i0, u32x4 (&regs)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int64_t row = i0 + ld_row + 16 * h;
            if (row > t - 1) row = t - 1;      // tokens past the end repeat the last one; P is zero there
            regs[h] = *reinterpret_cast<const u32x4*>(Q + row * ldq + ld_col);
        }
    };

    f32x4 acc[R16][2];
#pragma unroll
    for (int b = 0; b < R16; ++b)
#pragma unroll
        for (int f = 0; f < 2; ++f) acc[b][f] = (f32x4){0.f, 0.f, 0.f, 0.f};

    u32x4 regs[2];
    load_tile(i_begin, regs);
    for (int64_t i0 = i_begin; i0 < i_end; i0 += 32) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint8_t* dst = tile + (ld_row + 16 * h) * kGradRowBytes + (tid & 15) * 16;
            *reinterpret_cast<u32x2*>(dst) = (u32x2){regs[h][0], regs[h][1]};
            *reinterpret_cast<u32x2*>(dst + 8) = (u32x2){regs[h][2], regs[h][3]};
        }
        __syncthreads();
        if (i0 + 32 < i_end) load_tile(i0 + 32, regs);
        u32x4 ah[R16], al[R16];
#pragma unroll
        for (int b = 0; b < R16; ++b) {
            const int64_t o = (int64_t)(b * 16 + n) * t_pad + i0 + g * 8;
            ah[b] = *reinterpret_cast<const u32x4*>(Pt_hi + o);
            al[b] = *reinterpret_cast<const u32x4*>(Pt_lo + o);
        }
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            // second operand: tokens i0 + 8 g .. + 7 of column c0 + 16 (2 wave + f) + n
            const uint8_t* src = tile + (g * 8) * kGradRowBytes + ((wave * 2 + f) * 16 + n) * 2;
            u32x4 q;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                uint32_t lo = *reinterpret_cast<const uint16_t*>(src + (2 * jj) * kGradRowBytes);
                uint32_t hi = *reinterpret_cast<const uint16_t*>(src + (2 * jj + 1) * kGradRowBytes);
                q[jj] = lo | (hi << 16);
            }
#pragma unroll
            for (int b = 0; b < R16; ++b) {
                acc[b][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ah[b]),
                                                                    __builtin_bit_cast(bf16x8, q), acc[b][f], 0, 0, 0);
                acc[b][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, al[b]),
                                                                    __builtin_bit_cast(bf16x8, q), acc[b][f], 0, 0, 0);
            }
        }
        __syncthreads();
    }
    // element v of lane (n, g) is G[16 b + 4 g + v][c0 + 16 (2 wave + f) + n]
    float* out = partial + (int64_t)blockIdx.y * r * c;
#pragma unroll
    for (int f = 0; f < 2; ++f) {
        const int col = c0 + (wave * 2 + f) * 16 + n;
        if (col >= c) continue;
#pragma unroll
        for (int b = 0; b < R16; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) out[(int64_t)(b * 16 + g * 4 + v) * c + col] = acc[b][f][v];
    }
}

// out = sum over slabs (fixed order) of partial[slab]; transposed = write out[j][p] instead of out[p][j]
__global__ void __launch_bounds__(256)
lora_grad_reduce_kernel(GradPair pair, int r) {
    const GradProblem& pb = pair.p[blockIdx.y];
    const float* __restrict__ partial = pb.partial;
    float* __restrict__ out = pb.out;
    const int nslab = pb.nslab, c = pb.c, transposed = pb.transposed;
    const int64_t total = (int64_t)r * c;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        // consecutive threads take consecutive output addresses
        const int64_t p = transposed ? e % r : e / c, j = transposed ? e / r : e % c;
        float s = 0.0f;
        for (int sl = 0; sl < nslab; ++sl) s += partial[((int64_t)sl * r + p) * c + j];
        out[e] = s;
    }
}

hipError_t launch_lora_grad_prep(const uint16_t* T1_hi, const uint16_t* T1_lo, uint16_t* Pt1_hi, uint16_t* Pt1_lo,
                                 const uint16_t* T2_hi, const uint16_t* T2_lo, uint16_t* Pt2_hi, uint16_t* Pt2_lo,
                                 int64_t t, int32_t r, hipStream_t stream) {
    ProfScope prof(K_LORA_GRAD, stream);
    const int64_t t_pad = (t + 31) / 32 * 32;
    PrepArgs a{{T1_hi, T2_hi}, {T1_lo, T2_lo}, {Pt1_hi, Pt2_hi}, {Pt1_lo, Pt2_lo}};
    int64_t blocks = (t_pad * r + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(lora_grad_prep_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, stream, a, t, t_pad, r);
    return hipGetLastError();
}

// Both gradient products of a layer in one launch each (product, then slab reduction):
//   dA^T [r x c_in] = P1^T X (stored transposed as dA [c_in x r]),   dB [r x c_out] = P2^T dY
hipError_t launch_lora_grad_pair(const uint16_t* X, int64_t ldx, int64_t c_in, const uint16_t* Pt1_hi,
                                 const uint16_t* Pt1_lo, float* partial_a, float* dA, const uint16_t* dY, int64_t lddy,
                                 int64_t c_out, const uint16_t* Pt2_hi, const uint16_t* Pt2_lo, float* partial_b,
                                 float* dB, int64_t t, int32_t r, hipStream_t stream) {
    ProfScope prof(K_LORA_GRAD, stream);
    const int64_t t_pad = (t + 31) / 32 * 32;
    GradPair pair;
    auto fill = [&](GradProblem& p, const uint16_t* Q, int64_t ldq, int64_t c, const uint16_t* hi, const uint16_t* lo,
                    float* partial, float* out, int transposed) {
        p.Q = Q; p.ldq = ldq; p.c = (int)c; p.Pt_hi = hi; p.Pt_lo = lo;
        lora_grad_plan(t, c, &p.nslab, &p.rows_per_slab);
        p.chunks = (int)((c + kGradCols - 1) / kGradCols);
        p.partial = partial; p.out = out; p.transposed = transposed;
    };
    fill(pair.p[0], X, ldx, c_in, Pt1_hi, Pt1_lo, partial_a, dA, 1);
    fill(pair.p[1], dY, lddy, c_out, Pt2_hi, Pt2_lo, partial_b, dB, 0);
    const int gx = pair.p[0].chunks > pair.p[1].chunks ? pair.p[0].chunks : pair.p[1].chunks;
    const int gy = pair.p[0].nslab > pair.p[1].nslab ? pair.p[0].nslab : pair.p[1].nslab;
    dim3 grid((unsigned)gx, (unsigned)gy, 2);
#define QUAFF_GRAD(N)                                                                              \
    case N:                                                                                        \
        hipLaunchKernelGGL((lora_grad_kernel<N>), grid, dim3(256), 0, stream, pair, t, t_pad);     \
        break;
    switch (r / 16) {
        QUAFF_GRAD(1) QUAFF_GRAD(2) QUAFF_GRAD(3) QUAFF_GRAD(4)
    }
#undef QUAFF_GRAD
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t cmax = c_in > c_out ? c_in : c_out;
    int64_t blocks = ((int64_t)r * cmax + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(lora_grad_reduce_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, stream, pair, (int)r);
    return hipGetLastError();
}

}  // namespace quaff
