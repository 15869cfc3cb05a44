// LoRA weight gradients of the adapter branch Y_l = scale (X A) B (rank r; the paper's App. "Model and experimental
// settings" puts LoRA on every linear layer, the frozen quantized weight gets no gradient):
//     dA = scale X^T (dY B^T)   [c_in x r]          dB = scale (X A)^T dY   [r x c_out]
// Both are one skinny product  G[p, j] = sum_i P[i, p] Q[i, j]  that contracts over the t tokens:
//     dB:  P = scale X A   (the forward down-projection),  Q = dY
//     dA:  P = scale dY B^T (the backward down-projection), Q = X,  result stored transposed.
// HBM-bound: Q is read once.  bf16 MFMA 16x16x32 with fp32 accumulation.  Both operands have the tokens on the slow
// axis while the MFMA wants them contiguous per lane, so 64-token tiles of both are staged row-major in LDS (two
// buffers used in turn, one barrier per tile, the next tile's global loads in flight while this one is multiplied) and
// a lane gathers its eight tokens with 2-byte reads.  P arrives as the hi/lo bf16 parts the down-projection kernel
// writes (one pair per half of its contraction range) and is folded to one hi/lo pair while it is staged.  Both
// products of a layer run in one launch.  The token range is cut into slabs over workgroups; the slabs' partial
// results are summed in a fixed order by a second launch that fills the chip, so the result is deterministic.
// (Measured and dropped: the sum done inside the product launch by whichever workgroup of a column chunk finishes
// last, found with a ticket counter.  The sixteen partial results per element have to be fetched past the caches
// by a few workgroups at the tail of the launch; both Phi-3 attention projections took 0.129 ms against 0.079 ms.)
#include "quaff_internal.h"

namespace quaff {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kGradCols = 128;       // columns of Q per workgroup (eight 16-column MFMA blocks, two per wavefront)
constexpr int kGradTokens = 64;      // tokens per staged tile
constexpr int kGradRowBytes = 264;   // LDS row stride of a Q tile: 256 bytes of data + 8, so that the four 8-row groups
                                     // of a gather fall into disjoint banks

__device__ __forceinline__ uint32_t grad_f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

void lora_grad_plan(int64_t t, int64_t c, int* nslab, int* rows_per_slab) {
    const int64_t tiles = (t + kGradTokens - 1) / kGradTokens;
    const int64_t chunks = (c + kGradCols - 1) / kGradCols;
    int64_t want = (512 + chunks - 1) / chunks;            // about two workgroups per compute unit
    // at most eight slabs: the partial results are written and read once more, and the launch that sums them gets
    // longer with every slab (measured at 2048 tokens: 16 slabs 41 / 31 us per call for the two Phi-3 attention
    // projections, 8 slabs 36 / 29 us, 4 slabs 38 / 31 us)
    if (want > 8) want = 8;
    if (want > tiles) want = tiles;
    if (want < 1) want = 1;
    const int64_t rows = ((tiles + want - 1) / want) * kGradTokens;
    *rows_per_slab = (int)rows;
    *nslab = (int)((tiles * kGradTokens + rows - 1) / rows);
}
int lora_grad_chunks(int64_t c) { return (int)((c + kGradCols - 1) / kGradCols); }

// partial[slab][p][j] = sum over the slab's tokens i of P[i, p] Q[i, j];  P = the sum of the kLoraParts hi/lo pairs of T.
// One of the two products of a launch (blockIdx.z selects it).
struct GradProblem {
    const uint16_t* Q; int64_t ldq; int c;
    const uint16_t* T_hi; const uint16_t* T_lo;       // [kLoraParts][t][r]
    int rows_per_slab, nslab, chunks;
    float* partial; float* out; int transposed;
};
struct GradPair { GradProblem p[2]; };

template <int R16>
__global__ void __launch_bounds__(256)
lora_grad_kernel(GradPair pair, int64_t t) {
    constexpr int r = R16 * 16;
    constexpr int PSTR = r * 2 + 4;                       // bytes per token of a staged P tile (+4: disjoint banks)
    constexpr int QTILE = kGradTokens * kGradRowBytes, PTILE = kGradTokens * PSTR;
    constexpr int PV = kGradTokens * r / 8;               // 16-byte vectors of a P tile
    constexpr int PJ = (PV + 255) / 256;                  // ... per thread
    const GradProblem& pb = pair.p[blockIdx.z];
    if ((int)blockIdx.x >= pb.chunks || (int)blockIdx.y >= pb.nslab) return;
    const uint16_t* __restrict__ Q = pb.Q;
    const int64_t ldq = pb.ldq;
    const int c = pb.c;
    const uint16_t* __restrict__ T_hi = pb.T_hi;
    const uint16_t* __restrict__ T_lo = pb.T_lo;
    extern __shared__ __attribute__((aligned(16))) uint8_t grad_lds[];   // Q tiles [2], then P tiles [2][hi, lo]
    uint8_t* const qt = grad_lds;
    uint8_t* const pt = grad_lds + 2 * QTILE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int c0 = blockIdx.x * kGradCols;
    const int64_t t_pad = (t + kGradTokens - 1) / kGradTokens * kGradTokens;
    const int64_t i_begin = (int64_t)blockIdx.y * pb.rows_per_slab;
    const int64_t i_end = i_begin + pb.rows_per_slab < t_pad ? i_begin + pb.rows_per_slab : t_pad;

    // loaders.  Q: 64 rows x 256 bytes = 1024 vectors of 16 bytes, four per thread (rows tid / 16 + 16 h).
    // P: token tok, rank indices p0 .. p0 + 7 of each of the four arrays (hi / lo of the two contraction parts).
    const int ld_row = tid >> 4;
    int ld_col = c0 + (tid & 15) * 8;
    if (ld_col > c - 8) ld_col = c - 8;        // columns past the edge repeat valid data and are never stored
    struct TileRegs { u32x4 q[4]; u32x4 p[PJ][2 * kLoraParts]; };
    auto load_tile = [&](int64_t i0, TileRegs& tr) {
        u32x4 (&qreg)[4] = tr.q;
        u32x4 (&preg)[PJ][2 * kLoraParts] = tr.p;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            int64_t row = i0 + ld_row + 16 * h;
            if (row > t - 1) row = t - 1;      // tokens past the end repeat the last one; P is zero there
            qreg[h] = *reinterpret_cast<const u32x4*>(Q + row * ldq + ld_col);
        }
#pragma unroll
        for (int j = 0; j < PJ; ++j) {
            const int v = tid + 256 * j;
            const int tok = v / (r / 8), p0 = (v % (r / 8)) * 8;
            const int64_t i = i0 + tok;
#pragma unroll
            for (int part = 0; part < kLoraParts; ++part) {
                preg[j][2 * part] = preg[j][2 * part + 1] = (u32x4){0, 0, 0, 0};
                if (v < PV && i < t) {
                    const int64_t o = ((int64_t)part * t + i) * r + p0;
                    preg[j][2 * part] = *reinterpret_cast<const u32x4*>(T_hi + o);
                    preg[j][2 * part + 1] = *reinterpret_cast<const u32x4*>(T_lo + o);
                }
            }
        }
    };
    auto stage_tile = [&](int buf, const TileRegs& tr) {
        const u32x4 (&qreg)[4] = tr.q;
        const u32x4 (&preg)[PJ][2 * kLoraParts] = tr.p;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            uint8_t* dst = qt + buf * QTILE + (ld_row + 16 * h) * kGradRowBytes + (tid & 15) * 16;
            *reinterpret_cast<u32x2*>(dst) = (u32x2){qreg[h][0], qreg[h][1]};
            *reinterpret_cast<u32x2*>(dst + 8) = (u32x2){qreg[h][2], qreg[h][3]};
        }
#pragma unroll
        for (int j = 0; j < PJ; ++j) {
            const int v = tid + 256 * j;
            if (v >= PV) continue;
            const int tok = v / (r / 8), p0 = (v % (r / 8)) * 8;
            uint32_t hi2[4], lo2[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint32_t hpair = 0, lpair = 0;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    float sum = 0.0f;          // the parts in their order, each as hi + lo
#pragma unroll
                    for (int part = 0; part < kLoraParts; ++part) {
                        const uint32_t hw = preg[j][2 * part][w], lw = preg[j][2 * part + 1][w];
                        const float hf = __uint_as_float(half ? (hw & 0xFFFF0000u) : (hw << 16));
                        const float lf = __uint_as_float(half ? (lw & 0xFFFF0000u) : (lw << 16));
                        sum += hf + lf;
                    }
                    const uint32_t hi = grad_f32_to_bf16_rne(sum);
                    const uint32_t lo = grad_f32_to_bf16_rne(sum - __uint_as_float(hi << 16));
                    hpair |= hi << (16 * half);
                    lpair |= lo << (16 * half);
                }
                hi2[w] = hpair;
                lo2[w] = lpair;
            }
            uint32_t* dh = reinterpret_cast<uint32_t*>(pt + (buf * 2 + 0) * PTILE + tok * PSTR + p0 * 2);
            uint32_t* dl = reinterpret_cast<uint32_t*>(pt + (buf * 2 + 1) * PTILE + tok * PSTR + p0 * 2);
#pragma unroll
            for (int w = 0; w < 4; ++w) { dh[w] = hi2[w]; dl[w] = lo2[w]; }
        }
    };
    // eight tokens (rows row0 .. row0 + 7 of a staged tile) of one 2-byte column, as an MFMA operand
    auto gather8 = [&](const uint8_t* base, int stride) {
        u32x4 q;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const uint32_t lo = *reinterpret_cast<const uint16_t*>(base + (2 * jj) * stride);
            const uint32_t hi = *reinterpret_cast<const uint16_t*>(base + (2 * jj + 1) * stride);
            q[jj] = lo | (hi << 16);
        }
        return q;
    };

    f32x4 acc[R16][2];
#pragma unroll
    for (int b = 0; b < R16; ++b)
#pragma unroll
        for (int f = 0; f < 2; ++f) acc[b][f] = (f32x4){0.f, 0.f, 0.f, 0.f};

    auto multiply_tile = [&](int buf) {
#pragma unroll
        for (int sub = 0; sub < kGradTokens / 32; ++sub) {
            const int row0 = sub * 32 + g * 8;
            u32x4 ah[R16], al[R16];
#pragma unroll
            for (int b = 0; b < R16; ++b) {
                ah[b] = gather8(pt + (buf * 2 + 0) * PTILE + row0 * PSTR + (b * 16 + n) * 2, PSTR);
                al[b] = gather8(pt + (buf * 2 + 1) * PTILE + row0 * PSTR + (b * 16 + n) * 2, PSTR);
            }
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                // second operand: tokens row0 .. row0 + 7 of column c0 + 16 (2 wave + f) + n
                const u32x4 q = gather8(qt + buf * QTILE + row0 * kGradRowBytes + ((wave * 2 + f) * 16 + n) * 2,
                                        kGradRowBytes);
#pragma unroll
                for (int b = 0; b < R16; ++b) {
                    acc[b][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ah[b]),
                                                                        __builtin_bit_cast(bf16x8, q), acc[b][f], 0, 0, 0);
                    acc[b][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, al[b]),
                                                                        __builtin_bit_cast(bf16x8, q), acc[b][f], 0, 0, 0);
                }
            }
        }
    };
    // Two tiles are in flight from global memory at any time (two register sets used in turn; the loop body covers
    // two tiles so that which set a tile uses is fixed at compile time), a third is being multiplied out of LDS.
    // One barrier per tile: the barrier of the next tile separates this tile's gathers from the stores that reuse
    // its LDS buffer two tiles on.
    TileRegs ra, rb;
    load_tile(i_begin, ra);
    if (i_begin + kGradTokens < i_end) load_tile(i_begin + kGradTokens, rb);
    for (int64_t i0 = i_begin; i0 < i_end; i0 += 2 * kGradTokens) {
        stage_tile(0, ra);
        __syncthreads();
        if (i0 + 2 * kGradTokens < i_end) load_tile(i0 + 2 * kGradTokens, ra);
        multiply_tile(0);
        if (i0 + kGradTokens < i_end) {
            stage_tile(1, rb);
            __syncthreads();
            if (i0 + 3 * kGradTokens < i_end) load_tile(i0 + 3 * kGradTokens, rb);
            multiply_tile(1);
        }
    }
    // element v of lane (n, g) is G[16 b + 4 g + v][c0 + 16 (2 wave + f) + n]
    float* out = pb.partial + (int64_t)blockIdx.y * r * c;
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

size_t lora_grad_lds_bytes(int32_t r) {
    return 2 * (size_t)kGradTokens * kGradRowBytes + 4 * (size_t)kGradTokens * (r * 2 + 4);
}

// Both gradient products of a layer in one launch:
//   dA^T [r x c_in] = P1^T X (stored transposed as dA [c_in x r]),   dB [r x c_out] = P2^T dY
// with P1 = T1 (the down-projection of dY) and P2 = T2 (the down-projection of X), each given as the hi / lo parts
// [kLoraParts x t x r] that launch_lora_down writes.
hipError_t launch_lora_grad_pair(const uint16_t* X, int64_t ldx, int64_t c_in, const uint16_t* T1_hi,
                                 const uint16_t* T1_lo, float* partial_a, float* dA, const uint16_t* dY, int64_t lddy,
                                 int64_t c_out, const uint16_t* T2_hi, const uint16_t* T2_lo, float* partial_b,
                                 float* dB, int64_t t, int32_t r, hipStream_t stream) {
    ProfScope prof(K_LORA_GRAD, stream);
    GradPair pair;
    auto fill = [&](GradProblem& p, const uint16_t* Q, int64_t ldq, int64_t c, const uint16_t* hi, const uint16_t* lo,
                    float* partial, float* out, int transposed) {
        p.Q = Q; p.ldq = ldq; p.c = (int)c; p.T_hi = hi; p.T_lo = lo;
        lora_grad_plan(t, c, &p.nslab, &p.rows_per_slab);
        p.chunks = lora_grad_chunks(c);
        p.partial = partial; p.out = out; p.transposed = transposed;
    };
    fill(pair.p[0], X, ldx, c_in, T1_hi, T1_lo, partial_a, dA, 1);
    fill(pair.p[1], dY, lddy, c_out, T2_hi, T2_lo, partial_b, dB, 0);
    const int gx = pair.p[0].chunks > pair.p[1].chunks ? pair.p[0].chunks : pair.p[1].chunks;
    const int gy = pair.p[0].nslab > pair.p[1].nslab ? pair.p[0].nslab : pair.p[1].nslab;
    dim3 grid((unsigned)gx, (unsigned)gy, 2);
    const size_t lds = lora_grad_lds_bytes(r);
#define QUAFF_GRAD(N)                                                                                                 \
    case N: {                                                                                                         \
        auto kern = lora_grad_kernel<N>;                                                                              \
        hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                      \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                    \
        if (ea != hipSuccess) return ea;                                                                              \
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, pair, t);                                              \
    } break;
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
