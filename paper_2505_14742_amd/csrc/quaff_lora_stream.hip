// LoRA down-projection T = scale X L for long inputs (many 16-row blocks), rank 16: the persistent form of
// lora_down_kernel (quaff_lora.hip, same slices, same order of the sums, so the same bits).
//
// lora_down_kernel gives every 16-row block a workgroup of its own, and every workgroup fetches its share of L: at
// rank 16 that is as many bytes as the rows themselves (16 rows x c against c x 16), so with thousands of row blocks
// the cache path carries twice the traffic of X and the kernel runs at well under half the copy rate.  Here one
// workgroup per compute unit and contraction part keeps its wavefronts' fragments of L in registers for the whole
// launch (a [c x r] factor is transposed through LDS once, not once per row block) and walks the row blocks
// bx, bx + gridDim.x, ...; the next rows are requested before the current ones are multiplied, so X streams.
//
// With COLMAX the same pass also yields the abs-max of the outlier columns (Eq. 8 of the paper, max_i |X[i, O_k]|):
// the rows are in registers anyway; a lane whose eight columns of a step hold an outlier (a per-lane bit mask, built
// once from a column -> outlier table in LDS) raises that outlier's maximum in LDS.  Workgroup (bx, part) writes the
// partial maxima part[bx][k] of the outlier columns inside its part of the contraction range, which is the slab
// layout of the stand-alone abs-max kernel with gridDim.x slabs.
#include "quaff_lora_body.h"

namespace quaff {

struct LoraStreamArgs {
    const uint16_t* X; int64_t t; int c; int64_t ldx;
    const uint16_t* L; float scale;
    uint16_t* T_hi; uint16_t* T_lo; int row_blocks;
    const uint16_t* tr_src; uint16_t* tr_dst; int64_t tr_rows, tr_cols;
    const int32_t* O; int n; uint32_t* part; const float* s_O; float* s_prev;
};

constexpr int kStreamMaxOutliers = 1024;

// NS = 32-column contraction steps per wavefront (even), HB = steps whose rows are requested together (NS % HB == 0),
// PF = request the next unit's rows before this unit is multiplied.
template <int NS, int HB, bool PF, bool L_RC, bool COLMAX>
__global__ void __launch_bounds__(64 * kLoraWaves)
lora_stream_kernel(LoraStreamArgs a) {
    constexpr int r = 16;
    constexpr int NT = 64 * kLoraWaves;
    constexpr int TROW = 40;
    constexpr int NU = NS / HB;
    static_assert(NS % 2 == 0 && NS % HB == 0, "steps come in pairs that share whole cache lines");
    // The wavefronts' partial products of a row block; two copies used in turn, so that one barrier per row block
    // is enough (the barrier of block i + 1 separates the sums over copy i % 2 from the stores of block i + 2).
    // The transposition buffer of a [c x r] factor is only needed before the first row block and shares the space.
    __shared__ __attribute__((aligned(16))) float red_store[2 * kLoraWaves * 64 * 4];
    typedef float RedCopy[kLoraWaves][64][4];
    RedCopy* red2 = reinterpret_cast<RedCopy*>(red_store);
    typedef uint16_t LtPiece[r][TROW];
    LtPiece* lt = reinterpret_cast<LtPiece*>(red_store);
    static_assert(sizeof(LtPiece) * kLoraWaves <= sizeof(red_store), "transposition buffer fits");
    __shared__ uint16_t colslot[COLMAX ? NS * 32 * kLoraWaves : 1];     // column of this part -> outlier number
    __shared__ uint32_t cmx[COLMAX ? kStreamMaxOutliers : 1];          // |x| maxima (bf16 magnitude bits)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int bx = blockIdx.x, by = blockIdx.y, nbx = gridDim.x;
    const int c = a.c;
    const int64_t t = a.t;

    // the transposed copy some callers want next to the product (all workgroups share it)
    if (a.tr_src) {
        const int64_t total = a.tr_rows * a.tr_cols;
        for (int64_t e = ((int64_t)by * nbx + bx) * NT + threadIdx.x; e < total; e += (int64_t)nbx * kLoraParts * NT) {
            const int64_t col = e / a.tr_rows, row = e % a.tr_rows;
            a.tr_dst[e] = a.tr_src[row * a.tr_cols + col];
        }
    }

    // this workgroup's part of the contraction range and this wavefront's slice of it, as in lora_down_body
    const int cp = ((c + kLoraParts * 64 - 1) / (kLoraParts * 64)) * 64;
    const int cbeg = by * cp, cend = cbeg + cp < c ? cbeg + cp : c;
    const int kw = ((cend - cbeg + kLoraWaves * 64 - 1) / (kLoraWaves * 64)) * 64;
    const int kbeg = cbeg + wave * kw, kend = kbeg + kw < cend ? kbeg + kw : cend;
    auto col_of = [&](int s) { return kbeg + (s >> 1) * 64 + (s & 1) * 8 + g * 16; };   // this lane's eight columns of step s

    uint32_t msk[(NS + 3) / 4];
    if (COLMAX) {
        if (bx == 0 && by == 0)
            for (int k = threadIdx.x; k < a.n; k += NT) a.s_prev[k] = a.s_O[k];
        for (int i = threadIdx.x; i < NS * 32 * kLoraWaves; i += NT) colslot[i] = 0xFFFFu;
        for (int k = threadIdx.x; k < a.n; k += NT) cmx[k] = 0u;
        __syncthreads();
        for (int k = threadIdx.x; k < a.n; k += NT) {
            const int col = a.O[k];
            if (col >= cbeg && col < cend) colslot[col - cbeg] = (uint16_t)k;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < (NS + 3) / 4; ++i) msk[i] = 0u;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int k = col_of(s);
            uint32_t bits = 0u;
            if (k < kend) {
#pragma unroll
                for (int e = 0; e < 8; ++e) bits |= (colslot[k + e - cbeg] != 0xFFFFu ? 1u : 0u) << e;   // c is a multiple of 16
            }
            msk[s >> 2] |= bits << ((s & 3) * 8);
        }
    }

    // this wavefront's fragments of L, kept for the whole launch (all global loads first: one memory round trip)
    u32x4 lb[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int k0 = kbeg + (s >> 1) * 64 + (s & 1) * 8;
        const int k = k0 + g * 16;
        const int kc = k < kend ? k : c - 8;
        if (L_RC) {
            lb[s] = *reinterpret_cast<const u32x4*>(a.L + (int64_t)m * c + kc);
        } else {
            // L[k0 .. k0+32) x r arrives as 16-byte vectors along r
            const int kk = lane / (r / 8), p0 = (lane % (r / 8)) * 8;
            const int km = k0 + (kk >> 3) * 16 + (kk & 7);           // slot kk of the step holds this column
            const int kr = km < c ? km : c - 1;
            lb[s] = *reinterpret_cast<const u32x4*>(a.L + (int64_t)kr * r + p0);
        }
    }
    if (!L_RC) {
        // ... and is transposed through the wavefront's LDS piece, step by step
        const int kk = lane / (r / 8), p0 = (lane % (r / 8)) * 8;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                lt[wave][p0 + 2 * w][kk] = (uint16_t)(lb[s][w] & 0xFFFFu);
                lt[wave][p0 + 2 * w + 1][kk] = (uint16_t)(lb[s][w] >> 16);
            }
            lb[s] = *reinterpret_cast<const u32x4*>(&lt[wave][m][g * 8]);
        }
    }

    auto load_unit = [&](int rb, int h, u32x4 (&dst)[HB]) {
        const int64_t row = (int64_t)rb * 16 + m;
        const bool live = rb < a.row_blocks && row < t;
        const uint16_t* xrow = a.X + (live ? row : 0) * a.ldx;
#pragma unroll
        for (int uu = 0; uu < HB; ++uu) {
            const int k = col_of(h * HB + uu);
            const int kc = k < kend ? k : c - 8;          // unconditional loads, so that the whole unit is in flight together
            dst[uu] = *reinterpret_cast<const u32x4*>(xrow + kc);
        }
    };
    // Rows past the end and columns past the slice are cleared when a unit is used, not when it is requested: a
    // select on the loaded value right behind the load would make the wavefront wait for it there and then, and
    // nothing would be in flight while the previous unit is multiplied.
    auto clear_dead = [&](int rb, int h, u32x4 (&v)[HB]) {
        const bool live = (int64_t)rb * 16 + m < t;
#pragma unroll
        for (int uu = 0; uu < HB; ++uu)
            if (!(live && col_of(h * HB + uu) < kend)) v[uu] = (u32x4){0, 0, 0, 0};
    };

    if (!L_RC) __syncthreads();          // the transposition buffer becomes the first copy of the partial products
    uint16_t* T_hi = a.T_hi + (int64_t)by * t * r;
    uint16_t* T_lo = a.T_lo + (int64_t)by * t * r;
    // Units of HB steps are requested one unit ahead into two register buffers used in turn; the loop body covers an
    // even number of units (two row blocks when a block has an odd number of units), so that the buffer of every
    // unit and the fragments of L it meets are fixed at compile time and no loaded value is moved between registers
    // (a move would wait for the load).
    constexpr int BPI = (NU % 2) ? 2 : 1;          // row blocks per loop iteration
    u32x4 xb[2][HB];
    if (PF) load_unit(bx, 0, xb[0]);
    int copy = 0;
    for (int rb0 = bx; rb0 < a.row_blocks; rb0 += BPI * nbx) {
#pragma unroll
        for (int bb = 0; bb < BPI; ++bb) {
            const int rb = rb0 + bb * nbx;             // may lie past the last block: such a block multiplies zeros
            f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int h = 0; h < NU; ++h) {
                const int cur = PF ? ((bb * NU + h) & 1) : 0;
                u32x4 (&xa)[HB] = xb[cur];
                if (PF) {
                    if (h + 1 < NU) load_unit(rb, h + 1, xb[cur ^ 1]);
                    else load_unit(rb + nbx, 0, xb[cur ^ 1]);
                } else {
                    load_unit(rb, h, xa);
                }
                clear_dead(rb, h, xa);
                if (COLMAX) {
#pragma unroll
                    for (int uu = 0; uu < HB; ++uu) {
                        const int s = h * HB + uu;
                        const uint32_t mb = (msk[s >> 2] >> ((s & 3) * 8)) & 0xFFu;
                        if (mb) {                                   // rare: few lanes hold an outlier column
                            const int k = col_of(s) - cbeg;
                            uint32_t bits = mb;
                            while (bits) {
                                const int e = __builtin_ctz(bits);
                                bits &= bits - 1;
                                const uint32_t lo2 = (e & 4) ? xa[uu][2] : xa[uu][0], hi2 = (e & 4) ? xa[uu][3] : xa[uu][1];
                                const uint32_t pair = (e & 2) ? hi2 : lo2;
                                atomicMax(&cmx[colslot[k + e]], (pair >> ((e & 1) * 16)) & 0x7FFFu);
                            }
                        }
                    }
                }
#pragma unroll
                for (int uu = 0; uu < HB; ++uu)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[uu]),
                                                                  __builtin_bit_cast(bf16x8, lb[h * HB + uu]), acc, 0, 0, 0);
            }
            RedCopy& red = red2[copy];
            copy ^= 1;
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][lane][v] = acc[v];
            __syncthreads();
            // fixed-order sum over the wavefronts; element v of lane (m, g) is T[row0 + 4 g + v][m]
            if (threadIdx.x < 256) {
                const int v = threadIdx.x & 3, ln = threadIdx.x >> 2;
                float s = 0.0f;
#pragma unroll
                for (int w = 0; w < kLoraWaves; ++w) s += red[w][ln][v];
                s = s * a.scale;
                const int64_t orow = (int64_t)rb * 16 + (ln >> 4) * 4 + v;
                if (orow < t) {
                    const uint32_t hi = f32_to_bf16_rne(s);
                    const float rest = s - __uint_as_float(hi << 16);
                    T_hi[orow * r + (ln & 15)] = (uint16_t)hi;
                    T_lo[orow * r + (ln & 15)] = (uint16_t)f32_to_bf16_rne(rest);
                }
            }
        }
    }
    if (COLMAX) {
        __syncthreads();

        for (int k = threadIdx.x; k < a.n; k += NT) {
            const int col = a.O[k];
            if (col >= cbeg && col < cend) a.part[(int64_t)bx * a.n + k] = cmx[k] << 16;      // |x| as fp32 bits
        }
    }
}

// 32-column steps of a wavefront's slice of the first contraction part (the longer one)
static int stream_steps(int64_t c) {
    const int64_t cp = ((c + kLoraParts * 64 - 1) / (kLoraParts * 64)) * 64;
    const int64_t first = cp < c ? cp : c;
    const int64_t kw = ((first + kLoraWaves * 64 - 1) / (kLoraWaves * 64)) * 64;
    return (int)(kw / 32);
}

// Rank 16, at least two 16-row blocks per workgroup, slices short enough to keep their fragments of L in registers.
bool lora_stream_applies(int32_t r, int64_t t, int64_t c, int32_t n_colmax) {
    if (r != 16 || c < 64 || c % 16 != 0 || n_colmax > kStreamMaxOutliers) return false;
    if ((t + 15) / 16 < 2 * (int64_t)scale_update_blocks(t)) return false;
    return stream_steps(c) <= 14;
}

int lora_stream_row_groups(int64_t t) { return scale_update_blocks(t); }

hipError_t launch_lora_stream(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const uint16_t* L, bool L_is_r_by_c,
                              float scale, uint16_t* T_hi, uint16_t* T_lo, const uint16_t* tr_src, uint16_t* tr_dst,
                              int64_t tr_rows, int64_t tr_cols, const int32_t* O, int32_t n, uint32_t* part,
                              const float* s_O, float* s_prev, hipStream_t stream) {
    LoraStreamArgs a{X, t, (int)c, ldx, L, scale, T_hi, T_lo, (int)((t + 15) / 16), tr_src, tr_dst, tr_rows, tr_cols,
                     O, n, part, s_O, s_prev};
    const dim3 grid((unsigned)lora_stream_row_groups(t), kLoraParts), block(64 * kLoraWaves);
    const bool colmax = n > 0 && O && part;
    if (colmax && L_is_r_by_c) return hipErrorInvalidValue;   // the abs-max rides on the forward factor A [c x r] only
    const int ns = stream_steps(c);
#define QUAFF_LS4(NS, HB, PF, RC, CM)                                                                        \
    hipLaunchKernelGGL((lora_stream_kernel<NS, HB, PF, RC, CM>), grid, block, 0, stream, a)
#define QUAFF_LS(NS, HB, PF)                                                                                 \
    {                                                                                                        \
        if (L_is_r_by_c) QUAFF_LS4(NS, HB, PF, true, false);                                                 \
        else if (colmax) QUAFF_LS4(NS, HB, PF, false, true);                                                 \
        else QUAFF_LS4(NS, HB, PF, false, false);                                                            \
    }
    if (ns <= 4) QUAFF_LS(4, 4, true)
    else if (ns <= 6) QUAFF_LS(6, 6, true)
    else if (ns <= 8) QUAFF_LS(8, 4, true)
    else if (ns <= 10) QUAFF_LS(10, 2, true)
    else if (ns <= 12) QUAFF_LS(12, 3, true)
    else QUAFF_LS(14, 2, true)
#undef QUAFF_LS
#undef QUAFF_LS4
    return hipGetLastError();
}

}  // namespace quaff
