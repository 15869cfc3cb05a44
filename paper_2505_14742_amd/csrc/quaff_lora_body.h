// Device code of the LoRA down-projection, shared by its stand-alone launch and by the launch that runs it next to
// the quantizer (see quaff_lora.hip for the description).
#pragma once
#include "quaff_internal.h"

namespace quaff {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kLoraWaves = 16;
// contraction steps whose loads are issued together (latency hiding); even.  With the contraction-contiguous factor
// and r = 16 a wavefront's whole slice of a 9216-wide row (ten steps) is in flight at once.
template <int R16, bool L_RC, int RG = 1> struct LoraUnroll {
    static constexpr int value = RG == 2 ? 2 : (L_RC && R16 == 1) ? 10 : 6;
};
// Row groups of 16 rows per workgroup.  From rank 48 on a workgroup takes 32 rows: every workgroup fetches its share of
// L (c x r against 16 x c of rows: four times the rows' bytes at rank 64), and its 128 registers per lane leave room
// for one 16-wavefront workgroup per compute unit only, so 16-row workgroups would also need two rounds at 4096 rows.
// Measured at rank 64, 4096 rows: abs-max + down-projection launch 43 -> 30 us at 4096 columns, 86 -> 64 us at 11008;
// backward quantizer + down-projection launch 44 -> 30 us and 96 -> 80 us.
constexpr int lora_row_groups(int R16) { return R16 >= 3 ? 2 : 1; }
inline int lora_rows_per_block(int r) { return 16 * lora_row_groups(r / 16); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// R16 = r / 16 column blocks of T.  L_RC: L is [r x c] (contraction-contiguous) else [c x r].  RG = row groups of 16 rows.
// Work of one workgroup (64 * kLoraWaves threads): `bx` < row_blocks is its block of 16 RG rows and `by` its part of the
// contraction range; workgroups bx >= row_blocks (nbx in all, by = 0 only) write the transposed copy.
template <int R16, bool L_RC, int RG = 1>
__device__ __forceinline__ void lora_down_body(int bx, int by, int nbx, const uint16_t* __restrict__ X, int64_t t, int c,
                                               int64_t ldx, const uint16_t* __restrict__ L, float scale,
                                               uint16_t* __restrict__ T_hi, uint16_t* __restrict__ T_lo, int row_blocks,
                                               const uint16_t* __restrict__ tr_src, uint16_t* __restrict__ tr_dst,
                                               int64_t tr_rows, int64_t tr_cols) {
    static_assert(RG == 1 || L_RC, "several row groups only with a contraction-contiguous factor");
    constexpr int r = R16 * 16;
    constexpr int NT = 64 * kLoraWaves;
    constexpr int kLoraUnroll = LoraUnroll<R16, L_RC, RG>::value;
    constexpr int TROW = 40;                       // padded row (in bf16) of the transposed slice: 32 + 8
    if (bx >= row_blocks) {
        if (by != 0) return;
        // transposed copy: dst [cols x rows] <- src [rows x cols]
        int64_t total = tr_rows * tr_cols;
        int64_t nb = nbx - row_blocks;
        for (int64_t e = ((int64_t)bx - row_blocks) * NT + threadIdx.x; e < total; e += nb * NT) {
            int64_t col = e / tr_rows, row = e % tr_rows;
            tr_dst[e] = tr_src[row * tr_cols + col];
        }
        return;
    }
    __shared__ float red[kLoraWaves][R16][64][4];
    __shared__ __attribute__((aligned(16))) uint16_t lt[L_RC ? 1 : kLoraWaves][L_RC ? 1 : r][L_RC ? 8 : TROW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
    bool live[RG];
    const uint16_t* xrow[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
        const int64_t row = ((int64_t)bx * RG + rg) * 16 + m;
        live[rg] = row < t;
        xrow[rg] = X + (live[rg] ? row : 0) * ldx;
    }

    f32x4 acc[RG][R16];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg)
#pragma unroll
        for (int b = 0; b < R16; ++b) acc[rg][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // each wavefront owns one contiguous slice of the contraction range (kw columns), walked in 32-column steps
    // this workgroup's part of the contraction range, then this wavefront's slice of it
    // (multiples of 64 columns = 128 bytes, so that a pair of steps reads whole cache lines, see below)
    const int cp = ((c + kLoraParts * 64 - 1) / (kLoraParts * 64)) * 64;
    const int cbeg = by * cp, cend = cbeg + cp < c ? cbeg + cp : c;
    const int kw = ((cend - cbeg + kLoraWaves * 64 - 1) / (kLoraWaves * 64)) * 64;
    const int kbeg = cbeg + wave * kw, kend = kbeg + kw < cend ? kbeg + kw : cend;
    T_hi += (int64_t)by * t * r;
    T_lo += (int64_t)by * t * r;
    for (int kk0 = kbeg; kk0 < kend; kk0 += 32 * kLoraUnroll) {
        u32x4 xa[kLoraUnroll][RG], lb[kLoraUnroll][R16];
        // all global loads of the batch first
#pragma unroll
        for (int u = 0; u < kLoraUnroll; ++u) {
            // Two consecutive steps share 64 columns: lane group g takes columns 16 g .. 16 g + 7 in the even step
            // and 16 g + 8 .. 16 g + 15 in the odd one (any assignment of contraction indices to MFMA slots is
            // valid as long as both operands use it), so the four groups of a row read one whole 128-byte line
            // per step pair instead of two half lines.
            const int k0 = kk0 + (u >> 1) * 64 + (u & 1) * 8;
            const int k = k0 + g * 16;         // this lane's eight contraction indices
            // loads are unconditional (address clamped into the row) so that the whole batch is in flight together;
            // a step past the end contributes zero because its x fragment is cleared
            const int kc = k < kend ? k : c - 8;
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                xa[u][rg] = *reinterpret_cast<const u32x4*>(xrow[rg] + kc);
                if (!(live[rg] && k < kend)) xa[u][rg] = (u32x4){0, 0, 0, 0};
            }
            if (L_RC) {
#pragma unroll
                for (int b = 0; b < R16; ++b)
                    lb[u][b] = *reinterpret_cast<const u32x4*>(L + (int64_t)(b * 16 + m) * c + kc);
            } else {
                // L[k0 .. k0+32) x r arrives as 16-byte vectors along r; kept in lb[u][*] until it is transposed
                constexpr int VEC = 32 * r / 8;
#pragma unroll
                for (int b = 0; b < R16; ++b) {   // VEC = 64 * R16: one vector per lane per b
                    int v = b * 64 + lane;
                    int kk = v / (r / 8), p0 = (v % (r / 8)) * 8;
                    const int km = k0 + (kk >> 3) * 16 + (kk & 7);   // slot kk of the step holds this column
                    const int kr = km < c ? km : c - 1;
                    lb[u][b] = *reinterpret_cast<const u32x4*>(L + (int64_t)kr * r + p0);
                }
                (void)VEC;
            }
        }
#pragma unroll
        for (int u = 0; u < kLoraUnroll; ++u) {
            if (!L_RC) {
                // transpose this step's slice through the wavefront's LDS piece: lt[p][kk]
#pragma unroll
                for (int b = 0; b < R16; ++b) {
                    int v = b * 64 + lane;
                    int kk = v / (r / 8), p0 = (v % (r / 8)) * 8;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        lt[wave][p0 + 2 * w][kk] = (uint16_t)(lb[u][b][w] & 0xFFFFu);
                        lt[wave][p0 + 2 * w + 1][kk] = (uint16_t)(lb[u][b][w] >> 16);
                    }
                }
#pragma unroll
                for (int b = 0; b < R16; ++b)
                    lb[u][b] = *reinterpret_cast<const u32x4*>(&lt[wave][b * 16 + m][g * 8]);
            }
#pragma unroll
            for (int rg = 0; rg < RG; ++rg)
#pragma unroll
                for (int b = 0; b < R16; ++b)
                    acc[rg][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[u][rg]),
                                                                         __builtin_bit_cast(bf16x8, lb[u][b]), acc[rg][b],
                                                                         0, 0, 0);
        }
    }
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) {
        if (rg > 0) __syncthreads();               // the sums over the previous row group have been read
#pragma unroll
        for (int b = 0; b < R16; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][b][lane][v] = acc[rg][b][v];
        __syncthreads();
        // fixed-order sum over the wavefronts; element v of lane (m, g) is T[row0 + 4 g + v][16 b + m]
        for (int e = threadIdx.x; e < R16 * 64 * 4; e += NT) {
            int v = e & 3, ln = (e >> 2) & 63, b = e >> 8;
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < kLoraWaves; ++w) s += red[w][b][ln][v];
            s = s * scale;
            int64_t orow = ((int64_t)bx * RG + rg) * 16 + (ln >> 4) * 4 + v;
            if (orow < t) {
                uint32_t hi = f32_to_bf16_rne(s);
                float rest = s - __uint_as_float(hi << 16);
                T_hi[orow * r + b * 16 + (ln & 15)] = (uint16_t)hi;
                T_lo[orow * r + b * 16 + (ln & 15)] = (uint16_t)f32_to_bf16_rne(rest);
            }
        }
    }
}

}  // namespace quaff
