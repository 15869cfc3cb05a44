// Backward-pass launch that runs the per-token quantizer of dY * delta_w and the LoRA down-projection dY B^T side by
// side: both only read dY, neither fills the chip at a few thousand tokens, and each launch on its own costs several
// microseconds of ramp-up and drain.  Two forms:
//   quant_lora_kernel        the first workgroups of the grid take the down-projection (they are the longer ones),
//                            the rest quantize rows; the two roles share nothing but the launch;
//   quant_lora_rows8_kernel  (rank 16, rows of up to 5120 columns) one pass over dY: the registers that hold a row
//                            block as MFMA operands are also what the quantizer works on; persistent workgroups.
#include "quaff_lora_body.h"
#include "quaff_quant_body.h"

namespace quaff {

template <int R16, int TPR, int NV>
__global__ void __launch_bounds__(64 * kLoraWaves)
quant_lora_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const float* __restrict__ cs,
                  int8_t* __restrict__ Xq, float* __restrict__ delta, const uint16_t* __restrict__ L, float scale,
                  uint16_t* __restrict__ T_hi, uint16_t* __restrict__ T_lo, int lora_row_blocks) {
    constexpr int RG = lora_row_groups(R16);                 // 16-row groups per down-projection workgroup
    const int lora_blocks = lora_row_blocks * kLoraParts;
    if ((int)blockIdx.x < lora_blocks)
        lora_down_body<R16, true, RG>(blockIdx.x % lora_row_blocks, blockIdx.x / lora_row_blocks, lora_row_blocks, X, t, c,
                                      ldx, L, scale, T_hi, T_lo, lora_row_blocks, nullptr, nullptr, 0, 0);
    else {
        // The hardware deals consecutive workgroups to the eight XCDs in turn and every XCD has its own L2: the
        // quantizing workgroups of a row block are renumbered so that they land on the XCD whose down-projection
        // workgroups (index = row block of 16 RG rows, same residue modulo 8) read the same rows at about the same time.
        constexpr int QPG = 16 / ((64 * kLoraWaves) / TPR);   // quantizing workgroups per 16-row block (1 or 4)
        const int local = blockIdx.x - lora_blocks;
        const int xcd = local & 7, m = local >> 3;
        const int mq = m / QPG;
        const int rb = ((mq / RG) * 8 + xcd) * RG + mq % RG;   // 16-row block
        quant_rows_body<64 * kLoraWaves, TPR, NV>(rb * QPG + m % QPG, X, t, c, ldx, cs, nullptr, 0, 0, Xq, delta,
                                                  nullptr);
    }
}

// One pass over dY for both results.  A workgroup of 16 wavefronts owns 8 rows at a time; wavefront w holds its slice
// of the contraction range in registers, 64 columns per step: lane (m, g) keeps row m % 8, columns 32 (m / 8) + 8 g .. + 7
// of the step, so every lane holds data and a row's 64 columns are one 128-byte line.  As the A operand of the 16-row
// MFMA this is rows 0..7 over the first 32 columns of the step stacked on the same rows over the second 32; two MFMAs
// per step, one with each half of L as the B operand, leave the first half's products in result rows 0..7 of the one
// and the second half's in rows 8..15 of the other (the remaining result rows are products of mismatched halves and are
// dropped).  The same registers then feed the quantizer, once the row maxima have been exchanged through LDS.
// Wavefronts 0-7 and 8-15 produce the two parts of T.  NSTEP = steps per wavefront; the host picks the smallest
// instantiation with 8 * 64 * NSTEP >= cp.
// The workgroups are persistent: a wavefront's slice of L (NSTEP x 2 operand fragments) and the LDS copy of the column
// scales are fetched once and stay, and the rows of the workgroup's next 8-row group are requested before the current
// group is worked on, so that with many rows the kernel streams dY instead of paying a memory round trip per phase.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// RESIDENT = false: rows too long to keep a slice of L and a second group of rows in registers; L is fetched (from L2,
// where it stays) a few steps at a time for every group and the next group's rows are not requested ahead.
template <int R16, int NSTEP, bool RESIDENT = true>
__global__ void __launch_bounds__(64 * kLoraWaves)
quant_lora_rows8_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const float* __restrict__ cs,
                        int8_t* __restrict__ Xq, float* __restrict__ delta, const uint16_t* __restrict__ L, float scale,
                        uint16_t* __restrict__ T_hi, uint16_t* __restrict__ T_lo, int ngroups) {
    static_assert(kLoraParts == 2 && kLoraWaves == 16, "two parts of eight wavefronts each");
    constexpr int r = R16 * 16;
    __shared__ float red[kLoraWaves][R16][32][4];
    __shared__ float rmax[kLoraWaves][8];
    // The eight rows of a wavefront share their column scales, so a scale vector fetched from global memory would be
    // requested by eight lanes at once, twice per element (maximum pass, code pass): the texture path would then
    // carry several times the traffic of dY itself.  The workgroup keeps one copy of cs in LDS instead.
    extern __shared__ __attribute__((aligned(16))) float cs_copy[];   // [c], then the wavefronts' code rows
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, g = lane >> 4;
    constexpr int PS = NSTEP > 9 ? (NSTEP + 1) / 2 : NSTEP;      // steps whose codes are staged together
    char* cw = reinterpret_cast<char*>(cs_copy) + (((size_t)c * 4 + 255) & ~(size_t)255) + wave * (8 * PS * 64);

    const int part = wave >> 3;
    const int cp = ((c + kLoraParts * 64 - 1) / (kLoraParts * 64)) * 64;
    const int cbeg = part * cp, cend = cbeg + cp < c ? cbeg + cp : c;
    const int kw = ((cp + 8 * 64 - 1) / (8 * 64)) * 64;
    const int kbeg = cbeg + (wave & 7) * kw, kend = kbeg + kw < cend ? kbeg + kw : cend;

    // this lane's eight columns of step u, and the eight columns of L it supplies for the step's first / second half
    auto col_of = [&](int u) { return kbeg + u * 64 + (m >> 3) * 32 + g * 8; };
    auto lcol_of = [&](int u, int half) { return kbeg + u * 64 + half * 32 + g * 8; };
    auto load_rows = [&](int grp, u32x4 (&dst)[NSTEP]) {
        const int64_t row = (int64_t)grp * 8 + (m & 7);
        const bool live = grp < ngroups && row < t;
        const uint16_t* xrow = X + (live ? row : 0) * ldx;
#pragma unroll
        for (int u = 0; u < NSTEP; ++u) {
            const int k = col_of(u);
            dst[u] = (u32x4){0, 0, 0, 0};
            if (live && k < kend) dst[u] = *reinterpret_cast<const u32x4*>(xrow + k);
        }
    };
    // The next group's rows are requested ahead only where the registers allow it without spilling (three steps);
    // with five steps the version without is 4 % faster (16384 x 5120: 75.8 against 78.8 us) and writes no scratch.
    constexpr bool PF = RESIDENT && NSTEP <= 3;
    u32x4 xa[NSTEP], xn[NSTEP];                    // (xn costs no registers when PF is false)
    load_rows(blockIdx.x, xa);
    constexpr int BU = NSTEP > 9 ? 2 : 3;          // RESIDENT = false: steps whose fragments of L are in flight together
    constexpr int LSTEPS = RESIDENT ? NSTEP : BU;
    u32x4 lb[LSTEPS][2][R16];
    auto load_l = [&](int u0) {
#pragma unroll
        for (int uu = 0; uu < LSTEPS; ++uu)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int k = lcol_of(u0 + uu, h), kc = k < kend ? k : c - 8;
#pragma unroll
                for (int b = 0; b < R16; ++b) {
                    lb[uu][h][b] = (u32x4){0, 0, 0, 0};      // columns past the slice contribute nothing
                    if (u0 + uu < NSTEP) {
                        const u32x4 v = *reinterpret_cast<const u32x4*>(L + (int64_t)(b * 16 + m) * c + kc);
                        if (k < kend) lb[uu][h][b] = v;
                    }
                }
            }
    };
    if (RESIDENT) load_l(0);
    for (int i = threadIdx.x * 4; i < c; i += 64 * kLoraWaves * 4)     // c is a multiple of 16
        *reinterpret_cast<f32x4*>(cs_copy + i) = *reinterpret_cast<const f32x4*>(cs + i);
    __syncthreads();
    const lds_float* csl = (const lds_float*)cs_copy;

    for (int grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
        const int64_t row = (int64_t)grp * 8 + (m & 7);
        const bool live = row < t;
        if (PF) load_rows(grp + gridDim.x, xn);      // the next group's rows travel while this one is worked on
        f32x4 acc0[R16], acc1[R16];                  // first-half products (rows 0..7 valid), second-half (rows 8..15)
#pragma unroll
        for (int b = 0; b < R16; ++b) acc0[b] = acc1[b] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u0 = 0; u0 < NSTEP; u0 += LSTEPS) {
            if (!RESIDENT) load_l(u0);
#pragma unroll
            for (int uu = 0; uu < LSTEPS; ++uu)
#pragma unroll
                for (int b = 0; b < R16; ++b)
                    if (u0 + uu < NSTEP) {
                        const bf16x8 a = __builtin_bit_cast(bf16x8, xa[u0 + uu]);
                        acc0[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, lb[uu][0][b]), acc0[b], 0, 0, 0);
                        acc1[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, lb[uu][1][b]), acc1[b], 0, 0, 0);
                    }
        }
        // row maxima of dY * cs over this wavefront's slice
        float mx = 0.0f;
#pragma unroll
        for (int u = 0; u < NSTEP; ++u) {
            const int k = col_of(u);
            if (live && k < kend) {
                float v[8];
                widen_scale(xa[u], csl, k, v);
#pragma unroll
                for (int e = 0; e < 8; ++e) mx = fmaxf(mx, fabsf(v[e]));
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 8, 64));       // the two column halves of a row
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        if (lane < 8) rmax[wave][lane] = mx;
        // Element v of lane (p, g) of an MFMA result is row 4 g + v, column 16 b + p.  Row i < 8 of acc0 (lane groups
        // g < 2) and row i + 8 of acc1 (lane groups g >= 2, 32 lanes further on) are the two halves of T[i]'s partial sum.
#pragma unroll
        for (int b = 0; b < R16; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float second = __shfl_down(acc1[b][v], 32, 64);
                if (g < 2) red[wave][b][lane][v] = acc0[b][v] + second;
            }
        // (workgroup barriers that order LDS traffic only: a full fence would also wait for the previous group's
        // global stores to be acknowledged, once per group)
        lds_barrier();

        float d = 0.0f, cc = 0.0f;
        if (live) {
            float mrow = 0.0f;
#pragma unroll
            for (int w = 0; w < kLoraWaves; ++w) mrow = fmaxf(mrow, rmax[w][m & 7]);
            rtn_steps(mrow, d, cc);
            if (wave == 0 && lane < 8) delta[row] = d;
        }
        // The codes go to this wavefront's piece of LDS, [8 rows][PS * 64], and leave as 16-byte stores that cover a
        // row's slice with consecutive lanes, so that every store instruction writes whole lines; PS steps at a time
        // (all of them unless the slice is long: the staging area of 14 steps would not fit beside the column scales).
        // Writes and reads of the piece come from the same wavefront, whose LDS operations execute in order.
#pragma unroll
        for (int p0 = 0; p0 < NSTEP; p0 += PS) {
            if (live) {
#pragma unroll
                for (int u = p0; u < p0 + PS && u < NSTEP; ++u) {
                    const int k = col_of(u);
                    if (k < kend) {
                        float v[8];
                        widen_scale(xa[u], csl, k, v);
                        *reinterpret_cast<u32x2*>(cw + (m & 7) * (PS * 64) + (k - kbeg - p0 * 64)) = pack_codes(v, cc);
                    }
                }
            }
            const int pbeg = kbeg + p0 * 64;                                      // first column of this pass
            const int pend = pbeg + PS * 64 < kend ? pbeg + PS * 64 : kend;
            const int cpr = pend > pbeg ? (pend - pbeg + 15) >> 4 : 0;           // 16-byte chunks per row
            for (int q = lane; q < 8 * cpr; q += 64) {
                const int rr = q / cpr, ch = q - rr * cpr;
                const int64_t orow = (int64_t)grp * 8 + rr;
                if (orow < t)
                    *reinterpret_cast<u32x4*>(Xq + orow * (int64_t)c + pbeg + ch * 16) =
                        *reinterpret_cast<const u32x4*>(cw + rr * (PS * 64) + ch * 16);
            }
        }
        // fixed-order sums over the eight wavefronts of each part
        for (int e = threadIdx.x; e < kLoraParts * R16 * 32 * 4; e += 64 * kLoraWaves) {
            const int v = e & 3, ln = (e >> 2) & 31, b = (e >> 7) % R16, p = e / (R16 * 128);
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < 8; ++w) sum += red[p * 8 + w][b][ln][v];
            sum = sum * scale;
            const int64_t orow = (int64_t)grp * 8 + (ln >> 4) * 4 + v;
            if (orow < t) {
                const uint32_t hi = f32_to_bf16_rne(sum);
                const float rest = sum - __uint_as_float(hi << 16);
                const int64_t o = (int64_t)p * t * r + orow * r + b * 16 + (ln & 15);
                T_hi[o] = (uint16_t)hi;
                T_lo[o] = (uint16_t)f32_to_bf16_rne(rest);
            }
        }
        lds_barrier();                               // red and rmax are rewritten by the next group
        if (PF) {
#pragma unroll
            for (int u = 0; u < NSTEP; ++u) xa[u] = xn[u];
        } else if (grp + (int)gridDim.x < ngroups) {
            load_rows(grp + gridDim.x, xa);
        }
    }
}

template <int R16>
static bool launch_rows8(const uint16_t* X, int64_t t, int c, int64_t ldx, const float* cs, int8_t* Xq, float* delta,
                         const uint16_t* L, float scale, uint16_t* T_hi, uint16_t* T_lo, hipStream_t stream) {
    const int cp = ((c + kLoraParts * 64 - 1) / (kLoraParts * 64)) * 64;
    const int nstep = (cp + 8 * 64 - 1) / (8 * 64);          // 64-column steps per wavefront
    // one persistent workgroup per compute unit (fewer when there are fewer 8-row groups)
    const int ngroups = (int)((t + 7) / 8);
    const dim3 grid((unsigned)(ngroups < 256 ? ngroups : 256)), block(64 * kLoraWaves);
#define QUAFF_R8(NS, RES)                                                                                             \
    {                                                                                                                 \
        const size_t lds = (((size_t)c * 4 + 255) & ~(size_t)255) +                                                   \
                           (size_t)kLoraWaves * 8 * (NS > 9 ? (NS + 1) / 2 : NS) * 64;                                \
        auto kern = quant_lora_rows8_kernel<R16, NS, RES>;                                                            \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,      \
                                (int)lds) != hipSuccess)                                                              \
            return false;                                                                                             \
        hipLaunchKernelGGL(kern, grid, block, lds, stream, X, t, c, ldx, cs, Xq, delta, L, scale, T_hi, T_lo, ngroups); \
    }
    // Longer rows: nine and more steps of resident L fragments and prefetched rows do not fit the 128 registers a
    // 16-wavefront workgroup has per lane.  The form that fetches L again for every group then moves twice the bytes of
    // dY through the L2 -> L1 path and is level with the two-role launch up to a few thousand rows (31 against 28 us at
    // 2048 x 9216); with many rows it reads dY once from HBM where the two-role launch reads it twice: 16384 x 13824
    // 306 against 341 us, 16384 x 9216 177 against 180, 8192 x 9216 87 against 90.
    if (nstep <= 3) QUAFF_R8(3, true)
    else if (nstep <= 5) QUAFF_R8(5, true)
    else if (nstep <= 9 && ngroups >= 1024) QUAFF_R8(9, false)
    else if (nstep <= 14 && ngroups >= 1024) QUAFF_R8(14, false)
    else return false;
#undef QUAFF_R8
    return true;
}

template <int R16>
static bool launch_r(const uint16_t* X, int64_t t, int c, int64_t ldx, const float* cs, int8_t* Xq, float* delta,
                     const uint16_t* L, float scale, uint16_t* T_hi, uint16_t* T_lo, hipStream_t stream) {
    constexpr int NT = 64 * kLoraWaves;
    constexpr int RG = lora_row_groups(R16);
    const int row_blocks = (int)((t + 15) / 16);
    const int lora_row_blocks = (int)((t + 16 * RG - 1) / (16 * RG));
    const int vec = (c + 7) / 8;
#define QUAFF_QL(TPR, NV)                                                                                             \
    hipLaunchKernelGGL((quant_lora_kernel<R16, TPR, NV>),                                                             \
                       dim3((unsigned)(lora_row_blocks * kLoraParts +                                                 \
                                       8 * RG * ((row_blocks + 8 * RG - 1) / (8 * RG)) * (16 / (NT / TPR)))),         \
                       dim3(NT), 0,                                                                                   \
                       stream, X, t, c, ldx, cs, Xq, delta, L, scale, T_hi, T_lo, lora_row_blocks)
    if (vec <= 64 * 2) QUAFF_QL(64, 2);
    else if (vec <= 64 * 4) QUAFF_QL(64, 4);
    else if (vec <= 64 * 6) QUAFF_QL(64, 6);
    else if (vec <= 64 * 8) QUAFF_QL(64, 8);
    else if (vec <= 256 * 3) QUAFF_QL(256, 3);
    else if (vec <= 256 * 4) QUAFF_QL(256, 4);
    else if (vec <= 256 * 6) QUAFF_QL(256, 6);
    else if (vec <= 256 * 8) QUAFF_QL(256, 8);
    else return false;
#undef QUAFF_QL
    return true;
}

// Returns false (nothing enqueued) for shapes this launch does not cover: the caller then issues the two launches.
bool launch_quant_lora(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const float* cs, int8_t* Xq, float* delta,
                       const uint16_t* L_r_by_c, int32_t r, float scale, uint16_t* T_hi, uint16_t* T_lo,
                       hipStream_t stream, hipError_t* err) {
    if (r < 16 || r > 64 || r % 16 != 0 || c > 256 * 8 * 8) return false;
    ProfScope prof(K_QUANT_LORA, stream);
    bool ok = false;
    // One pass over dY with eight rows per persistent workgroup where it pays: the smallest rank (a wavefront keeps
    // its slice of L in registers) and rows short enough for the registers.  Measured at 16384 x 5120: 85 us against
    // 130 us for the two-role launch (which reads dY twice); at 2048 and 4096 rows the two forms are level.
    if (r == 16 && cs != nullptr) {
        ok = launch_rows8<1>(X, t, (int)c, ldx, cs, Xq, delta, L_r_by_c, scale, T_hi, T_lo, stream);
        if (ok) { *err = hipGetLastError(); return true; }
    }
    switch (r / 16) {
        case 1: ok = launch_r<1>(X, t, (int)c, ldx, cs, Xq, delta, L_r_by_c, scale, T_hi, T_lo, stream); break;
        case 2: ok = launch_r<2>(X, t, (int)c, ldx, cs, Xq, delta, L_r_by_c, scale, T_hi, T_lo, stream); break;
        case 3: ok = launch_r<3>(X, t, (int)c, ldx, cs, Xq, delta, L_r_by_c, scale, T_hi, T_lo, stream); break;
        case 4: ok = launch_r<4>(X, t, (int)c, ldx, cs, Xq, delta, L_r_by_c, scale, T_hi, T_lo, stream); break;
    }
    *err = hipGetLastError();
    return ok;
}

}  // namespace quaff
