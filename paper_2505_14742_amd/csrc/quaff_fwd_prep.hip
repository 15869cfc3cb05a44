// Forward preparation of a layer in ONE launch and one pass over X (quaff_linear_fwd_step, up to 2048 tokens):
//   the outlier-column abs-max (Eq. 8), the momentum update (Eq. 7), the requantization of what = (s_O - 1) W_O
//   (Eq. 5, Eq. 9), the scaled per-token quantizer of X (Eq. 5, Eq. 1) with the compact outlier codes (remark after
//   Eq. 9), the LoRA down-projection X A and the transposed copy of B that the product's epilogue reads.
// A workgroup of 16 wavefronts owns 8 token rows and keeps them in registers from the first load to the last store.
// The column maxima are the one step that needs all rows: every workgroup writes the maxima of its rows, does the
// work that does not depend on them (down-projection, copy of the column scales) and then reads everybody's maxima.
// No read-modify-write atomic is involved (256 workgroups arriving at one counter within a microsecond serialise at
// one memory round trip each): a maximum travels as a 32-bit word whose upper half is the bf16 magnitude and whose
// lower half is a tag, the low 16 bits of (epoch + 1); `epoch` is a word of the workspace that every workgroup reads
// before it writes and that is set to epoch + 1 once all maxima of the launch have been seen - so words left by an
// earlier launch, or by anything else that used the memory, do not carry this launch's tag.  A workgroup has
// everything when all n x groups words carry the tag.  The wait is bounded: a workgroup that has not seen them within
// `wait_ticks` (100 MHz ticks) computes the maxima of ALL rows itself from X - slower, the same bits - so the result
// never depends on how many workgroups the hardware keeps resident at once.  Every workgroup that saw all maxima
// (the last one to write always does) publishes s, 1/s and cmax - the same values - and the new epoch: by then every
// workgroup has read the previous scales, so nobody overwrites state that a later workgroup still has to read.
//
// Results are bit-identical to the separate launches: the down-projection sums its contraction range in the
// order of lora_down_body (32 slices, each accumulated through the same MFMA slots, added in slice order).
#include "quaff_lora_body.h"
#include "quaff_quant_body.h"
#include "quaff_scale_body.h"

namespace quaff {

constexpr int kPrepRows = 8;
constexpr int kPrepThreads = 64 * kLoraWaves;      // 1024
constexpr int kPrepMaxGroups = 256;                // one workgroup per compute unit: all resident at once
constexpr int kPrepLtBlock = 640;                  // bytes of 16 rows of a wavefront's slice of A in LDS: 16 x 32 + padding
constexpr int kWhatChunk = 64;                     // output channels of what requantized per round

struct FwdPrepArgs {
    const uint16_t* X; int64_t t; int c; int64_t ldx;
    const int32_t* O; int n; int n_pad;
    const float* wmax_O; float gamma; float* s_O; float* colscale; float* cmax_out;
    const float* W_O; int64_t c_out; int8_t* what_int; float* delta_what;
    int8_t* Xq; float* delta; int8_t* xq_O;
    const uint16_t* A; float scale; uint16_t* T_hi; uint16_t* T_lo;     // LoRA (HAS_LORA)
    const uint16_t* B; uint16_t* Bt;                                    // B [16 x c_out] -> Bt [c_out x 16]
    uint32_t* part;               // [n][groups] maxima of each workgroup's rows: bf16 magnitude << 16 | tag
    uint32_t* epoch;              // launch counter of this workspace (any start value)
    int groups; long long wait_ticks;
};


// NSTEP: 64-column steps a wavefront holds (two slices of the down-projection's summation order)
template <int NSTEP, bool HAS_LORA>
__global__ void __launch_bounds__(kPrepThreads)
fwd_prep_kernel(const FwdPrepArgs a) {
    static_assert(kLoraParts == 2 && kLoraWaves == 16, "two parts of eight wavefronts each");
    constexpr int SPS = NSTEP / 2;                 // steps per slice
    // dynamic LDS: the column scales of this step [c], then a staging region used twice: by the down-projection
    // (lt: a wavefront's slice of A, [64 columns][16] bf16 in padded blocks; red: per slice, this workgroup's 8 x 16
    // partial sums of T) and afterwards by the quantizer (the wavefronts' code rows on their way to whole-line stores)
    extern __shared__ __attribute__((aligned(16))) char dyn_lds[];
    float* cs_copy = reinterpret_cast<float*>(dyn_lds);
    char* stage = dyn_lds + (((size_t)a.c * 4 + 255) & ~(size_t)255);
    char (*lt)[4 * kPrepLtBlock] = reinterpret_cast<char (*)[4 * kPrepLtBlock]>(stage);
    float (*red)[32][4] = reinterpret_cast<float (*)[32][4]>(stage + kLoraWaves * 4 * kPrepLtBlock);
    __shared__ float rmax[kLoraWaves][kPrepRows];
    __shared__ uint32_t smax[64];                  // column maxima over all rows
    __shared__ float sm1[64], rinv[64], sprev[64], wmx[64];
    __shared__ int ocol[64];
    __shared__ float rowc[kPrepRows];
    __shared__ uint32_t wmaxbits[kWhatChunk];
    __shared__ __attribute__((aligned(16))) int8_t wcodes[kWhatChunk][64];
    __shared__ int flag_ok, flag_all, flag_timeout;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 15, g = lane >> 4;
    const int blk = blockIdx.x, G = a.groups, n = a.n, c = a.c;
    const int64_t row0 = (int64_t)blk * kPrepRows;
    const int64_t row = row0 + (m & 7);
    const bool live = row < a.t;
    const uint16_t* xrow = a.X + (live ? row : 0) * a.ldx;

    // ---- this wavefront's columns: part p of the contraction range, slices 2 w' and 2 w' + 1 of its sixteen
    const int partno = wave >> 3;
    const int cp = ((c + kLoraParts * 64 - 1) / (kLoraParts * 64)) * 64;
    const int cbeg = partno * cp, cend = cbeg + cp < c ? cbeg + cp : c;
    const int kw = ((cend - cbeg + kLoraWaves * 64 - 1) / (kLoraWaves * 64)) * 64;     // columns per slice
    const int kbeg0 = cbeg + (wave & 7) * 2 * kw;
    // step u belongs to slice u / SPS; lane (m, g) holds row m % 8, columns 16 g + 8 (m / 8) .. + 7 of the step
    auto step_base = [&](int u) { return kbeg0 + (u / SPS) * kw + (u % SPS) * 64; };
    auto slice_end = [&](int u) {
        const int e = kbeg0 + (u / SPS + 1) * kw;
        return e < cend ? e : cend;
    };
    auto col_of = [&](int u) { return step_base(u) + g * 16 + (m >> 3) * 8; };

    u32x4 xa[NSTEP];
#pragma unroll
    for (int u = 0; u < NSTEP; ++u) {
        const int k = col_of(u);
        xa[u] = (u32x4){0, 0, 0, 0};
        if (live && k < slice_end(u) && (u % SPS) * 64 < kw) xa[u] = *reinterpret_cast<const u32x4*>(xrow + k);
    }
    // Every global load that depends on nothing computed here is issued now, so that the kernel pays for few memory
    // round trips one after the other: the slices of A of the first AB steps, this thread's element of the transposed
    // copy of B, and its share of the first chunk of W_O.
    constexpr int AB = NSTEP < 4 ? NSTEP : 4;      // steps of A in flight together
    u32x4 av[AB][2];
    auto load_a = [&](int u0) {
#pragma unroll
        for (int uu = 0; uu < AB; ++uu) {
            const int u = u0 + uu;
            const int kb = step_base(u);
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                // A [c x 16]: the step's 64 x 16 slice is 2 KiB contiguous; lane l takes rows l / 2 and 32 + l / 2
                int kr = kb + v * 32 + (lane >> 1);
                kr = kr < c ? kr : c - 1;                 // (a row past the end meets a cleared x fragment)
                kr = kr > 0 ? kr : 0;
                av[uu][v] = *reinterpret_cast<const u32x4*>(a.A + (int64_t)kr * 16 + (lane & 1) * 8);
            }
        }
    };
    if (HAS_LORA) load_a(0);
    const int64_t bt_total = HAS_LORA ? 16 * a.c_out : 0;     // Bt [c_out x 16] <- B [16 x c_out]
    const int64_t bt_e0 = (int64_t)blk * kPrepThreads + tid;
    uint16_t bt_first = 0;
    if (bt_e0 < bt_total) bt_first = a.B[(bt_e0 & 15) * a.c_out + (bt_e0 >> 4)];
    const int64_t per = (a.c_out + G - 1) / G;
    const int64_t j0 = (int64_t)blk * per, j1 = j0 + per < a.c_out ? j0 + per : a.c_out;
    float w_first[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = tid + i * kPrepThreads;          // thread (k, jl) of a 64 x 64 chunk, channels fastest
        const int k = e >> 6, jl = e & 63;
        w_first[i] = 0.0f;
        if (k < n && j0 + jl < j1) w_first[i] = a.W_O[(int64_t)k * a.c_out + j0 + jl];
    }
    f32x4 cs_first[2];        // this thread's vectors of the column scales (c <= 8192: at most two)
#pragma unroll
    for (int v = 0; v < 2; ++v) {
        const int i = (tid + v * kPrepThreads) * 4;
        cs_first[v] = (f32x4){1.f, 1.f, 1.f, 1.f};
        if (i < c) cs_first[v] = *reinterpret_cast<const f32x4*>(a.colscale + i);
    }
    // per-outlier constants and the previous scales, and the epoch (all read before this workgroup's maxima are written)
    if (tid < 64) {
        const int k = tid < n ? tid : n - 1;
        ocol[tid] = a.O[k];
        sprev[tid] = a.s_O[k];
        wmx[tid] = a.wmax_O[k];
    }
    // Device-scope atomic loads and stores go past the per-XCD L2s: no cache write-back or invalidation is needed to
    // hand the words from one workgroup to another.
    const uint32_t epoch = __hip_atomic_load(a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t tag = (epoch + 1u) & 0xFFFFu;
    // ---- maxima of this workgroup's rows on the outlier columns: lanes 8 k .. 8 k + 7 hold the eight rows of column k
    uint16_t xo_raw = 0;     // X[row0 + tid % 8, O[tid / 8]]: also what the compact outlier codes are made from
    {
        const int k = tid >> 3, rr = tid & 7;
        uint32_t v = 0;
        if (k < n && row0 + rr < a.t) {
            xo_raw = a.X[(row0 + rr) * a.ldx + a.O[k]];
            v = ((uint32_t)xo_raw & 0x7FFFu) << 16;
        }
        v = max(v, (uint32_t)__shfl_xor((int)v, 1, 64));
        v = max(v, (uint32_t)__shfl_xor((int)v, 2, 64));
        v = max(v, (uint32_t)__shfl_xor((int)v, 4, 64));
        // The previous scales must have been READ (not just requested) by this workgroup before its maxima become
        // visible, because whoever sees all maxima may overwrite them: the barrier follows the LDS writes of the
        // loaded values.  (The epoch feeds the stored word itself.)
        __syncthreads();
        if (k < n && rr == 0)
            __hip_atomic_store(&a.part[(int64_t)k * G + blk], v | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- work that needs no other workgroup: transposed copy of B, copy of the column scales, down-projection
    if (HAS_LORA) {
        if (bt_e0 < bt_total) a.Bt[bt_e0] = bt_first;
        for (int64_t e = bt_e0 + (int64_t)G * kPrepThreads; e < bt_total; e += (int64_t)G * kPrepThreads)
            a.Bt[e] = a.B[(e & 15) * a.c_out + (e >> 4)];
    }
#pragma unroll
    for (int v = 0; v < 2; ++v) {                           // c is a multiple of 16
        const int i = (tid + v * kPrepThreads) * 4;
        if (i < c) *reinterpret_cast<f32x4*>(cs_copy + i) = cs_first[v];
    }
    if (HAS_LORA) {
        f32x4 acc[2];
        acc[0] = acc[1] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < NSTEP; ++u) {
            const int kb = step_base(u);
            if (u > 0 && u % AB == 0) load_a(u);             // (NSTEP = 8: the second batch)
            if ((u % SPS) * 64 < kw && kb < cend) {          // uniform over the wavefront
                const u32x4 (&avu)[2] = av[u % AB];
                // The slice goes to LDS as it is (column-major: 32 bytes per column, 16 columns per padded block) and
                // the MFMA operand - for lane (p, g) eight columns of one rank index p - comes back through the
                // transposing LDS read: in each group of 16 lanes, lane i receives 16-bit element i % 4 of the 8-byte
                // pieces addressed by lanes i / 4 + 4 j, j = 0..3.  Lane a of a group therefore addresses column a / 4
                // of the four it wants, rank indices 4 (a % 4) .. + 3.
                typedef short v4s __attribute__((ext_vector_type(4)));
                typedef __attribute__((address_space(3))) v4s lds_v4s;
#pragma unroll
                for (int v = 0; v < 2; ++v) {
                    const int kk = v * 32 + (lane >> 1);
                    *reinterpret_cast<u32x4*>(&lt[wave][(kk >> 4) * kPrepLtBlock + (kk & 15) * 32 + (lane & 1) * 16]) = avu[v];
                }
                // even MFMA: contraction slots (g, e) <-> columns 16 g + e; odd: 16 g + 8 + e.  Rows 0..7 of the x
                // operand must hold the matching columns: the lanes m >= 8 hold the odd ones, swapped in for the second.
                const char* piece = &lt[wave][g * kPrepLtBlock + (m >> 2) * 32 + (m & 3) * 8];
                auto four = [&](int col0) {
                    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(piece + col0 * 32));
                };
                const v4s e0 = four(0), e1 = four(4), o0 = four(8), o1 = four(12);
                const u32x4 l_even = __builtin_bit_cast(u32x4, (short __attribute__((ext_vector_type(8)))){
                    e0[0], e0[1], e0[2], e0[3], e1[0], e1[1], e1[2], e1[3]});
                const u32x4 l_odd = __builtin_bit_cast(u32x4, (short __attribute__((ext_vector_type(8)))){
                    o0[0], o0[1], o0[2], o0[3], o1[0], o1[1], o1[2], o1[3]});
                u32x4 x_odd;
#pragma unroll
                for (int w = 0; w < 4; ++w) x_odd[w] = (uint32_t)__shfl_xor((int)xa[u][w], 8, 64);
                f32x4& ac = acc[u / SPS];
                ac = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, xa[u]),
                                                             __builtin_bit_cast(bf16x8, l_even), ac, 0, 0, 0);
                ac = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x_odd),
                                                             __builtin_bit_cast(bf16x8, l_odd), ac, 0, 0, 0);
            }
        }
        // element v of lane (p, g) is row 4 g + v, column p: rows 0..7 are lane groups g < 2
        if (g < 2) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[2 * wave + s][lane][v] = acc[s][v];
        }
    }
    __syncthreads();
    if (HAS_LORA) {
        // fixed-order sums over the sixteen slices of each part
        for (int e = tid; e < kLoraParts * 32 * 4; e += kPrepThreads) {
            const int v = e & 3, ln = (e >> 2) & 31, p = e >> 7;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < 16; ++w) sum += red[p * 16 + w][ln][v];
            sum = sum * a.scale;
            const int64_t orow = row0 + (ln >> 4) * 4 + v;
            if (orow < a.t) {
                const uint32_t hi = f32_to_bf16_rne(sum);
                const float rest = sum - __uint_as_float(hi << 16);
                const int64_t o = (int64_t)p * a.t * 16 + orow * 16 + (ln & 15);
                a.T_hi[o] = (uint16_t)hi;
                a.T_lo[o] = (uint16_t)f32_to_bf16_rne(rest);
            }
        }
    }

    // ---- bounded wait for the other workgroups' maxima: wavefront w reads columns w, w + 16, ... (G contiguous words
    // each) and reduces them with wavefront shuffles; the pass is repeated until every word carries this launch's tag
    const long long t0 = (long long)wall_clock64();
    for (;;) {
        if (tid == 0) flag_all = 1;
        if (tid < 64) smax[tid] = 0u;
        __syncthreads();
        bool mine = true;
        // a wavefront has at most four columns (n <= 64) of at most four words per lane (G <= 256): all loads first
        uint32_t wv4[4][4];
#pragma unroll
        for (int kc = 0; kc < 4; ++kc)
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                const int k = wave + kc * kLoraWaves, i = lane + ii * 64;
                wv4[kc][ii] = tag;                        // (absent words count as present, magnitude 0)
                if (k < n && i < G)
                    wv4[kc][ii] = __hip_atomic_load(&a.part[(int64_t)k * G + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
            const int k = wave + kc * kLoraWaves;
            uint32_t v = 0;
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                mine = mine && (wv4[kc][ii] & 0xFFFFu) == tag;
                v = max(v, wv4[kc][ii] & 0xFFFF0000u);
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, off, 64));
            if (lane == 0 && k < n) smax[k] = v;
        }
        if (!mine) flag_all = 0;
        __syncthreads();
        if (flag_all) break;
        if (tid == 0) flag_timeout = (long long)wall_clock64() - t0 >= a.wait_ticks;
        __syncthreads();
        if (flag_timeout) break;
        __builtin_amdgcn_s_sleep(16);
    }
    if (tid == 0) flag_ok = flag_all;
    __syncthreads();
    if (flag_ok) {
        // (smax holds the maxima over all rows)
    } else {
        // gave up waiting: the maxima of all rows straight from X (any order gives the same maximum)
        if (tid < 64) smax[tid] = 0u;
        __syncthreads();
        const int64_t total = a.t * n;
        for (int64_t e0 = tid; e0 < total; e0 += kPrepThreads * 4) {
            uint32_t mag[4];
            int kk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t e = e0 + (int64_t)u * kPrepThreads;
                const int64_t ec = e < total ? e : total - 1;
                const int64_t r = ec / n;
                kk[u] = (int)(ec - r * n);
                mag[u] = ((uint32_t)a.X[r * a.ldx + ocol[kk[u]]] & 0x7FFFu) << 16;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (e0 + (int64_t)u * kPrepThreads < total) atomicMax(&smax[kk[u]], mag[u]);
        }
    }
    __syncthreads();
    if (tid < n) {
        const float cmax = __uint_as_float(smax[tid]);
        const float s = momentum_scale(cmax, wmx[tid], sprev[tid], a.gamma);
        const float ri = __fdiv_rn(1.0f, s);
        sm1[tid] = __fsub_rn(s, 1.0f);
        rinv[tid] = ri;
        cs_copy[ocol[tid]] = ri;
        if (flag_ok) {             // every workgroup has written its maxima, so it has read the previous scales
            a.s_O[tid] = s;
            a.colscale[ocol[tid]] = ri;
            if (a.cmax_out) a.cmax_out[tid] = cmax;
        }
    }
    if (tid == 0 && flag_ok) __hip_atomic_store(a.epoch, epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();

    // ---- per-token quantization of this workgroup's rows, from the registers
    const lds_float* csl = (const lds_float*)cs_copy;
    constexpr bool KEEP = NSTEP <= 4;              // the scaled fp32 values stay in registers for the code pass
    float xs[KEEP ? NSTEP : 1][8];
    float mx = 0.0f;
    if (live) {
#pragma unroll
        for (int u = 0; u < NSTEP; ++u) {
            const int k = col_of(u);
            if (k < slice_end(u) && (u % SPS) * 64 < kw) {
                float v[8];
                widen_scale(xa[u], csl, k, v);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    mx = fmaxf(mx, fabsf(v[e]));
                    if (KEEP) xs[KEEP ? u : 0][e] = v[e];
                }
            }
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 8, 64));       // the two column halves of a row
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (lane < 8) rmax[wave][lane] = mx;
    __syncthreads();
    float cc = 0.0f;
    {
        float mrow = 0.0f;
#pragma unroll
        for (int w = 0; w < kLoraWaves; ++w) mrow = fmaxf(mrow, rmax[w][m & 7]);
        float d;
        rtn_steps(mrow, d, cc);
        if (wave == 0 && lane < 8) {
            rowc[lane] = cc;
            if (live) a.delta[row] = d;
        }
    }
    // The codes leave through LDS so that every store instruction writes whole 128-byte lines: a wavefront's rows of
    // one slice are [8][kw] bytes; lane q of the store pass takes 16-byte chunk q % (kw / 16) of row q / (kw / 16).
    {
        char* cw = stage + wave * (2 * kPrepRows * SPS * 64);
        if (live) {
#pragma unroll
            for (int u = 0; u < NSTEP; ++u) {
                const int k = col_of(u);
                if (k < slice_end(u) && (u % SPS) * 64 < kw) {
                    float v[8];
                    if (KEEP) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = xs[KEEP ? u : 0][e];
                    } else {
                        widen_scale(xa[u], csl, k, v);
                    }
                    *reinterpret_cast<u32x2*>(cw + ((u / SPS) * kPrepRows + (m & 7)) * (SPS * 64) + (u % SPS) * 64 + g * 16 +
                                              (m >> 3) * 8) = pack_codes(v, cc);
                }
            }
        }
        const int cpr = kw >> 4;                         // 16-byte chunks per row of a slice
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            const int kb = kbeg0 + sl * kw;
            const int ke = kb + kw < cend ? kb + kw : cend;
            for (int q = lane; q < kPrepRows * cpr; q += 64) {
                const int rr = q / cpr, ch = q - rr * cpr;
                const int col = kb + ch * 16;
                if (row0 + rr < a.t && col < ke) {
                    *reinterpret_cast<u32x4*>(a.Xq + (row0 + rr) * (int64_t)c + col) =
                        *reinterpret_cast<const u32x4*>(cw + (sl * kPrepRows + rr) * (SPS * 64) + ch * 16);
                }
            }
        }
    }
    __syncthreads();
    // compact copy of the outlier columns' codes (zero beyond n): thread 8 k + rr holds X[row0 + rr, O[k]]
    if (a.xq_O) {
        const int k = tid >> 3, rr = tid & 7;
        if (k < a.n_pad && row0 + rr < a.t) {
            int q = 0;
            if (k < n) q = rtn_code(__fmul_rn(bf16_bits_to_f32(xo_raw), rinv[k]), rowc[rr]);
            a.xq_O[(row0 + rr) * a.n_pad + k] = (int8_t)q;
        }
    }

    // ---- this workgroup's share of what = (s_O - 1) W_O, requantized per output channel (Eq. 5, Eq. 1)
    for (int64_t jc = j0; jc < j1; jc += kWhatChunk) {
        const int nj = (int)(j1 - jc < kWhatChunk ? j1 - jc : kWhatChunk);
        if (tid < kWhatChunk) wmaxbits[tid] = 0u;
        __syncthreads();
        // thread (k, jl): channels are the fast index, so a wavefront reads runs of one row of W_O
        float wv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * kPrepThreads;          // e < 64 * 64
            const int k = e >> 6, jl = e & 63;
            wv[i] = 0.0f;
            if (k < n && jl < nj) {
                const float w = jc == j0 ? w_first[i] : a.W_O[(int64_t)k * a.c_out + jc + jl];
                wv[i] = __fmul_rn(sm1[k], w);
                atomicMax(&wmaxbits[jl], __float_as_uint(fabsf(wv[i])));
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + i * kPrepThreads;
            const int k = e >> 6, jl = e & 63;
            if (k < a.n_pad && jl < nj) {
                float d, cw;
                rtn_steps(__uint_as_float(wmaxbits[jl]), d, cw);
                wcodes[jl][k] = (int8_t)(k < n ? rtn_code(wv[i], cw) : 0);
                if (k == 0) a.delta_what[jc + jl] = d;
            }
        }
        __syncthreads();
        // rows of what_int are n_pad = 64 bytes: four 16-byte stores each
        if (tid < nj * 4)
            *reinterpret_cast<u32x4*>(a.what_int + (jc + (tid >> 2)) * a.n_pad + (tid & 3) * 16) =
                *reinterpret_cast<const u32x4*>(&wcodes[tid >> 2][(tid & 3) * 16]);
        __syncthreads();
    }
}

int fwd_prep_groups(int64_t t) { return (int)((t + kPrepRows - 1) / kPrepRows); }

// shapes the one-launch preparation covers
bool fwd_prep_covers(int64_t t, int64_t c_in, int32_t n, int32_t r) {
    return t >= 1 && fwd_prep_groups(t) <= kPrepMaxGroups && n >= 1 && n <= 64 && (r == 0 || r == 16) && c_in <= 8192;
}

size_t fwd_prep_scratch_bytes(int32_t n) { return ((size_t)n * kPrepMaxGroups * 4 + 255) / 256 * 256 + 256; }

template <int NSTEP>
static hipError_t launch_prep(bool has_lora, dim3 grid, size_t lds, hipStream_t stream, const FwdPrepArgs& a) {
    auto k = has_lora ? fwd_prep_kernel<NSTEP, true> : fwd_prep_kernel<NSTEP, false>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k, grid, dim3(kPrepThreads), lds, stream, a);
    return hipGetLastError();
}

hipError_t launch_fwd_prep(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const int32_t* O, int32_t n,
                           const float* wmax_O, float gamma, float* s_O, float* colscale, float* cmax_out,
                           const float* W_O, int64_t c_out, int8_t* what_int, float* delta_what, int8_t* Xq,
                           float* delta, int8_t* xq_O, const uint16_t* A, const uint16_t* B, int32_t r, float scale,
                           uint16_t* T_hi, uint16_t* T_lo, uint16_t* Bt, void* scratch, long long wait_ticks,
                           hipStream_t stream) {
    ProfScope prof(K_FWD_PREP, stream);
    FwdPrepArgs a{};
    a.X = X; a.t = t; a.c = (int)c; a.ldx = ldx;
    a.O = O; a.n = n; a.n_pad = (n + kPadK - 1) / kPadK * kPadK;
    a.wmax_O = wmax_O; a.gamma = gamma; a.s_O = s_O; a.colscale = colscale; a.cmax_out = cmax_out;
    a.W_O = W_O; a.c_out = c_out; a.what_int = what_int; a.delta_what = delta_what;
    a.Xq = Xq; a.delta = delta; a.xq_O = xq_O;
    a.A = A; a.scale = scale; a.T_hi = T_hi; a.T_lo = T_lo; a.B = B; a.Bt = Bt;
    a.groups = fwd_prep_groups(t);
    a.part = reinterpret_cast<uint32_t*>(static_cast<char*>(scratch) + 256);
    a.epoch = reinterpret_cast<uint32_t*>(scratch);
    a.wait_ticks = wait_ticks;
    // steps per wavefront: two slices of the down-projection's sixteen per part
    const int cp = (((int)c + kLoraParts * 64 - 1) / (kLoraParts * 64)) * 64;
    const int kw = ((cp + kLoraWaves * 64 - 1) / (kLoraWaves * 64)) * 64;
    const int nstep = 2 * (kw / 64);
    const dim3 grid((unsigned)a.groups);
    // column scales, then the larger of the down-projection's staging (A slices + partial sums) and the code rows
    const size_t stage_lora = (size_t)kLoraWaves * 4 * kPrepLtBlock + 2 * kLoraWaves * 32 * 4 * sizeof(float);
    const size_t stage_codes = (size_t)kLoraWaves * 2 * kPrepRows * (nstep <= 2 ? 1 : nstep <= 4 ? 2 : 4) * 64;
    const size_t lds = (((size_t)c * 4 + 255) & ~(size_t)255) + (stage_lora > stage_codes ? stage_lora : stage_codes);
    const bool has_lora = r == 16;
    if (nstep <= 2) return launch_prep<2>(has_lora, grid, lds, stream, a);
    if (nstep <= 4) return launch_prep<4>(has_lora, grid, lds, stream, a);
    if (nstep <= 8) return launch_prep<8>(has_lora, grid, lds, stream, a);
    return hipErrorInvalidValue;
}

}  // namespace quaff
