// Internal declarations shared by the translation units of libquaff (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace quaff {

constexpr int kWave = 64;
constexpr int kPadK = 64;   // outlier count is padded to the INT8 MFMA contraction step
constexpr int kLoraParts = 2;   // the LoRA down-projection splits its contraction range over this many workgroups;
                                // the partial results T[p] ([t x r] each, hi/lo bf16 pairs) are summed by the GEMM epilogue

// ---- device helpers -------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// Eq. 1 for one value: code = clamp(rne(x * c), -127, 127) with c = 127 / max, in fp32, one rounding per op.
__device__ __forceinline__ int rtn_code(float x, float c) {
    float q = __builtin_rintf(__fmul_rn(x, c));
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}

// Step size Delta = m / 127 and reciprocal step c = 127 / m of a group with absolute maximum m (both 0 if m = 0).
__device__ __forceinline__ void rtn_steps(float m, float& delta, float& c) {
    if (m > 0.0f) {
        delta = __fdiv_rn(m, 127.0f);
        c = __fdiv_rn(127.0f, m);
    } else {
        delta = 0.0f;
        c = 0.0f;
    }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// ---- optional per-launch timing (see quaff_profile_* in the C ABI) ------------------------------------
enum KernelKind { K_PREPARE = 0, K_COLMAX, K_MOMENTUM, K_QUANT, K_LORA, K_GEMM, K_LORA_GRAD, K_OUTLIER_GRAD, K_CALIB, K_QUANT_LORA, K_COLMAX_LORA, K_WHAT_QUANT, K_FWD_PREP, KERNEL_KINDS };
class ProfScope {
public:
    ProfScope(int kind, hipStream_t stream);
    ~ProfScope();
private:
    hipStream_t stream_;
    int idx_;
};

// ---- host-side launchers (each enqueues on `stream`, returns a hipError_t) -------------------------
hipError_t launch_prepare_weight(const float* W, int64_t c_in, int64_t c_out, int64_t ldw, const int32_t* O, int32_t n,
                                 int8_t* Wp, float* delta_w, float* W_O, float* wmax_O, int8_t* Wq_plain,
                                 float* ws, hipStream_t stream);

hipError_t launch_scale_update(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O, int32_t n,
                               const float* W_O, const float* wmax_O, int64_t c_out, float gamma, float* s_O,
                               float* colscale, int8_t* what_int, float* delta_what, float* cmax_out, float* ws,
                               hipStream_t stream);
int scale_update_blocks(int64_t t);   // number of partial-max slabs (workspace sizing)
// quaff_scale_update_static: device address of this device's static scratch (room for scale_update_blocks slabs of
// up to scale_update_static_max_outliers() channels, plus the previous scales); looked up once per device
int scale_update_static_max_outliers();
hipError_t scale_update_static_scratch(float** ptr);

hipError_t launch_check_outliers(const int32_t* O, int32_t n, int64_t c_in, int32_t* result, hipStream_t stream);

hipError_t launch_quant_act(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const float* colscale,
                            const int32_t* O, int32_t n, int8_t* Xq, float* delta, int8_t* xq_O, hipStream_t stream);

// LoRA down-projection T = scale * (X [t x c] bf16) * (L [c x r] or [r x c] bf16), kept as a bf16 hi/lo pair, and an
// optional transposed copy of a second factor (src [rows x cols] -> dst [cols x rows]).
hipError_t launch_lora_down(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const uint16_t* L, bool L_is_r_by_c,
                            int32_t r, float scale, uint16_t* T_hi, uint16_t* T_lo, const uint16_t* tr_src,
                            uint16_t* tr_dst, int64_t tr_rows, int64_t tr_cols, hipStream_t stream,
                            uint16_t* Lt_scratch = nullptr);
// The two down-projections of the LoRA weight gradients, T1 = scale dY B^T (B [r x c_out]) and T2 = scale X A
// (A [c_in x r]), in one launch where that is possible (rank 16, inputs short enough for the per-block kernel), else
// one after the other; same bits as two launch_lora_down calls.
hipError_t launch_lora_down_pair(const uint16_t* dY, int64_t lddy, int64_t c_out, const uint16_t* B, uint16_t* T1_hi,
                                 uint16_t* T1_lo, const uint16_t* X, int64_t ldx, int64_t c_in, const uint16_t* A,
                                 uint16_t* T2_hi, uint16_t* T2_lo, int64_t t, int32_t r, float scale,
                                 uint16_t* At_scratch, hipStream_t stream);
// A [c x r] factor of rank 32 or more is better transposed once to [r x c] (scratch of c * r elements) than slice by
// slice through LDS by every workgroup (the result is the same bit for bit).  At rank 16 it is not, not even with
// 1024 row blocks: 16384 x 5120 takes 118 us with the transposed copy against 89 us without (measured).
inline bool lora_prefers_transposed(int32_t r, int64_t /*t*/) { return r >= 32; }
hipError_t launch_transpose_bf16(const uint16_t* src, int64_t rows, int64_t cols, uint16_t* dst, hipStream_t stream);

// LoRA weight gradients (quaff_lora_grad.hip).  lora_grad_plan: how the token range is cut into slabs (workspace
// sizing); launch_lora_grad_pair: both gradient products (out = sum_i P[i, :]^T Q[i, :]) in one launch, P given as
// the hi / lo parts [kLoraParts x t x r] of a down-projection, followed by the launch that sums the slabs; partial
// [nslab x r x c] scratch each.
void lora_grad_plan(int64_t t, int64_t c, int* nslab, int* rows_per_slab);
hipError_t launch_lora_grad_pair(const uint16_t* X, int64_t ldx, int64_t c_in, const uint16_t* T1_hi,
                                 const uint16_t* T1_lo, float* partial_a, float* dA, const uint16_t* dY, int64_t lddy,
                                 int64_t c_out, const uint16_t* T2_hi, const uint16_t* T2_lo, float* partial_b,
                                 float* dB, int64_t t, int32_t r, hipStream_t stream);

// Full-precision dX on the outlier channels (quaff_outlier_grad.hip).  Scratch: L [64 x c_out] bf16,
// T_hi / T_lo [kLoraParts x t x 64] bf16.
hipError_t launch_outlier_grad(const uint16_t* dY, int64_t t, int64_t lddy, int64_t c_out, const int32_t* O, int32_t n,
                               const float* W_O, const uint16_t* lora_A, const uint16_t* lora_B, int32_t r, float scale,
                               float* dX, int64_t lddx, uint16_t* L, uint16_t* T_hi, uint16_t* T_lo,
                               hipStream_t stream);

// Outlier-channel identification (quaff_calib.hip).  Scratch: colmax [n_samples x 8 x c_in] bf16 magnitudes, part_sum
// [n_samples x 8 x ceil(c_in / 2048)] fp64 (8 row slabs per sample), rank [c_in] int32.
hipError_t launch_calibrate(const uint16_t* X, int64_t ldx, int64_t c_in, int64_t t_total, const int64_t* offsets,
                            int32_t n_samples, double ratio, int32_t budget, int32_t* xi, int32_t* O, int32_t* n_out,
                            uint16_t* colmax, double* part_sum, int32_t* rank, hipStream_t stream);

// Quantizer (colscale = cs, no outlier copy) and LoRA down-projection with a contraction-contiguous factor
// L [r x c] of the same bf16 matrix X in ONE launch (quaff_quant_lora.hip).  Returns false, with nothing enqueued,
// for shapes it does not cover; otherwise *err holds the launch status.
bool launch_quant_lora(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const float* cs, int8_t* Xq, float* delta,
                       const uint16_t* L_r_by_c, int32_t r, float scale, uint16_t* T_hi, uint16_t* T_lo,
                       hipStream_t stream, hipError_t* err);

// Persistent LoRA down-projection for long inputs at rank 16 (quaff_lora_stream.hip): same bits as launch_lora_down.
// With O / part / s_O / s_prev (n > 0) the same pass writes the abs-max slabs part [lora_stream_row_groups(t) x n] of the
// outlier columns and copies s_O to s_prev, as the stand-alone abs-max kernel does.
bool lora_stream_applies(int32_t r, int64_t t, int64_t c, int32_t n_colmax);
int lora_stream_row_groups(int64_t t);
hipError_t launch_lora_stream(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const uint16_t* L, bool L_is_r_by_c,
                              float scale, uint16_t* T_hi, uint16_t* T_lo, const uint16_t* tr_src, uint16_t* tr_dst,
                              int64_t tr_rows, int64_t tr_cols, const int32_t* O, int32_t n, uint32_t* part,
                              const float* s_O, float* s_prev, hipStream_t stream);

// Pieces of the fused forward step (quaff_linear_fwd_step): the abs-max slabs and the LoRA down-projection of X in
// one launch (quaff_fwd_step.hip), then the momentum / what kernel on those slabs (quaff_scale.hip).
int scale_update_gather_slabs(int64_t t, int32_t n);   // slab count the gather variant of the abs-max uses
hipError_t launch_colmax_lora(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const int32_t* O, int32_t n,
                              uint32_t* part, const float* s_O, float* s_prev, int nslab, const uint16_t* A, int32_t r,
                              float scale, uint16_t* T_hi, uint16_t* T_lo, const uint16_t* B, uint16_t* Bt,
                              int64_t c_out, hipStream_t stream, uint16_t* At_scratch = nullptr);
hipError_t launch_momentum(const uint32_t* part, int nslab, int n, int n_pad, const float* wmax_O, const float* s_prev,
                           float gamma, const int32_t* O, float* s_O, float* colscale, float* cmax_out,
                           const float* W_O, int64_t c_out, int8_t* what_int, float* delta_what, hipStream_t stream);

// Momentum / what requantization and the quantizer of X in ONE launch (quaff_what_quant.hip); arguments as for
// launch_momentum and launch_quant_act.  Returns false, with nothing enqueued, for shapes it does not cover.
bool launch_what_quant(const uint32_t* part, int nslab, int32_t n, const float* wmax_O, const float* s_prev, float gamma,
                       const int32_t* O, float* s_O, float* colscale, float* cmax_out, const float* W_O, int64_t c_out,
                       int8_t* what_int, float* delta_what, const uint16_t* X, int64_t t, int64_t c, int64_t ldx,
                       int8_t* Xq, float* delta, int8_t* xq_O, hipStream_t stream, hipError_t* err);

// The whole forward preparation (abs-max, momentum, what, quantizer, down-projection, transposed B) in one launch and
// one pass over X (quaff_fwd_prep.hip).  `scratch` (fwd_prep_scratch_bytes(n) bytes, 256-byte aligned) holds the arrival
// word of the bounded grid-wide wait and the per-workgroup column maxima; wait_ticks bounds that wait (100 MHz ticks).
bool fwd_prep_covers(int64_t t, int64_t c_in, int32_t n, int32_t r);
size_t fwd_prep_scratch_bytes(int32_t n);
hipError_t launch_fwd_prep(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const int32_t* O, int32_t n,
                           const float* wmax_O, float gamma, float* s_O, float* colscale, float* cmax_out,
                           const float* W_O, int64_t c_out, int8_t* what_int, float* delta_what, int8_t* Xq,
                           float* delta, int8_t* xq_O, const uint16_t* A, const uint16_t* B, int32_t r, float scale,
                           uint16_t* T_hi, uint16_t* T_lo, uint16_t* Bt, void* scratch, long long wait_ticks,
                           hipStream_t stream);

// Packed weight codes: one int8 copy that serves both products.  Element (j, k) of the [c_out x c_in] code matrix
// sits in a 128-byte line that holds 64 consecutive k of the two rows j & ~1 and j | 1: every 16-byte chunk is
// contraction-contiguous for the forward product, and both products fetch whole lines (the input-gradient tiles are
// 128 rows tall and a multiple of 64 columns wide).  `cpad` = c_in rounded up to a multiple of 64.
enum BLayout { kPlain = 0, kPackedNK = 1, kPackedKN = 2 };
__host__ __device__ inline int64_t weight_code_offset(int64_t j, int64_t k, int64_t cpad) {
    return (j >> 1) * (2 * cpad) + (k >> 6) * 128 + (j & 1) * 64 + (k & 63);
}

inline int64_t packed_weight_cpad(int64_t c_in) { return (c_in + 63) / 64 * 64; }
inline size_t packed_weight_bytes(int64_t c_in, int64_t c_out) {
    return (size_t)((c_out + 1) / 2 * 2) * (size_t)packed_weight_cpad(c_in);
}

struct GemmArgs {
    // C[M x N] from A [M x K] int8 (lda) and B [N x K] int8 (ldb), both contraction-contiguous
    const int8_t* A; int64_t lda;
    const int8_t* B; int64_t ldb;
    // Layout of B.  kPlain: [N x K] as above.  The other two read the packed weight codes (weight_code_offset):
    // kPackedNK as [N x K] with N = c_out rows and K = c_in (the forward product), kPackedKN as [K x N] with
    // K = c_out and N = c_in (the input-gradient product, transposing LDS reads); ldb is then c_in rounded up to 64.
    int32_t b_layout;
    int64_t M, N, K;
    // optional second product with its own column scale: A2 [M x K2], B2 [N x K2], K2 a multiple of 64 (0 = none)
    const int8_t* A2; const int8_t* B2; int32_t K2;
    const float* row_scale;    // [M]
    const float* col_scale;    // [N] or nullptr (= 1)
    const float* col_scale2;   // [N]
    // optional low-rank fp term: sum over kLoraParts parts p of (T_hi[p] + T_lo[p]) [M x r] bf16, times L [N x r] bf16
    // (r-contiguous); part p starts M * r elements after part p - 1
    const uint16_t* T_hi; const uint16_t* T_lo; const uint16_t* L; int32_t r;
    float* C; int64_t ldc;         // fp32 output (mode 0)
    uint16_t* C16;                 // fast kernel only: bf16 output instead of C (same ldc, in elements; not with accumulate)
    int32_t accumulate;            // fast kernel only: add the result to what C already holds instead of overwriting it
                                   // (selects a separate kernel instantiation)
    int32_t* acc1; int32_t* acc2;  // int32 dumps (mode 1), dense ld = N
    // optional scratch for a contraction split over two workgroups per tile (fast kernel; gemm_split_bytes(M, N) bytes,
    // 256-byte aligned; nullptr = never split) and the bound of the taker's wait in 100 MHz ticks
    void* split_scratch; long long split_wait_ticks;
};
size_t gemm_split_bytes(int64_t M, int64_t N, int64_t K);   // 0 for products that are not split
hipError_t launch_gemm(const GemmArgs& g, bool dump_acc, hipStream_t stream);

}  // namespace quaff
