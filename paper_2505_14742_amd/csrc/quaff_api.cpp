// C ABI of libquaff: argument checking, workspace carving and kernel launches.  No computation happens here.
#include "../../include/quaff.h"
#include "quaff_internal.h"
#include <atomic>
#include <functional>

namespace {

thread_local int g_last_hip_error = 0;
// bound of the grid-wide wait of the one-launch forward preparation, in 100 MHz ticks (quaff_debug_grid_wait_ticks)
std::atomic<long long> g_grid_wait_ticks{5000};

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int32_t pad_outliers(int32_t n) { return (n + quaff::kPadK - 1) / quaff::kPadK * quaff::kPadK; }

int hip_status(hipError_t e) {
    if (e == hipSuccess) return QUAFF_OK;
    g_last_hip_error = (int)e;
    return QUAFF_ERR_HIP;
}

bool dims_ok(int64_t t, int64_t c_in, int64_t c_out) {
    const int64_t lim = (int64_t)1 << 30;
    return t >= 1 && t < lim && c_in >= 16 && c_out >= 16 && c_in < (1 << 20) && c_out < (1 << 20) &&
           c_in % 16 == 0 && c_out % 16 == 0;
}
bool rank_ok(int32_t r) { return r == 0 || (r > 0 && r <= 64 && r % 16 == 0); }
// leading dimension of an output of the products (the store addressing keeps four rows in a 32-bit offset)
bool out_ld_ok(int64_t ld, int64_t cols) { return ld >= cols && ld < ((int64_t)1 << 27); }

// the packed weight codes as the B operand of the forward (c_out x c_in) or of the input-gradient product
void set_weight_operand(quaff::GemmArgs& g, const void* packed, int64_t c_in, bool gradient) {
    g.B = static_cast<const int8_t*>(packed);
    g.ldb = quaff::packed_weight_cpad(c_in);
    g.b_layout = gradient ? quaff::kPackedKN : quaff::kPackedNK;
}

// workspace layouts -------------------------------------------------------------------------------
size_t ws_scale(int64_t t, int32_t n) { return align_up(((size_t)quaff::scale_update_blocks(t) * n + n) * sizeof(float)); }
struct FwdWs { size_t t_hi, t_lo, lt, at, total; };
FwdWs ws_fwd(int64_t t, int64_t c_in, int64_t c_out, int32_t r) {
    FwdWs w{};
    size_t off = 0;
    w.t_hi = off; off += align_up((size_t)quaff::kLoraParts * t * r * 2);
    w.t_lo = off; off += align_up((size_t)quaff::kLoraParts * t * r * 2);
    w.lt = off;   off += align_up((size_t)c_out * r * 2);
    w.at = off;   off += quaff::lora_prefers_transposed(r, t) ? align_up((size_t)c_in * r * 2) : 0;   // A^T [r x c_in]
    w.total = off;
    return w;
}
struct BwdWs { size_t gq, dg, t_hi, t_lo, split, total; };
BwdWs ws_bwd(int64_t t, int64_t c_in, int64_t c_out, int32_t r) {
    BwdWs w{};
    size_t off = 0;
    w.gq = off;   off += align_up((size_t)t * c_out);
    w.dg = off;   off += align_up((size_t)t * 4);
    w.t_hi = off; off += align_up((size_t)quaff::kLoraParts * t * r * 2);
    w.t_lo = off; off += align_up((size_t)quaff::kLoraParts * t * r * 2);
    w.split = off; off += align_up(quaff::gemm_split_bytes(t, c_in, c_out));   // dX [t x c_in], contraction c_out
    w.total = off;
    return w;
}

struct GradWs { size_t t1_hi, t1_lo, t2_hi, t2_lo, part_a, part_b, at, total; };
GradWs ws_grad(int64_t t, int64_t c_in, int64_t c_out, int32_t r) {
    GradWs w{};
    const size_t tbytes = align_up((size_t)quaff::kLoraParts * t * r * 2);
    int nslab_a, nslab_b, rows;
    quaff::lora_grad_plan(t, c_in, &nslab_a, &rows);
    quaff::lora_grad_plan(t, c_out, &nslab_b, &rows);
    size_t off = 0;
    w.t1_hi = off; off += tbytes;
    w.t1_lo = off; off += tbytes;
    w.t2_hi = off; off += tbytes;
    w.t2_lo = off; off += tbytes;
    w.part_a = off; off += align_up((size_t)nslab_a * r * c_in * 4);
    w.part_b = off; off += align_up((size_t)nslab_b * r * c_out * 4);
    w.at = off; off += quaff::lora_prefers_transposed(r, t) ? align_up((size_t)c_in * r * 2) : 0;   // A^T [r x c_in]
    w.total = off;
    return w;
}

}  // namespace

extern "C" {

const char* quaff_status_string(int status) {
    switch (status) {
        case QUAFF_OK: return "QUAFF_OK";
        case QUAFF_ERR_NULL: return "QUAFF_ERR_NULL: a required pointer is NULL";
        case QUAFF_ERR_SHAPE: return "QUAFF_ERR_SHAPE: a size is out of the supported range";
        case QUAFF_ERR_WORKSPACE: return "QUAFF_ERR_WORKSPACE: workspace missing or too small";
        case QUAFF_ERR_ALIGN: return "QUAFF_ERR_ALIGN: a pointer or leading dimension is misaligned";
        case QUAFF_ERR_HIP: return "QUAFF_ERR_HIP: a HIP call failed";
        default: return "unknown quaff status";
    }
}

int quaff_last_hip_error(void) { return g_last_hip_error; }

int32_t quaff_padded_outliers(int32_t n_outlier) { return n_outlier <= 0 ? 0 : pad_outliers(n_outlier); }

size_t quaff_packed_weight_bytes(int64_t c_in, int64_t c_out) {
    if (c_in <= 0 || c_out <= 0) return 0;
    return align_up(quaff::packed_weight_bytes(c_in, c_out));
}

int64_t quaff_packed_weight_offset(int64_t c_in, int64_t c_out, int64_t k, int64_t j) {
    if (c_in <= 0 || c_out <= 0 || k < 0 || k >= c_in || j < 0 || j >= c_out) return -1;
    return quaff::weight_code_offset(j, k, quaff::packed_weight_cpad(c_in));
}

size_t quaff_prepare_workspace_bytes(int64_t c_in, int64_t c_out) {
    if (c_in <= 0 || c_out <= 0) return 0;
    return align_up(((size_t)((c_in + 63) / 64) + 1) * (size_t)c_out * sizeof(float));
}

size_t quaff_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t n_outlier, int32_t lora_rank) {
    if (t <= 0 || c_in <= 0 || c_out <= 0 || n_outlier < 0 || lora_rank < 0) return 0;
    size_t a = ws_scale(t, n_outlier), b = ws_fwd(t, c_in, c_out, lora_rank).total, c = ws_bwd(t, c_in, c_out, lora_rank).total;
    size_t m = a > b ? a : b;
    return (m > c ? m : c) + 256;
}

int quaff_prepare_weight(const float* W, int64_t c_in, int64_t c_out, int64_t ldw, const int32_t* O, int32_t n_outlier,
                         void* Wq_packed, float* delta_w, float* W_O, float* wmax_O, int8_t* Wq_plain, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (!W || !Wq_packed || !delta_w) return QUAFF_ERR_NULL;
    if (n_outlier > 0 && (!O || !W_O || !wmax_O)) return QUAFF_ERR_NULL;
    if (!dims_ok(1, c_in, c_out) || n_outlier < 0 || n_outlier > c_in || ldw < c_out) return QUAFF_ERR_SHAPE;
    if (!workspace || workspace_bytes < quaff_prepare_workspace_bytes(c_in, c_out)) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(W) || !aligned16(Wq_packed) || !aligned16(workspace)) return QUAFF_ERR_ALIGN;
    return hip_status(quaff::launch_prepare_weight(W, c_in, c_out, ldw, O, n_outlier, static_cast<int8_t*>(Wq_packed), delta_w, W_O,
                                                   wmax_O, Wq_plain, static_cast<float*>(workspace),
                                                   static_cast<hipStream_t>(stream)));
}

int quaff_scale_update(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O, int32_t n_outlier,
                       const float* W_O, const float* wmax_O, int64_t c_out, float gamma, float* s_O, float* colscale,
                       int8_t* what_int, float* delta_what, float* cmax_out, void* workspace, size_t workspace_bytes,
                       void* stream) {
    if (n_outlier == 0) return dims_ok(t, c_in, c_out) ? QUAFF_OK : QUAFF_ERR_SHAPE;
    if (!X || !O || !W_O || !wmax_O || !s_O || !colscale || !what_int || !delta_what) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || n_outlier < 0 || n_outlier > c_in || n_outlier > 8192 || ldx < c_in ||
        !(gamma >= 0.0f && gamma <= 1.0f))
        return QUAFF_ERR_SHAPE;
    if (!workspace || workspace_bytes < ws_scale(t, n_outlier)) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(what_int) || !aligned16(workspace) || ldx % 8 != 0) return QUAFF_ERR_ALIGN;
    return hip_status(quaff::launch_scale_update(X, t, c_in, ldx, O, n_outlier, W_O, wmax_O, c_out, gamma, s_O,
                                                 colscale, what_int, delta_what, cmax_out,
                                                 static_cast<float*>(workspace), static_cast<hipStream_t>(stream)));
}

int quaff_check_outliers(const int32_t* O, int32_t n_outlier, int64_t c_in, int32_t* result, void* stream) {
    if (!result || (n_outlier > 0 && !O)) return QUAFF_ERR_NULL;
    if (n_outlier < 0 || c_in < 1 || c_in >= (1 << 20)) return QUAFF_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(O) | reinterpret_cast<uintptr_t>(result)) & 3u) return QUAFF_ERR_ALIGN;
    return hip_status(quaff::launch_check_outliers(O, n_outlier, c_in, result, static_cast<hipStream_t>(stream)));
}

int32_t quaff_scale_update_static_max_outliers(void) { return quaff::scale_update_static_max_outliers(); }

int quaff_scale_update_static(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O,
                              int32_t n_outlier, const float* W_O, const float* wmax_O, int64_t c_out, float gamma,
                              float* s_O, float* colscale, int8_t* what_int, float* delta_what, float* cmax_out,
                              void* stream) {
    if (n_outlier == 0) return dims_ok(t, c_in, c_out) ? QUAFF_OK : QUAFF_ERR_SHAPE;
    if (!X || !O || !W_O || !wmax_O || !s_O || !colscale || !what_int || !delta_what) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || n_outlier < 0 || n_outlier > c_in ||
        n_outlier > quaff::scale_update_static_max_outliers() || ldx < c_in || !(gamma >= 0.0f && gamma <= 1.0f))
        return QUAFF_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(what_int) || ldx % 8 != 0) return QUAFF_ERR_ALIGN;
    float* scratch_ptr = nullptr;
    int st = hip_status(quaff::scale_update_static_scratch(&scratch_ptr));
    if (st != QUAFF_OK) return st;
    return hip_status(quaff::launch_scale_update(X, t, c_in, ldx, O, n_outlier, W_O, wmax_O, c_out, gamma, s_O,
                                                 colscale, what_int, delta_what, cmax_out, scratch_ptr,
                                                 static_cast<hipStream_t>(stream)));
}

int quaff_quant_act(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const float* colscale, const int32_t* O,
                    int32_t n_outlier, int8_t* Xq, float* delta, int8_t* xq_O, void* stream) {
    if (!X || !Xq || !delta) return QUAFF_ERR_NULL;
    if (xq_O && n_outlier > 0 && !O) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c, 16) || n_outlier < 0 || n_outlier > c || ldx < c) return QUAFF_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Xq) || (colscale && !aligned16(colscale)) || ldx % 8 != 0) return QUAFF_ERR_ALIGN;
    if (n_outlier == 0) xq_O = nullptr;
    return hip_status(quaff::launch_quant_act(X, t, c, ldx, colscale, O, n_outlier, Xq, delta, xq_O,
                                              static_cast<hipStream_t>(stream)));
}

static int fwd_common(const int8_t* Xq, const float* delta_x, const int8_t* xq_O, int64_t t, const void* Wq_packed,
                      const float* delta_w, int64_t c_in, int64_t c_out, const int8_t* what_int,
                      const float* delta_what, int32_t n_outlier, quaff::GemmArgs& g) {
    if (!Xq || !Wq_packed) return QUAFF_ERR_NULL;
    if (n_outlier > 0 && (!xq_O || !what_int)) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || n_outlier < 0 || n_outlier > c_in) return QUAFF_ERR_SHAPE;
    if (!aligned16(Xq) || !aligned16(Wq_packed) || (n_outlier > 0 && (!aligned16(xq_O) || !aligned16(what_int))))
        return QUAFF_ERR_ALIGN;
    g = quaff::GemmArgs{};
    g.A = Xq; g.lda = c_in;
    set_weight_operand(g, Wq_packed, c_in, false);
    g.M = t; g.N = c_out; g.K = c_in;
    g.K2 = n_outlier > 0 ? pad_outliers(n_outlier) : 0;
    g.A2 = xq_O; g.B2 = what_int;
    g.row_scale = delta_x; g.col_scale = delta_w; g.col_scale2 = delta_what;
    return QUAFF_OK;
}

// Y32 (fp32) or Y16 (bf16) receives the result
static int linear_fwd_impl(const int8_t* Xq, const float* delta_x, const int8_t* xq_O, int64_t t, const void* Wq_packed,
                           const float* delta_w, int64_t c_in, int64_t c_out, const int8_t* what_int,
                           const float* delta_what, int32_t n_outlier, const uint16_t* X, int64_t ldx,
                           const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale,
                           float* Y, uint16_t* Y16, int64_t ldy, void* workspace, size_t workspace_bytes,
                           void* stream) {
    quaff::GemmArgs g;
    int st = fwd_common(Xq, delta_x, xq_O, t, Wq_packed, delta_w, c_in, c_out, what_int, delta_what, n_outlier, g);
    if (st != QUAFF_OK) return st;
    if (!delta_x || !delta_w || (!Y && !Y16) || (n_outlier > 0 && !delta_what)) return QUAFF_ERR_NULL;
    if (!rank_ok(lora_rank) || !out_ld_ok(ldy, c_out)) return QUAFF_ERR_SHAPE;
    if (Y16 && (c_in % 64 != 0 || n_outlier > 128)) return QUAFF_ERR_SHAPE;
    if (Y16 && (!aligned16(Y16) || ldy % 8 != 0)) return QUAFF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lora_rank > 0) {
        if (!X || !lora_A || !lora_B) return QUAFF_ERR_NULL;
        if (ldx < c_in) return QUAFF_ERR_SHAPE;
        FwdWs w = ws_fwd(t, c_in, c_out, lora_rank);
        if (!workspace || workspace_bytes < w.total) return QUAFF_ERR_WORKSPACE;
        if (!aligned16(X) || !aligned16(lora_A) || !aligned16(lora_B) || !aligned16(workspace) || ldx % 8 != 0)
            return QUAFF_ERR_ALIGN;
        char* base = static_cast<char*>(workspace);
        uint16_t* t_hi = reinterpret_cast<uint16_t*>(base + w.t_hi);
        uint16_t* t_lo = reinterpret_cast<uint16_t*>(base + w.t_lo);
        uint16_t* lt = reinterpret_cast<uint16_t*>(base + w.lt);
        // T = scale * X A (A is [c_in x r]); B [r x c_out] -> B^T [c_out x r] for the epilogue
        st = hip_status(quaff::launch_lora_down(X, t, c_in, ldx, lora_A, false, lora_rank, lora_scale, t_hi, t_lo,
                                                lora_B, lt, lora_rank, c_out, s,
                                                reinterpret_cast<uint16_t*>(base + w.at)));
        if (st != QUAFF_OK) return st;
        g.T_hi = t_hi; g.T_lo = t_lo; g.L = lt; g.r = lora_rank;
    }
    g.C = Y; g.C16 = Y16; g.ldc = ldy;
    return hip_status(quaff::launch_gemm(g, false, s));
}

int quaff_linear_fwd(const int8_t* Xq, const float* delta_x, const int8_t* xq_O, int64_t t, const void* Wq_packed,
                     const float* delta_w, int64_t c_in, int64_t c_out, const int8_t* what_int,
                     const float* delta_what, int32_t n_outlier, const uint16_t* X, int64_t ldx,
                     const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* Y,
                     int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    return linear_fwd_impl(Xq, delta_x, xq_O, t, Wq_packed, delta_w, c_in, c_out, what_int, delta_what, n_outlier, X,
                           ldx, lora_A, lora_B, lora_rank, lora_scale, Y, nullptr, ldy, workspace, workspace_bytes,
                           stream);
}

int quaff_linear_fwd_bf16(const int8_t* Xq, const float* delta_x, const int8_t* xq_O, int64_t t, const void* Wq_packed,
                          const float* delta_w, int64_t c_in, int64_t c_out, const int8_t* what_int,
                          const float* delta_what, int32_t n_outlier, const uint16_t* X, int64_t ldx,
                          const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale,
                          uint16_t* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    if (!Y) return QUAFF_ERR_NULL;
    return linear_fwd_impl(Xq, delta_x, xq_O, t, Wq_packed, delta_w, c_in, c_out, what_int, delta_what, n_outlier, X,
                           ldx, lora_A, lora_B, lora_rank, lora_scale, nullptr, Y, ldy, workspace, workspace_bytes,
                           stream);
}

int quaff_linear_fwd_acc(const int8_t* Xq, const int8_t* xq_O, int64_t t, const void* Wq_packed, int64_t c_in,
                         int64_t c_out, const int8_t* what_int, int32_t n_outlier, int32_t* acc1, int32_t* acc2,
                         void* stream) {
    quaff::GemmArgs g;
    int st = fwd_common(Xq, nullptr, xq_O, t, Wq_packed, nullptr, c_in, c_out, what_int, nullptr, n_outlier, g);
    if (st != QUAFF_OK) return st;
    if (!acc1) return QUAFF_ERR_NULL;
    g.acc1 = acc1; g.acc2 = acc2;
    return hip_status(quaff::launch_gemm(g, true, static_cast<hipStream_t>(stream)));
}

static int linear_bwd_dx_impl(const uint16_t* dY, int64_t t, int64_t lddy, const void* Wq_packed, const float* delta_w,
                              int64_t c_in, int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B,
                              int32_t lora_rank, float lora_scale, float* dX, uint16_t* dX16, int64_t lddx,
                              void* workspace, size_t workspace_bytes, void* stream,
                              const std::function<int()>* before_product = nullptr) {
    if (!dY || !Wq_packed || !delta_w || (!dX && !dX16)) return QUAFF_ERR_NULL;
    if (dX16 && c_out % 64 != 0) return QUAFF_ERR_SHAPE;
    if (dX16 && (!aligned16(dX16) || lddx % 8 != 0)) return QUAFF_ERR_ALIGN;
    if (lora_rank > 0 && (!lora_A || !lora_B)) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || !rank_ok(lora_rank) || lddy < c_out || !out_ld_ok(lddx, c_in)) return QUAFF_ERR_SHAPE;
    BwdWs w = ws_bwd(t, c_in, c_out, lora_rank);
    if (!workspace || workspace_bytes < w.total) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(dY) || !aligned16(Wq_packed) || !aligned16(delta_w) || !aligned16(workspace) || lddy % 8 != 0 ||
        (lora_rank > 0 && (!aligned16(lora_A) || !aligned16(lora_B))))
        return QUAFF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    int8_t* gq = reinterpret_cast<int8_t*>(base + w.gq);
    float* dg = reinterpret_cast<float*>(base + w.dg);
    quaff::GemmArgs g{};
    g.A = gq; g.lda = c_out;
    set_weight_operand(g, Wq_packed, c_in, true);
    g.M = t; g.N = c_in; g.K = c_out;
    g.row_scale = dg;
    int st;
    bool quantized = false;
    if (lora_rank > 0) {
        uint16_t* t_hi = reinterpret_cast<uint16_t*>(base + w.t_hi);
        uint16_t* t_lo = reinterpret_cast<uint16_t*>(base + w.t_lo);
        // T = scale * dY B^T (B is [r x c_out], contraction-contiguous); the epilogue multiplies by A [c_in x r].
        // The quantizer and this down-projection both only read dY: one launch runs them side by side when it can.
        hipError_t e = hipSuccess;
        quantized = quaff::launch_quant_lora(dY, t, c_out, lddy, delta_w, gq, dg, lora_B, lora_rank, lora_scale, t_hi,
                                             t_lo, s, &e);
        if (quantized) {
            if ((st = hip_status(e)) != QUAFF_OK) return st;
        } else {
            st = hip_status(quaff::launch_lora_down(dY, t, c_out, lddy, lora_B, true, lora_rank, lora_scale, t_hi,
                                                    t_lo, nullptr, nullptr, 0, 0, s));
            if (st != QUAFF_OK) return st;
        }
        g.T_hi = t_hi; g.T_lo = t_lo; g.L = lora_A; g.r = lora_rank;
    }
    if (!quantized) {
        st = hip_status(quaff::launch_quant_act(dY, t, c_out, lddy, delta_w, nullptr, 0, gq, dg, nullptr, s));
        if (st != QUAFF_OK) return st;
    }
    g.C = dX; g.C16 = dX16; g.ldc = lddx;
    if (w.total > w.split) { g.split_scratch = base + w.split; g.split_wait_ticks = g_grid_wait_ticks.load(); }
    // (the one-call backward step forks its weight-gradient work here: the quantizer and the down-projection are
    // enqueued, the long product is not yet)
    if (before_product && (st = (*before_product)()) != QUAFF_OK) return st;
    return hip_status(quaff::launch_gemm(g, false, s));
}

int quaff_linear_bwd_dx(const uint16_t* dY, int64_t t, int64_t lddy, const void* Wq_packed, const float* delta_w,
                        int64_t c_in, int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank,
                        float lora_scale, float* dX, int64_t lddx, void* workspace, size_t workspace_bytes,
                        void* stream) {
    return linear_bwd_dx_impl(dY, t, lddy, Wq_packed, delta_w, c_in, c_out, lora_A, lora_B, lora_rank, lora_scale, dX,
                              nullptr, lddx, workspace, workspace_bytes, stream);
}

int quaff_linear_bwd_dx_bf16(const uint16_t* dY, int64_t t, int64_t lddy, const void* Wq_packed, const float* delta_w,
                             int64_t c_in, int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B,
                             int32_t lora_rank, float lora_scale, uint16_t* dX, int64_t lddx, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (!dX) return QUAFF_ERR_NULL;
    return linear_bwd_dx_impl(dY, t, lddy, Wq_packed, delta_w, c_in, c_out, lora_A, lora_B, lora_rank, lora_scale,
                              nullptr, dX, lddx, workspace, workspace_bytes, stream);
}

int quaff_linear_bwd_dx_acc(const uint16_t* dY, int64_t t, int64_t lddy, const void* Wq_packed, const float* delta_w,
                            int64_t c_in, int64_t c_out, int8_t* Gq, float* delta_g, int32_t* acc, void* stream) {
    if (!dY || !Wq_packed || !delta_w || !Gq || !delta_g || !acc) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || lddy < c_out) return QUAFF_ERR_SHAPE;
    if (!aligned16(dY) || !aligned16(Wq_packed) || !aligned16(delta_w) || !aligned16(Gq) || lddy % 8 != 0)
        return QUAFF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int st = hip_status(quaff::launch_quant_act(dY, t, c_out, lddy, delta_w, nullptr, 0, Gq, delta_g, nullptr, s));
    if (st != QUAFF_OK) return st;
    quaff::GemmArgs g{};
    g.A = Gq; g.lda = c_out;
    set_weight_operand(g, Wq_packed, c_in, true);
    g.M = t; g.N = c_in; g.K = c_out;
    g.acc1 = acc;
    return hip_status(quaff::launch_gemm(g, true, s));
}

size_t quaff_lora_bwd_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t lora_rank) {
    if (t <= 0 || c_in <= 0 || c_out <= 0 || lora_rank <= 0) return 0;
    return ws_grad(t, c_in, c_out, lora_rank).total + 256;
}

int quaff_lora_bwd_weights(const uint16_t* X, int64_t ldx, const uint16_t* dY, int64_t lddy, int64_t t, int64_t c_in,
                           int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank,
                           float lora_scale, float* dA, float* dB, void* workspace, size_t workspace_bytes,
                           void* stream) {
    if (!X || !dY || !lora_A || !lora_B || !dA || !dB) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || !rank_ok(lora_rank) || lora_rank == 0 || ldx < c_in || lddy < c_out)
        return QUAFF_ERR_SHAPE;
    GradWs w = ws_grad(t, c_in, c_out, lora_rank);
    if (!workspace || workspace_bytes < w.total) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(dY) || !aligned16(lora_A) || !aligned16(lora_B) || !aligned16(workspace) ||
        ldx % 8 != 0 || lddy % 8 != 0)
        return QUAFF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    auto u16 = [&](size_t off) { return reinterpret_cast<uint16_t*>(base + off); };
    // T1 = scale dY B^T (B is [r x c_out]) and T2 = scale X A (A is [c_in x r]), as the hi/lo parts of the
    // down-projection
    int st = hip_status(quaff::launch_lora_down_pair(dY, lddy, c_out, lora_B, u16(w.t1_hi), u16(w.t1_lo), X, ldx, c_in,
                                                     lora_A, u16(w.t2_hi), u16(w.t2_lo), t, lora_rank, lora_scale,
                                                     u16(w.at), s));
    if (st != QUAFF_OK) return st;
    // dA^T [r x c_in] = T1^T X, stored transposed;  dB [r x c_out] = T2^T dY
    return hip_status(quaff::launch_lora_grad_pair(X, ldx, c_in, u16(w.t1_hi), u16(w.t1_lo),
                                                   reinterpret_cast<float*>(base + w.part_a), dA, dY, lddy, c_out,
                                                   u16(w.t2_hi), u16(w.t2_lo),
                                                   reinterpret_cast<float*>(base + w.part_b), dB, t, lora_rank, s));
}

size_t quaff_bwd_step_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t lora_rank) {
    if (t <= 0 || c_in <= 0 || c_out <= 0 || lora_rank <= 0) return 0;
    return ws_bwd(t, c_in, c_out, lora_rank).total + ws_grad(t, c_in, c_out, lora_rank).total + 256;
}

int quaff_linear_bwd_step(const uint16_t* dY, int64_t t, int64_t lddy, const uint16_t* X, int64_t ldx,
                          const void* Wq_packed, const float* delta_w, int64_t c_in, int64_t c_out,
                          const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* dX,
                          int64_t lddx, float* dA, float* dB, void* workspace, size_t workspace_bytes, void* stream,
                          void* side_stream, void* fork_event, void* join_event) {
    if (!X || !dA || !dB) return QUAFF_ERR_NULL;
    if (!rank_ok(lora_rank) || lora_rank == 0 || t <= 0 || c_in <= 0 || c_out <= 0 || ldx < c_in) return QUAFF_ERR_SHAPE;
    const BwdWs wb = ws_bwd(t, c_in, c_out, lora_rank);
    const GradWs w = ws_grad(t, c_in, c_out, lora_rank);
    if (!workspace || workspace_bytes < wb.total + w.total) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(workspace) || ldx % 8 != 0) return QUAFF_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* bwd = static_cast<char*>(workspace);
    char* base = bwd + wb.total;
    auto u16 = [&](size_t off) { return reinterpret_cast<uint16_t*>(base + off); };
    uint16_t* t1_hi = reinterpret_cast<uint16_t*>(bwd + wb.t_hi);
    uint16_t* t1_lo = reinterpret_cast<uint16_t*>(bwd + wb.t_lo);
    // T2 = scale X A, then the two products of quaff_lora_bwd_weights, on stream `gs`; T1 = scale dY B^T (hi / lo parts)
    // is what the dX call leaves in its part of the workspace
    auto weight_grads = [&](hipStream_t gs) -> int {
        int st = hip_status(quaff::launch_lora_down(X, t, c_in, ldx, lora_A, false, lora_rank, lora_scale, u16(w.t2_hi),
                                                    u16(w.t2_lo), nullptr, nullptr, 0, 0, gs, u16(w.at)));
        if (st != QUAFF_OK) return st;
        return hip_status(quaff::launch_lora_grad_pair(X, ldx, c_in, t1_hi, t1_lo,
                                                       reinterpret_cast<float*>(base + w.part_a), dA, dY, lddy, c_out,
                                                       u16(w.t2_hi), u16(w.t2_lo),
                                                       reinterpret_cast<float*>(base + w.part_b), dB, t, lora_rank,
                                                       gs));
    };
    // With a second stream and two events from the caller, the weight gradients (short, memory-bound kernels) run
    // beside the input-gradient product (long, MFMA-bound): forked from `stream` once T1 exists, joined back into it
    // at the end.  Without them everything runs on `stream`.  The library creates neither streams nor events.
    const bool use_side = side_stream && fork_event && join_event && side_stream != stream;
    hipStream_t gs = static_cast<hipStream_t>(side_stream);
    hipEvent_t ev_fork = static_cast<hipEvent_t>(fork_event), ev_join = static_cast<hipEvent_t>(join_event);
    bool forked = false;
    int side_status = QUAFF_OK;
    const std::function<int()> fork = [&]() -> int {
        if (!use_side) return QUAFF_OK;
        int st = hip_status(hipEventRecord(ev_fork, s));
        if (st != QUAFF_OK) return st;
        if ((st = hip_status(hipStreamWaitEvent(gs, ev_fork, 0))) != QUAFF_OK) return st;
        forked = true;
        side_status = weight_grads(gs);   // reported after the join below
        return QUAFF_OK;
    };
    int st = linear_bwd_dx_impl(dY, t, lddy, Wq_packed, delta_w, c_in, c_out, lora_A, lora_B, lora_rank, lora_scale, dX,
                                nullptr, lddx, workspace, wb.total, stream, &fork);
    if (forked) {
        // Whatever happened after the fork, the caller's stream joins everything that was put on the side stream,
        // so that the buffers that work reads and writes stay ordered before the caller's next use of them.
        int st_rec = hip_status(hipEventRecord(ev_join, gs));
        int st_wait = st_rec == QUAFF_OK ? hip_status(hipStreamWaitEvent(s, ev_join, 0)) : st_rec;
        if (st != QUAFF_OK) return st;
        if (side_status != QUAFF_OK) return side_status;
        return st_wait;
    }
    if (st != QUAFF_OK) return st;
    return weight_grads(s);
}

size_t quaff_bwd_dx_outlier_workspace_bytes(int64_t t, int64_t c_out) {
    if (t <= 0 || c_out <= 0) return 0;
    return align_up((size_t)64 * c_out * 2) + 2 * align_up((size_t)quaff::kLoraParts * t * 64 * 2) + 256;
}

int quaff_bwd_dx_outlier_exact(const uint16_t* dY, int64_t t, int64_t lddy, int64_t c_in, int64_t c_out,
                               const int32_t* O, int32_t n_outlier, const float* W_O, const uint16_t* lora_A,
                               const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* dX, int64_t lddx,
                               void* workspace, size_t workspace_bytes, void* stream) {
    if (n_outlier == 0) return dims_ok(t, c_in, c_out) ? QUAFF_OK : QUAFF_ERR_SHAPE;
    if (!dY || !O || !W_O || !dX) return QUAFF_ERR_NULL;
    if (lora_rank > 0 && (!lora_A || !lora_B)) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || !rank_ok(lora_rank) || n_outlier < 0 || n_outlier > c_in || lddy < c_out ||
        lddx < c_in)
        return QUAFF_ERR_SHAPE;
    const size_t lbytes = align_up((size_t)64 * c_out * 2), tbytes = align_up((size_t)quaff::kLoraParts * t * 64 * 2);
    if (!workspace || workspace_bytes < lbytes + 2 * tbytes) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(dY) || !aligned16(workspace) || lddy % 8 != 0) return QUAFF_ERR_ALIGN;
    char* base = static_cast<char*>(workspace);
    return hip_status(quaff::launch_outlier_grad(
        dY, t, lddy, c_out, O, n_outlier, W_O, lora_A, lora_B, lora_rank, lora_scale, dX, lddx,
        reinterpret_cast<uint16_t*>(base), reinterpret_cast<uint16_t*>(base + lbytes),
        reinterpret_cast<uint16_t*>(base + lbytes + tbytes), static_cast<hipStream_t>(stream)));
}

size_t quaff_calibrate_workspace_bytes(int64_t c_in, int32_t n_samples) {
    if (c_in <= 0 || n_samples <= 0) return 0;
    return align_up((size_t)n_samples * 8 * c_in * 2) + align_up((size_t)n_samples * 8 * ((c_in + 2047) / 2048) * 8) +
           align_up((size_t)c_in * 4) + 256;
}

int quaff_calibrate_outliers(const uint16_t* X, int64_t t_total, int64_t c_in, int64_t ldx,
                             const int64_t* sample_offsets, int32_t n_samples, double ratio, int32_t budget,
                             int32_t* xi, int32_t* O, int32_t* n_outlier, void* workspace, size_t workspace_bytes,
                             void* stream) {
    if (!X || !sample_offsets || !xi) return QUAFF_ERR_NULL;
    if (budget > 0 && (!O || !n_outlier)) return QUAFF_ERR_NULL;
    if (!dims_ok(t_total, c_in, 16) || ldx < c_in || n_samples < 1 || n_samples > 65535 || budget < 0 ||
        budget > c_in || !(ratio > 0.0))
        return QUAFF_ERR_SHAPE;
    const size_t cm = align_up((size_t)n_samples * 8 * c_in * 2);              // 8 row slabs per sample
    const size_t ps = align_up((size_t)n_samples * 8 * ((c_in + 2047) / 2048) * 8);
    if (!workspace || workspace_bytes < cm + ps + align_up((size_t)c_in * 4)) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(workspace) || ldx % 8 != 0) return QUAFF_ERR_ALIGN;
    char* base = static_cast<char*>(workspace);
    return hip_status(quaff::launch_calibrate(X, ldx, c_in, t_total, sample_offsets, n_samples, ratio, budget, xi,
                                              budget > 0 ? O : nullptr, n_outlier, reinterpret_cast<uint16_t*>(base),
                                              reinterpret_cast<double*>(base + cm),
                                              reinterpret_cast<int32_t*>(base + cm + ps),
                                              static_cast<hipStream_t>(stream)));
}

size_t quaff_fwd_step_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t n_outlier, int32_t lora_rank) {
    if (t <= 0 || c_in <= 0 || c_out <= 0 || n_outlier < 0 || lora_rank < 0) return 0;
    return ws_scale(t, n_outlier) + ws_fwd(t, c_in, c_out, lora_rank).total +
           quaff::fwd_prep_scratch_bytes(n_outlier < 64 ? n_outlier : 64) + 256;
}

long long quaff_debug_grid_wait_ticks(long long ticks) {
    return ticks < 0 ? g_grid_wait_ticks.load() : g_grid_wait_ticks.exchange(ticks);
}

int quaff_linear_fwd_step(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O, int32_t n_outlier,
                          const float* W_O, const float* wmax_O, int64_t c_out, float gamma, float* s_O,
                          float* colscale, int8_t* what_int, float* delta_what, float* cmax_out, int8_t* Xq,
                          float* delta_x, int8_t* xq_O, const void* Wq_packed, const float* delta_w,
                          const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* Y,
                          int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    if (t <= 0 || c_in <= 0 || c_out <= 0 || n_outlier < 0 || !rank_ok(lora_rank)) return QUAFF_ERR_SHAPE;
    const size_t scale_bytes = ws_scale(t, n_outlier);
    const FwdWs wf = ws_fwd(t, c_in, c_out, lora_rank);
    const size_t prep_bytes = quaff::fwd_prep_scratch_bytes(n_outlier < 64 ? n_outlier : 64);
    if (!workspace || workspace_bytes < scale_bytes + wf.total + prep_bytes) return QUAFF_ERR_WORKSPACE;
    if (!aligned16(workspace)) return QUAFF_ERR_ALIGN;
    if (!colscale) return QUAFF_ERR_NULL;
    if (n_outlier > 0 && !xq_O) return QUAFF_ERR_NULL;
    char* base = static_cast<char*>(workspace);
    void* ws_lin = base + scale_bytes;
    const size_t ws_lin_bytes = wf.total;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // One launch prepares everything the product needs where it can (a few thousand tokens, at most 64 outlier
    // channels, rank 0 or 16); two combined launches cover the other usual cases; everything else is the three calls
    // one after the other.
    const bool fused = quaff::fwd_prep_covers(t, c_in, n_outlier, lora_rank);
    const bool combined = !fused && n_outlier > 0 && n_outlier <= 1024 && (int64_t)n_outlier * 64 < c_in && lora_rank > 0;
    if (!fused && !combined) {
        int st = quaff_scale_update(X, t, c_in, ldx, O, n_outlier, W_O, wmax_O, c_out, gamma, s_O, colscale, what_int,
                                    delta_what, cmax_out, workspace, scale_bytes, stream);
        if (st != QUAFF_OK) return st;
        st = quaff_quant_act(X, t, c_in, ldx, colscale, O, n_outlier, Xq, delta_x, xq_O, stream);
        if (st != QUAFF_OK) return st;
        return quaff_linear_fwd(Xq, delta_x, xq_O, t, Wq_packed, delta_w, c_in, c_out, what_int, delta_what,
                                n_outlier, X, ldx, lora_A, lora_B, lora_rank, lora_scale, Y, ldy, ws_lin, ws_lin_bytes,
                                stream);
    }
    // argument checks of the three calls (same conditions, same codes)
    if (!X || !O || !W_O || !wmax_O || !s_O || !what_int || !delta_what || !Xq || !delta_x || !Wq_packed || !delta_w || !Y)
        return QUAFF_ERR_NULL;
    if (lora_rank > 0 && (!lora_A || !lora_B)) return QUAFF_ERR_NULL;
    if (!dims_ok(t, c_in, c_out) || n_outlier > c_in || ldx < c_in || !out_ld_ok(ldy, c_out) || !(gamma >= 0.0f && gamma <= 1.0f))
        return QUAFF_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(what_int) || !aligned16(Xq) || !aligned16(colscale) || !aligned16(xq_O) ||
        !aligned16(Wq_packed) || (lora_rank > 0 && (!aligned16(lora_A) || !aligned16(lora_B))) || ldx % 8 != 0)
        return QUAFF_ERR_ALIGN;
    char* lin = static_cast<char*>(ws_lin);
    uint16_t* t_hi = reinterpret_cast<uint16_t*>(lin + wf.t_hi);
    uint16_t* t_lo = reinterpret_cast<uint16_t*>(lin + wf.t_lo);
    uint16_t* lt = reinterpret_cast<uint16_t*>(lin + wf.lt);
    if (fused) {
        int st = hip_status(quaff::launch_fwd_prep(X, t, c_in, ldx, O, n_outlier, wmax_O, gamma, s_O, colscale, cmax_out,
                                                   W_O, c_out, what_int, delta_what, Xq, delta_x, xq_O, lora_A, lora_B,
                                                   lora_rank, lora_scale, t_hi, t_lo, lt,
                                                   base + scale_bytes + wf.total, g_grid_wait_ticks.load(), s));
        if (st != QUAFF_OK) return st;
        quaff::GemmArgs g;
        st = fwd_common(Xq, delta_x, xq_O, t, Wq_packed, delta_w, c_in, c_out, what_int, delta_what, n_outlier, g);
        if (st != QUAFF_OK) return st;
        if (lora_rank > 0) { g.T_hi = t_hi; g.T_lo = t_lo; g.L = lt; g.r = lora_rank; }
        g.C = Y; g.ldc = ldy;
        return hip_status(quaff::launch_gemm(g, false, s));
    }
    float* wsf = static_cast<float*>(workspace);
    // (the persistent down-projection of long inputs yields the abs-max slabs itself, one per row group)
    const int nslab = quaff::lora_stream_applies(lora_rank, t, c_in, n_outlier) ? quaff::lora_stream_row_groups(t)
                                                                                : quaff::scale_update_gather_slabs(t, n_outlier);
    uint32_t* part = reinterpret_cast<uint32_t*>(wsf);
    float* s_prev = wsf + (int64_t)nslab * n_outlier;
    int st = hip_status(quaff::launch_colmax_lora(X, t, c_in, ldx, O, n_outlier, part, s_O, s_prev, nslab, lora_A,
                                                  lora_rank, lora_scale, t_hi, t_lo, lora_B, lt, c_out, s,
                                                  reinterpret_cast<uint16_t*>(lin + wf.at)));
    if (st != QUAFF_OK) return st;
    // The second combined launch pays off while all its workgroups are resident at once (it runs the quantizer at
    // the requantization role's register budget); long inputs take the two stand-alone kernels.
    hipError_t e = hipSuccess;
    if (t <= 4096 &&
        quaff::launch_what_quant(part, nslab, n_outlier, wmax_O, s_prev, gamma, O, s_O, colscale, cmax_out, W_O, c_out,
                                 what_int, delta_what, X, t, c_in, ldx, Xq, delta_x, xq_O, s, &e)) {
        if ((st = hip_status(e)) != QUAFF_OK) return st;
    } else {
        st = hip_status(quaff::launch_momentum(part, nslab, n_outlier, pad_outliers(n_outlier), wmax_O, s_prev, gamma,
                                               O, s_O, colscale, cmax_out, W_O, c_out, what_int, delta_what, s));
        if (st != QUAFF_OK) return st;
        st = hip_status(quaff::launch_quant_act(X, t, c_in, ldx, colscale, O, n_outlier, Xq, delta_x, xq_O, s));
        if (st != QUAFF_OK) return st;
    }
    quaff::GemmArgs g;
    st = fwd_common(Xq, delta_x, xq_O, t, Wq_packed, delta_w, c_in, c_out, what_int, delta_what, n_outlier, g);
    if (st != QUAFF_OK) return st;
    g.T_hi = t_hi; g.T_lo = t_lo; g.L = lt; g.r = lora_rank;
    g.C = Y; g.ldc = ldy;
    return hip_status(quaff::launch_gemm(g, false, s));
}

}  // extern "C"
