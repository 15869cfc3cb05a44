/*
 * CPU oracle for the Quaff weight-activation-quantized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, step-by-step statement
 * of what the layer computes, written from the paper (arXiv 2505.14742).  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline leg;
 * the product (the HIP library) never calls it and shares no code with it.
 *
 * Notation (Sec. 2.2): X is [t x c_in] (t tokens), W is [c_in x c_out], Y = X W.
 * A vector times a matrix scales by row index: [sW]_{i,j} = s_i W_{i,j}
 * (footnote to Eq. 3).  X_{:,O} are the O columns of X, W_O the O rows of W
 * (footnote to Eq. 5).  All matrices are row-major with explicit leading
 * dimensions.  bf16 values arrive as uint16 bit patterns and are widened
 * exactly to fp32.
 *
 * Arithmetic that decides an integer code is done in IEEE fp32, one rounding per
 * written operation (compile with -ffp-contract=off, no fast-math), rounding
 * half to even.  Dequantised outputs are evaluated in fp64 and stored as fp32.
 *
 * Readings where the paper is silent (each is listed in the design notes too):
 *  - [.] in Eq. 1 is round-half-to-even.
 *  - Eq. 1 is evaluated as code = rne(x * c) with c = fl(127 / max|x|) and the
 *    step size Delta = fl(max|x| / 127) kept separately; codes are clamped to
 *    [-127, 127].  An all-zero row/column gets Delta = 0 and all codes 0.
 *  - X s^-1 multiplies by rinv = fl(1 / s), computed once per channel.
 *  - Delta_what is per output channel, like Delta_W.
 *  - max|W_i| in Eq. 8 is the row max of the retained full-precision W_O.
 *  - The backward pass (not described in the paper) uses dX = dY W^T, where s
 *    cancels (Eq. 3): Delta_W is folded into dY before per-token quantization
 *    because it lies on the contraction axis.
 *  - LoRA sees the unscaled, unquantized X; no dropout.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline float bf16_to_f32(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Eq. 1, scalar form: code of x given the reciprocal step c = fl(127/max). */
static inline int8_t rtn_code(float x, float c) {
    float q = nearbyintf(x * c); /* default rounding mode = half to even */
    if (q > 127.0f) q = 127.0f;
    if (q < -127.0f) q = -127.0f;
    return (int8_t)q;
}

/* Step size and its reciprocal for a group whose absolute maximum is m. */
static inline void rtn_steps(float m, float* delta, float* c) {
    if (m > 0.0f) {
        *delta = m / 127.0f;
        *c = 127.0f / m;
    } else {
        *delta = 0.0f;
        *c = 0.0f;
    }
}

/* ------------------------------------------------------------------------
 * Offline preprocessing (Sec. 3.3, first paragraph): W -> W_int, Delta_W per
 * output channel (Eq. 1; App. "Quantization Granularity"), quantized before
 * and independently of s.
 * W [c_in x c_out] fp32 -> Wq [c_in x c_out] int8, delta_w [c_out].
 * ---------------------------------------------------------------------- */
void oracle_weight_quantize(const float* W, int64_t c_in, int64_t c_out, int8_t* Wq, float* delta_w) {
    for (int64_t j = 0; j < c_out; ++j) {
        float m = 0.0f;
        for (int64_t i = 0; i < c_in; ++i) {
            float a = fabsf(W[i * c_out + j]);
            if (a > m) m = a;
        }
        float d, c;
        rtn_steps(m, &d, &c);
        delta_w[j] = d;
        for (int64_t i = 0; i < c_in; ++i) Wq[i * c_out + j] = rtn_code(W[i * c_out + j], c);
    }
}

/* Retained full-precision outlier rows W_O [n x c_out] and wmax_k = max_j |W_O[k,j]|
 * (the max|W_i| of Eq. 8). */
void oracle_outlier_rows(const float* W, int64_t c_in, int64_t c_out, const int32_t* O, int32_t n,
                         float* W_O, float* wmax_O) {
    (void)c_in;
    for (int32_t k = 0; k < n; ++k) {
        float m = 0.0f;
        for (int64_t j = 0; j < c_out; ++j) {
            float w = W[(int64_t)O[k] * c_out + j];
            W_O[(int64_t)k * c_out + j] = w;
            if (fabsf(w) > m) m = fabsf(w);
        }
        wmax_O[k] = m;
    }
}

/* ------------------------------------------------------------------------
 * Targeted momentum scaling (Eq. 7, Eq. 8) and the dynamic outlier weights
 * what = (s_O - 1) W_O with their quantization (Eq. 5, Eq. 9).
 *
 * In/out: s_O [n].  Out: colscale [c_in] gets rinv_k = 1/s_k at O_k (other
 * entries untouched), what_int [n x c_out], delta_what [c_out], cmax_out [n]
 * (optional).
 * ---------------------------------------------------------------------- */
void oracle_scale_update(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O, int32_t n,
                         const float* W_O, const float* wmax_O, int64_t c_out, float gamma, float* s_O,
                         float* colscale, int8_t* what_int, float* delta_what, float* cmax_out) {
    (void)c_in;
    for (int32_t k = 0; k < n; ++k) {
        /* max |X_{:,i}| over all tokens of the current batch, unscaled X */
        float cmax = 0.0f;
        for (int64_t i = 0; i < t; ++i) {
            float a = fabsf(bf16_to_f32(X[i * ldx + O[k]]));
            if (a > cmax) cmax = a;
        }
        if (cmax_out) cmax_out[k] = cmax;
        /* Eq. 8 on i in O */
        float beta = 1.0f;
        if (wmax_O[k] > 0.0f) {
            float q = cmax / wmax_O[k];
            float r = sqrtf(q);
            beta = r > 1.0f ? r : 1.0f;
        }
        /* Eq. 7 */
        float keep = gamma * s_O[k];
        float one_minus_gamma = 1.0f - gamma;
        float fresh = one_minus_gamma * beta;
        float s = keep + fresh;
        s_O[k] = s;
        colscale[O[k]] = 1.0f / s;
    }
    /* what = (s_O - 1) W_O, then Eq. 1 per output channel */
    float* col = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    for (int64_t j = 0; j < c_out; ++j) {
        float m = 0.0f;
        for (int32_t k = 0; k < n; ++k) {
            float sm1 = s_O[k] - 1.0f;
            float w = sm1 * W_O[(int64_t)k * c_out + j];
            col[k] = w;
            if (fabsf(w) > m) m = fabsf(w);
        }
        float d, c;
        rtn_steps(m, &d, &c);
        delta_what[j] = d;
        for (int32_t k = 0; k < n; ++k) what_int[(int64_t)k * c_out + j] = rtn_code(col[k], c);
    }
    free(col);
}

/* ------------------------------------------------------------------------
 * Xhat = X s^-1 on the O columns (Eq. 5), then per-token Eq. 1.
 * colscale may be NULL (all ones).  Used for X (forward) and, with
 * colscale = Delta_W, for dY (backward).
 * Out: Xq [t x c] (ld = c), delta [t], xq_O [t x n] = codes[:, O] (Eq. 9's
 * remark: xhat_int inherits the activation codes).  xq_O may be NULL.
 * ---------------------------------------------------------------------- */
void oracle_quant_act(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const float* colscale, const int32_t* O,
                      int32_t n, int8_t* Xq, float* delta, int8_t* xq_O) {
    float* row = (float*)malloc(sizeof(float) * (size_t)c);
    for (int64_t i = 0; i < t; ++i) {
        float m = 0.0f;
        for (int64_t j = 0; j < c; ++j) {
            float x = bf16_to_f32(X[i * ldx + j]);
            if (colscale) x = x * colscale[j];
            row[j] = x;
            if (fabsf(x) > m) m = fabsf(x);
        }
        float d, cc;
        rtn_steps(m, &d, &cc);
        delta[i] = d;
        for (int64_t j = 0; j < c; ++j) Xq[i * c + j] = rtn_code(row[j], cc);
        if (xq_O)
            for (int32_t k = 0; k < n; ++k) xq_O[i * n + k] = Xq[i * c + O[k]];
    }
    free(row);
}

/* exact integer product C[i,j] = sum_k A[i,k] B[k,j]; A [m x kk] int8, B [kk x nn] int8 (both row-major).
 * |a|,|b| <= 127 so the sum fits int32 whenever 127*127*kk < 2^31; beyond that int64 is used and
 * the caller is told (return value 0) if any element left the int32 range. */
#define INT32_SAFE_K 133000
__attribute__((target_clones("avx2", "default")))
static int int8_matmul(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb, int64_t m, int64_t kk, int64_t nn,
                       int32_t* C) {
    int ok = 1;
    if (kk < INT32_SAFE_K) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            int32_t* c = C + i * nn;
            for (int64_t j = 0; j < nn; ++j) c[j] = 0;
            for (int64_t k = 0; k < kk; ++k) {
                int32_t a = A[i * lda + k];
                const int8_t* b = B + k * ldb;
                for (int64_t j = 0; j < nn; ++j) c[j] += a * (int32_t)b[j];
            }
        }
    } else {
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < nn; ++j) {
                int64_t s = 0;
                for (int64_t k = 0; k < kk; ++k) s += (int64_t)A[i * lda + k] * (int64_t)B[k * ldb + j];
                if (s > INT32_MAX || s < INT32_MIN) ok = 0;
                C[i * nn + j] = (int32_t)s;
            }
    }
    return ok;
}

/* ------------------------------------------------------------------------
 * Integer forward (Eq. 9) plus the LoRA branch:
 *   acc1 = Xq Wq, acc2 = xq_O what_int               (exact integers)
 *   Y = delta_x (acc1 delta_w + acc2 delta_what) + lora_scale (X A) B
 * Wq [c_in x c_out], what_int [n x c_out], xq_O [t x n], A [c_in x r] bf16,
 * B [r x c_out] bf16.  acc1_out/acc2_out [t x c_out] are optional dumps.
 * Returns 1 on success, 0 if an accumulator left the int32 range.
 * ---------------------------------------------------------------------- */
int oracle_linear_fwd(const int8_t* Xq, const float* delta_x, const int8_t* xq_O, int64_t t, const int8_t* Wq,
                      const float* delta_w, int64_t c_in, int64_t c_out, const int8_t* what_int,
                      const float* delta_what, int32_t n, const uint16_t* X, int64_t ldx, const uint16_t* lora_A,
                      const uint16_t* lora_B, int32_t r, float lora_scale, float* Y, int64_t ldy, int32_t* acc1_out,
                      int32_t* acc2_out) {
    int32_t* acc1 = acc1_out ? acc1_out : (int32_t*)malloc(sizeof(int32_t) * (size_t)(t * c_out));
    int32_t* acc2 = acc2_out ? acc2_out : (int32_t*)malloc(sizeof(int32_t) * (size_t)(t * c_out));
    int ok = int8_matmul(Xq, c_in, Wq, c_out, t, c_in, c_out, acc1);
    if (n > 0)
        ok &= int8_matmul(xq_O, n, what_int, c_out, t, n, c_out, acc2);
    else
        memset(acc2, 0, sizeof(int32_t) * (size_t)(t * c_out));

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i) {
        double* T = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        for (int32_t p = 0; p < r; ++p) {
            double s = 0.0;
            for (int64_t k = 0; k < c_in; ++k)
                s += (double)bf16_to_f32(X[i * ldx + k]) * (double)bf16_to_f32(lora_A[k * r + p]);
            T[p] = s;
        }
        for (int64_t j = 0; j < c_out; ++j) {
            double main_term = (double)acc1[i * c_out + j] * (double)delta_w[j];
            double corr_term = (n > 0) ? (double)acc2[i * c_out + j] * (double)delta_what[j] : 0.0;
            double y = (double)delta_x[i] * (main_term + corr_term);
            if (r > 0) {
                double l = 0.0;
                for (int32_t p = 0; p < r; ++p) l += T[p] * (double)bf16_to_f32(lora_B[(int64_t)p * c_out + j]);
                y += (double)lora_scale * l;
            }
            Y[i * ldy + j] = (float)y;
        }
        free(T);
    }
    if (!acc1_out) free(acc1);
    if (!acc2_out) free(acc2);
    return ok;
}

/* ------------------------------------------------------------------------
 * Backward input gradient (reading stated in the header):
 *   G = dY * delta_w (per output channel), per-token Eq. 1 -> Gq, delta_g
 *   acc[i,k] = sum_j Gq[i,j] Wq[k,j]
 *   dX = delta_g acc + lora_scale (dY B^T) A^T
 * Optional dumps: Gq_out [t x c_out], delta_g_out [t], acc_out [t x c_in].
 * ---------------------------------------------------------------------- */
int oracle_linear_bwd_dx(const uint16_t* dY, int64_t t, int64_t lddy, const int8_t* Wq, const float* delta_w,
                         int64_t c_in, int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B, int32_t r,
                         float lora_scale, float* dX, int64_t lddx, int8_t* Gq_out, float* delta_g_out,
                         int32_t* acc_out) {
    int8_t* Gq = Gq_out ? Gq_out : (int8_t*)malloc((size_t)(t * c_out));
    float* dg = delta_g_out ? delta_g_out : (float*)malloc(sizeof(float) * (size_t)t);
    int32_t* acc = acc_out ? acc_out : (int32_t*)malloc(sizeof(int32_t) * (size_t)(t * c_in));
    oracle_quant_act(dY, t, c_out, lddy, delta_w, NULL, 0, Gq, dg, NULL);

    /* W^T as a [c_out x c_in] matrix so the same product routine applies */
    int8_t* Wt = (int8_t*)malloc((size_t)(c_in * c_out));
    for (int64_t k = 0; k < c_in; ++k)
        for (int64_t j = 0; j < c_out; ++j) Wt[j * c_in + k] = Wq[k * c_out + j];
    int ok = int8_matmul(Gq, c_out, Wt, c_in, t, c_out, c_in, acc);
    free(Wt);

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i) {
        double* T = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        for (int32_t p = 0; p < r; ++p) {
            double s = 0.0;
            for (int64_t j = 0; j < c_out; ++j)
                s += (double)bf16_to_f32(dY[i * lddy + j]) * (double)bf16_to_f32(lora_B[(int64_t)p * c_out + j]);
            T[p] = s;
        }
        for (int64_t k = 0; k < c_in; ++k) {
            double g = (double)dg[i] * (double)acc[i * c_in + k];
            if (r > 0) {
                double l = 0.0;
                for (int32_t p = 0; p < r; ++p) l += T[p] * (double)bf16_to_f32(lora_A[k * r + p]);
                g += (double)lora_scale * l;
            }
            dX[i * lddx + k] = (float)g;
        }
        free(T);
    }
    if (!Gq_out) free(Gq);
    if (!delta_g_out) free(dg);
    if (!acc_out) free(acc);
    return ok;
}

/* ------------------------------------------------------------------------
 * Unquantized fp64 references on the full-precision W (for invariants and
 * error-magnitude checks only):
 *   Y*  = X W + lora_scale (X A) B          dX* = dY W^T + lora_scale (dY B^T) A^T
 * ---------------------------------------------------------------------- */
void oracle_ref_fwd_fp64(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const float* W, int64_t c_out,
                         const uint16_t* lora_A, const uint16_t* lora_B, int32_t r, float lora_scale, double* Y) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i) {
        double* y = Y + i * c_out;
        for (int64_t j = 0; j < c_out; ++j) y[j] = 0.0;
        for (int64_t k = 0; k < c_in; ++k) {
            double x = (double)bf16_to_f32(X[i * ldx + k]);
            for (int64_t j = 0; j < c_out; ++j) y[j] += x * (double)W[k * c_out + j];
        }
        for (int32_t p = 0; p < r; ++p) {
            double s = 0.0;
            for (int64_t k = 0; k < c_in; ++k)
                s += (double)bf16_to_f32(X[i * ldx + k]) * (double)bf16_to_f32(lora_A[k * r + p]);
            for (int64_t j = 0; j < c_out; ++j)
                y[j] += (double)lora_scale * s * (double)bf16_to_f32(lora_B[(int64_t)p * c_out + j]);
        }
    }
}

void oracle_ref_bwd_fp64(const uint16_t* dY, int64_t t, int64_t c_out, int64_t lddy, const float* W, int64_t c_in,
                         const uint16_t* lora_A, const uint16_t* lora_B, int32_t r, float lora_scale, double* dX) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i) {
        double* g = dX + i * c_in;
        for (int64_t k = 0; k < c_in; ++k) {
            double s = 0.0;
            for (int64_t j = 0; j < c_out; ++j) s += (double)bf16_to_f32(dY[i * lddy + j]) * (double)W[k * c_out + j];
            g[k] = s;
        }
        for (int32_t p = 0; p < r; ++p) {
            double s = 0.0;
            for (int64_t j = 0; j < c_out; ++j)
                s += (double)bf16_to_f32(dY[i * lddy + j]) * (double)bf16_to_f32(lora_B[(int64_t)p * c_out + j]);
            for (int64_t k = 0; k < c_in; ++k)
                g[k] += (double)lora_scale * s * (double)bf16_to_f32(lora_A[k * r + p]);
        }
    }
}

/* ------------------------------------------------------------------------
 * LoRA weight gradients of the adapter branch Y_l = lora_scale (X A) B (App.
 * "Model and experimental settings": LoRA on every linear layer; the frozen
 * quantized weight gets no gradient, Sec. 2.1).  Plain calculus on the bf16
 * input values, fp64 throughout:
 *   dA[k,p] = lora_scale * sum_i X[i,k]  * (sum_j dY[i,j] B[p,j])
 *   dB[p,j] = lora_scale * sum_i (sum_k X[i,k] A[k,p]) * dY[i,j]
 * Reading (the paper is silent): the adapter's backward uses the unquantized
 * X and dY, like its forward; no dropout.
 * Out: dA [c_in x r], dB [r x c_out] (fp64; callers round to fp32).
 * ---------------------------------------------------------------------- */
void oracle_lora_grads(const uint16_t* X, const uint16_t* dY, int64_t t, int64_t c_in, int64_t c_out, int64_t ldx,
                       int64_t lddy, const uint16_t* lora_A, const uint16_t* lora_B, int32_t r, float lora_scale,
                       double* dA, double* dB) {
    double* T1 = (double*)malloc(sizeof(double) * (size_t)(t * r + 1)); /* dY B^T */
    double* T2 = (double*)malloc(sizeof(double) * (size_t)(t * r + 1)); /* X A    */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i)
        for (int32_t p = 0; p < r; ++p) {
            double s1 = 0.0, s2 = 0.0;
            for (int64_t j = 0; j < c_out; ++j)
                s1 += (double)bf16_to_f32(dY[i * lddy + j]) * (double)bf16_to_f32(lora_B[(int64_t)p * c_out + j]);
            for (int64_t k = 0; k < c_in; ++k)
                s2 += (double)bf16_to_f32(X[i * ldx + k]) * (double)bf16_to_f32(lora_A[k * r + p]);
            T1[i * r + p] = s1;
            T2[i * r + p] = s2;
        }
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < c_in; ++k)
        for (int32_t p = 0; p < r; ++p) {
            double s = 0.0;
            for (int64_t i = 0; i < t; ++i) s += (double)bf16_to_f32(X[i * ldx + k]) * T1[i * r + p];
            dA[k * r + p] = (double)lora_scale * s;
        }
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < c_out; ++j)
        for (int32_t p = 0; p < r; ++p) {
            double s = 0.0;
            for (int64_t i = 0; i < t; ++i) s += T2[i * r + p] * (double)bf16_to_f32(dY[i * lddy + j]);
            dB[(int64_t)p * c_out + j] = (double)lora_scale * s;
        }
    free(T1);
    free(T2);
}

/* ------------------------------------------------------------------------
 * Input gradient on the outlier channels, three candidate forms (the paper
 * does not describe its backward pass; Sec. 3.3 retains W_O in full precision).
 * For k in O, with T1 = dY B^T and the LoRA term l[i,k] = lora_scale sum_p T1[i,p] A[O_k,p]:
 *   exact[i,k] = sum_j dY[i,j] W_O[k,j] + l[i,k]
 *       (true gradient of X W on these columns: s cancels, Eq. 3)
 *   ste[i,k]   = rinv_k * sum_j dY[i,j] (Wq[O_k,j] delta_w[j] + what_int[k,j] delta_what[j]) + l[i,k]
 *       (gradient of Eq. 9 as evaluated, quantizers treated as identity; rinv_k = colscale[O_k])
 * The third form, the s-free quantized product, is oracle_linear_bwd_dx's output at columns O.
 * Out: exact, ste [t x n] fp64.  Either may be NULL.
 * ---------------------------------------------------------------------- */
void oracle_bwd_dx_outlier_cols(const uint16_t* dY, int64_t t, int64_t c_out, int64_t lddy, const int32_t* O, int32_t n,
                                const float* W_O, const int8_t* Wq, const float* delta_w, const int8_t* what_int,
                                const float* delta_what, const float* colscale, const uint16_t* lora_A,
                                const uint16_t* lora_B, int32_t r, float lora_scale, double* exact, double* ste) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < t; ++i) {
        double* T1 = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        for (int32_t p = 0; p < r; ++p) {
            double s = 0.0;
            for (int64_t j = 0; j < c_out; ++j)
                s += (double)bf16_to_f32(dY[i * lddy + j]) * (double)bf16_to_f32(lora_B[(int64_t)p * c_out + j]);
            T1[p] = s;
        }
        for (int32_t k = 0; k < n; ++k) {
            double l = 0.0;
            for (int32_t p = 0; p < r; ++p) l += T1[p] * (double)bf16_to_f32(lora_A[(int64_t)O[k] * r + p]);
            l *= (double)lora_scale;
            if (exact) {
                double s = 0.0;
                for (int64_t j = 0; j < c_out; ++j)
                    s += (double)bf16_to_f32(dY[i * lddy + j]) * (double)W_O[(int64_t)k * c_out + j];
                exact[i * n + k] = s + l;
            }
            if (ste) {
                double s = 0.0;
                for (int64_t j = 0; j < c_out; ++j) {
                    double w = (double)Wq[(int64_t)O[k] * c_out + j] * (double)delta_w[j] +
                               (double)what_int[(int64_t)k * c_out + j] * (double)delta_what[j];
                    s += (double)bf16_to_f32(dY[i * lddy + j]) * w;
                }
                ste[i * n + k] = (double)colscale[O[k]] * s + l;
            }
        }
        free(T1);
    }
}

/* ------------------------------------------------------------------------
 * Outlier-channel identification on calibration data (Eq. 6, Sec. 3.3):
 *   xi_o = number of calibration samples i with  max_rows |X^i[:, o]| > ratio * mean(|X^i|)
 * X holds the samples one after the other: sample i is rows offsets[i] .. offsets[i+1]-1 of X [.. x c_in].
 * The mean is over all elements of the sample.  Reading: the comparison is strict and is made in fp64 with
 * mean = (fp64 sum of |x|) / count; the paper uses ratio = 100.  An empty sample flags nothing.
 * Out: xi [c_in] (int32).
 * ---------------------------------------------------------------------- */
void oracle_outlier_criterion(const uint16_t* X, int64_t ldx, int64_t c_in, const int64_t* offsets, int32_t n_samples,
                              double ratio, int32_t* xi) {
    for (int64_t o = 0; o < c_in; ++o) xi[o] = 0;
    float* colmax = (float*)malloc(sizeof(float) * (size_t)c_in);
    for (int32_t i = 0; i < n_samples; ++i) {
        const int64_t r0 = offsets[i], r1 = offsets[i + 1];
        if (r1 <= r0) continue;
        double sum = 0.0;
        for (int64_t o = 0; o < c_in; ++o) colmax[o] = 0.0f;
        for (int64_t row = r0; row < r1; ++row)
            for (int64_t o = 0; o < c_in; ++o) {
                float a = fabsf(bf16_to_f32(X[row * ldx + o]));
                sum += (double)a;
                if (a > colmax[o]) colmax[o] = a;
            }
        const double mean = sum / ((double)(r1 - r0) * (double)c_in);
        const double thr = ratio * mean;
        for (int64_t o = 0; o < c_in; ++o)
            if ((double)colmax[o] > thr) xi[o] += 1;
    }
    free(colmax);
}

/* Selection of O from xi (Sec. 3.3: "selecting outlier channels based on xi_o", within a per-layer budget).
 * Reading: the `budget` channels with the largest xi, ties to the lower channel index, channels that were never
 * flagged (xi = 0) excluded; O is returned in ascending channel order.  Returns |O|. */
int32_t oracle_select_outliers(const int32_t* xi, int64_t c_in, int32_t budget, int32_t* O) {
    int32_t n = 0;
    char* taken = (char*)calloc((size_t)c_in, 1);
    for (int32_t pick = 0; pick < budget; ++pick) {
        int64_t best = -1;
        for (int64_t o = 0; o < c_in; ++o)
            if (!taken[o] && xi[o] > 0 && (best < 0 || xi[o] > xi[best])) best = o;
        if (best < 0) break;
        taken[best] = 1;
    }
    for (int64_t o = 0; o < c_in; ++o)
        if (taken[o]) O[n++] = (int32_t)o;
    free(taken);
    return n;
}

/* thread control for the row-parallel loops (rows are independent in every step but the column max) */
#ifdef _OPENMP
#include <omp.h>
void oracle_set_threads(int n) { omp_set_num_threads(n > 0 ? n : 1); }
int oracle_max_threads(void) { return omp_get_max_threads(); }
#else
void oracle_set_threads(int n) { (void)n; }
int oracle_max_threads(void) { return 1; }
#endif
