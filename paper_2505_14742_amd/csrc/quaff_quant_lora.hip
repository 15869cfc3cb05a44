// Backward-pass launch that runs the per-token quantizer of dY * delta_w and the LoRA down-projection dY B^T side by
// side: both only read dY, neither fills the chip at a few thousand tokens, and each launch on its own costs several
// microseconds of ramp-up and drain.  The first workgroups of the grid take the down-projection (they are the longer
// ones), the rest quantize rows; the two roles share nothing but the launch.
#include "quaff_lora_body.h"
#include "quaff_quant_body.h"

namespace quaff {

template <int R16, int TPR, int NV>
__global__ void __launch_bounds__(64 * kLoraWaves)
quant_lora_kernel(const uint16_t* __restrict__ X, int64_t t, int c, int64_t ldx, const float* __restrict__ cs,
                  int8_t* __restrict__ Xq, float* __restrict__ delta, const uint16_t* __restrict__ L, float scale,
                  uint16_t* __restrict__ T_hi, uint16_t* __restrict__ T_lo, int row_blocks) {
    const int lora_blocks = row_blocks * kLoraParts;
    if ((int)blockIdx.x < lora_blocks)
        lora_down_body<R16, true>(blockIdx.x % row_blocks, blockIdx.x / row_blocks, row_blocks, X, t, c, ldx, L, scale,
                                  T_hi, T_lo, row_blocks, nullptr, nullptr, 0, 0);
    else {
        // The hardware deals consecutive workgroups to the eight XCDs in turn and every XCD has its own L2: the
        // quantizing workgroups of a 16-row block are renumbered so that they land on the XCD whose down-projection
        // workgroups (index = row block, same residue modulo 8) read the same rows at about the same time.
        constexpr int QPG = 16 / ((64 * kLoraWaves) / TPR);   // quantizing workgroups per 16-row block (1 or 4)
        const int local = blockIdx.x - lora_blocks;
        const int xcd = local & 7, m = local >> 3;
        const int rb = (m / QPG) * 8 + xcd;                   // row block
        quant_rows_body<64 * kLoraWaves, TPR, NV>(rb * QPG + m % QPG, X, t, c, ldx, cs, nullptr, 0, 0, Xq, delta,
                                                  nullptr);
    }
}

template <int R16>
static bool launch_r(const uint16_t* X, int64_t t, int c, int64_t ldx, const float* cs, int8_t* Xq, float* delta,
                     const uint16_t* L, float scale, uint16_t* T_hi, uint16_t* T_lo, hipStream_t stream) {
    constexpr int NT = 64 * kLoraWaves;
    const int row_blocks = (int)((t + 15) / 16);
    const int vec = (c + 7) / 8;
#define QUAFF_QL(TPR, NV)                                                                                             \
    hipLaunchKernelGGL((quant_lora_kernel<R16, TPR, NV>),                                                             \
                       dim3((unsigned)(row_blocks * kLoraParts + 8 * ((row_blocks + 7) / 8) * (16 / (NT / TPR)))),   \
                       dim3(NT), 0,                                                                                   \
                       stream, X, t, c, ldx, cs, Xq, delta, L, scale, T_hi, T_lo, row_blocks)
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
