// Kernel arguments of the nested GEMM / convolution and the launcher that every
// (h, l) translation unit instantiates.  Internal to libnq.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nq {

struct GemmParams {
    const int8_t *x;
    const uint32_t *ph;
    const uint32_t *pl;
    const float *scale;
    void *y;
    const float *bias;
    const int8_t *resid;
    int32_t *acc_dump;
    int64_t M;
    int N, K, KB, NB;
    // geometry of the implicit GEMM; a plain GEMM is H = W = Ho = Wo = KH = KW = 1, Cin = K
    int H, W, Cin, Ho, Wo, KH, KW, stride, pad;
    float act_scale, resid_scale, inv_out_scale, part_mul;
    int relu, out_int8, fast_a;
};

// Tile shapes: 0 = 256x64 (narrow outputs), 1 = 128x256 (large), 2 = 64x256 (few rows).
constexpr int NQ_TILE_BM[3] = {256, 128, 64};
constexpr int NQ_TILE_BN[3] = {64, 256, 256};

// Defined in nq_gemm_kernel.h, instantiated once per (h, l) by nq_gemm_inst.hip.
template <int H, int L>
void launch_nested_gemm(bool full, int tile, const GemmParams &p, hipStream_t st);

}  // namespace nq
