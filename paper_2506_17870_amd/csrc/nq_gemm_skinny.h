// Nested-integer GEMM for few rows (M <= 64): the regime in which the packed weights are the
// traffic and the part-bit mode pays off in proportion to h / n (paper Sec. 3.3: the part-bit model
// reads the higher-bit page only; Eq. 4 / Eq. 8 for the two modes).
//
// One block per 32-column tile of the weights, so that a layer with N columns spreads over N / 32
// blocks however few rows there are.  The NWS waves of a block (four, or eight where a layer has no
// more blocks than there are compute units: twice the packed bytes in flight per unit) split the
// reduction: wave w takes the K steps w, w + NWS, ..., which together are one contiguous stream of
// the tile's packed dwords.
// Every wave keeps its own accumulators; at the end they are added up through LDS (integer sums, so
// the order does not matter) and wave 0 runs the epilogue.  Activations are small and shared by all
// blocks (they stay in L2): a lane loads its 16-byte fragments straight from memory, rows past M
// through the range check of buffer loads.  Weights and activations are requested SK_PD K steps
// ahead in rolling register pipelines; nothing goes through LDS but the final sums.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int k_v4i __attribute__((ext_vector_type(4)));
typedef int k_v16i __attribute__((ext_vector_type(16)));


// TMS: 32-row tiles (1: M <= 32, 2: M <= 64).  NWS: waves per block (4 or 8).
template <int H, int L, int FULL, int EPI, int TMS, int NWS>
__global__ void __launch_bounds__(64 * NWS, NWS == 4 ? 2 : 1) k_nested_gemm_skinny(const GemmParams p)
{
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;
    // K steps in flight per wave; three where four would not fit the register file
    constexpr int SK_PD = (TMS == 2 && H + LP::DW > 8) ? 3 : 4;

    __shared__ int red[NWS - 1][TMS][16][64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nb = blockIdx.x;
    const int wslot = epi_weight_slot<EPI>(lane);

    // activations: row = lane & 31 (+ 32 per tile), bytes [64*kb + 32*g + 16*hf, +16) of the row
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0,
                                                                           (int)(p.M * p.K), 0x00020000);
    int a_row[TMS];
#pragma unroll
    for (int i = 0; i < TMS; ++i) a_row[i] = (32 * i + (lane & 31)) * p.K + 32 * (lane >> 5);

    uint32_t P[SK_PD][H];
    uint32_t Q[SK_PD][LP::ARR];
    k_v4i A[SK_PD][TMS][2];
    const int64_t tile0 = (int64_t)nb * p.KB;
    // K steps past the end are requested like the last real one (weights) and out of range
    // (activations, which read as zero): straight-line code, exact load counts
    auto request = [&](int slot, int kb) {
        const int kbc = min(kb, p.KB - 1);
        const uint32_t *src = p.ph + (tile0 + kbc) * (H * 64);
#pragma unroll
        for (int i = 0; i < H; ++i) P[slot][i] = src[(unsigned)(i * 64 + wslot)];
        if constexpr (FULL != 0) {
            const uint32_t *srcl = p.pl + (tile0 + kbc) * (LP::DW * 64);
#pragma unroll
            for (int i = 0; i < LP::DW; ++i) Q[slot][i] = srcl[(unsigned)(i * 64 + wslot)];
        }
        const int koff = kb < p.KB ? 64 * kb : 0x7fff0000;
#pragma unroll
        for (int i = 0; i < TMS; ++i)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const auto v = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, a_row[i] + koff + 16 * hf, 0, 0);
                A[slot][i][hf] = k_v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
            }
    };

    k_v16i acc[TMS];
#pragma unroll
    for (int i = 0; i < TMS; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;

#pragma unroll
    for (int d = 0; d < SK_PD; ++d) request(d, wave + NWS * d);

    // wave w: K steps w + NWS*j; all waves run the same number of rounds (the extra ones add zeros)
    const int rounds = (p.KB + NWS - 1) / NWS;
    for (int j0 = 0; j0 < rounds; j0 += SK_PD) {
#pragma unroll
        for (int d = 0; d < SK_PD; ++d) {
            uint32_t D[8];
            HighCodec<H>::decode(P[d], D);
            LP::apply(Q[d], D);
            k_v4i a[TMS][2];
#pragma unroll
            for (int i = 0; i < TMS; ++i)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) a[i][hf] = A[d][i][hf];
            request(d, wave + NWS * (j0 + d + SK_PD));
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const k_v4i b = k_v4i{(int)D[4 * hf], (int)D[4 * hf + 1], (int)D[4 * hf + 2], (int)D[4 * hf + 3]};
#pragma unroll
                for (int i = 0; i < TMS; ++i) acc[i] = epi_mfma<EPI>(b, a[i][hf], acc[i]);
            }
        }
    }

    // ---- add the partial sums of the waves ---------------------------------------------------------------
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < TMS; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) red[wave - 1][i][r][lane] = acc[i][r];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < NWS - 1; ++w)
#pragma unroll
        for (int i = 0; i < TMS; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] += red[w][i][r][lane];

    // ---- epilogue (Eq. 2 / Eq. 8) ----------------------------------------------------------------
    EpiCols<EPI> e;
    epi_cols<EPI>(p, nb * 32, lane, FULL, e);
#pragma unroll
    for (int i = 0; i < TMS; ++i) {
        const int64_t left = p.M - 32 * i;
        const int rows = left > 32 ? 32 : (left < 0 ? 0 : (int)left);
        e_v4i res;
        epi_resid_load<EPI>(p, 32 * i, rows, nb * 32, lane, res);
        epi_tile<EPI>(p, acc[i], SHIFT, e, 32 * i, rows, nb * 32, lane, res);
    }
}

template <int H, int L>
void launch_nested_gemm_skinny(bool full, const GemmParams &p, hipStream_t st, void *ev_start, void *ev_stop)
{
    const dim3 grid((unsigned)p.NB);
    const int mode = epi_mode(p);
    // eight waves where every compute unit gets at most one block, the reduction is long enough to share and
    // there is one row tile (with two, measured slower: 25.8 us against 23.1 us at 64 x 8192 -> 8192)
    const bool wide = p.NB <= 256 && p.KB >= 32 && p.M <= 32;
#define NQ_SK_LAUNCH(FULLV, EPIV)                                                                                 \
    do {                                                                                                          \
        if (wide)                                                                                                 \
            launch_timed(k_nested_gemm_skinny<H, L, FULLV, EPIV, 1, 8>, grid, dim3(512), 0, st, ev_start, ev_stop, p); \
        else if (p.M <= 32)                                                                                       \
            launch_timed(k_nested_gemm_skinny<H, L, FULLV, EPIV, 1, 4>, grid, dim3(256), 0, st, ev_start, ev_stop, p); \
        else                                                                                                      \
            launch_timed(k_nested_gemm_skinny<H, L, FULLV, EPIV, 2, 4>, grid, dim3(256), 0, st, ev_start, ev_stop, p); \
    } while (0)
#define NQ_SK_MODES(FULLV)                                       \
    do {                                                         \
        if (mode == EPI_ANY) NQ_SK_LAUNCH(FULLV, EPI_ANY);       \
        else if (mode == EPI_I8) NQ_SK_LAUNCH(FULLV, EPI_I8);    \
        else NQ_SK_LAUNCH(FULLV, EPI_F32);                       \
    } while (0)
    if (full && p.low_signed) NQ_SK_MODES(2); else if (full) NQ_SK_MODES(1); else NQ_SK_MODES(0);
}

}  // namespace nq
