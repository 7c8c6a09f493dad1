// Nested-integer convolution for layers with very few input channels (the 7x7, 3-channel stem of
// a CNN; paper Sec. 3.3 modes, Eq. 4 / Eq. 8; 8-bit activations Sec. 4.2).
//
// With Cin = 3 the 16-byte pieces an implicit GEMM is built from would straddle pixels and filter
// taps, and gathering the K dimension byte by byte costs more than the arithmetic.  Instead the
// reduction is re-ordered per filter ROW: the KW*Cin bytes (at most 32) that filter row kh touches
// are contiguous in the NHWC input, so one v_mfma_i32_32x32x32_i8 consumes one filter row: its 32
// k-bytes are those KW*Cin bytes followed by whatever comes next in the input row, against weights
// that are zero past KW*Cin.  Integer sums are associative, so this is the same accumulator.
//
// A block is persistent over work units of R output rows of one image.  The input rows of a unit
// are staged in LDS (dword copies; rows above or below the image read as zero through the range
// check of buffer loads, the left and right halo is zero bytes the kernel writes once).  A lane's
// 16-byte fragment starts at an arbitrary byte of the window: it reads the five aligned dwords
// that cover it and funnel-shifts them.  The weights of the block's channel tiles are decoded once
// into a plain [channel][k] byte matrix in LDS, from which every lane gathers its KH fragments per
// tile; they then stay in registers for the whole kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int s_v4i __attribute__((ext_vector_type(4)));
typedef int s_v16i __attribute__((ext_vector_type(16)));

constexpr int SC_NLD = 8;        // dwords of a window a thread stages (window data <= 8 KiB)
constexpr int SC_CT = 2;         // 32-channel tiles per block

// KHC: filter rows (exact, so the K loop is straight-line code).
template <int H, int L, int FULL, int EPI, int KHC>
__global__ void __launch_bounds__(256, 2) k_nested_conv_smallcin(const GemmParams p, const SmallCinGeom g)
{
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t *win0 = lds;                                   // two windows of g.win_bytes
    uint8_t *wmat = lds + 2 * g.win_bytes;                 // [SC_CT*32][KB*64] decoded weights
    float *cols_lds = reinterpret_cast<float *>(wmat + SC_CT * 32 * p.KB * 64);   // [SC_CT][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nb0 = blockIdx.y * SC_CT;
    const int rg = lane >> 5;

    // ---- zero both windows once: the halo bytes are never written again -------------------------
    for (int q = tid; q < 2 * g.win_bytes / 16; q += 256)
        reinterpret_cast<s_v4i *>(lds)[q] = s_v4i{0, 0, 0, 0};

    // ---- weights -> plain byte matrix in LDS ----------------------------------------------------
    for (int idx = wave; idx < SC_CT * p.KB; idx += 4) {
        const int t = idx / p.KB, kb = idx - t * p.KB;
        const int nb = min(nb0 + t, p.NB - 1);             // tiles past N repeat the last one, never stored
        const int64_t tile = (int64_t)nb * p.KB + kb;
        uint32_t P[H], D[8];
#pragma unroll
        for (int i = 0; i < H; ++i) P[i] = p.ph[tile * (H * 64) + lane * H + i];
        HighCodec<H>::decode(P, D);
        if constexpr (FULL != 0) {
            uint32_t Q[LP::ARR];
#pragma unroll
            for (int i = 0; i < LP::DW; ++i) Q[i] = p.pl[tile * (LP::DW * 64) + lane * LP::DW + i];
            LP::apply(Q, D);
        }
        // slot = 32*g + row holds columns 32*g .. 32*g + 31 of the K step, four per dword
        uint8_t *dst = wmat + (t * 32 + (lane & 31)) * (p.KB * 64) + kb * 64 + 32 * (lane >> 5);
        *reinterpret_cast<s_v4i *>(dst) = s_v4i{(int)D[0], (int)D[1], (int)D[2], (int)D[3]};
        *reinterpret_cast<s_v4i *>(dst + 16) = s_v4i{(int)D[4], (int)D[5], (int)D[6], (int)D[7]};
    }
    // per-channel constants of the block's tiles (read back per tile in the epilogue)
    if (wave < SC_CT) {
        EpiCols<EPI> e0;
        epi_cols<EPI>(p, (nb0 + wave) * 32, lane, FULL, e0);
        if constexpr (EPI == EPI_F32) {
            cols_lds[wave * 64 + (lane & 31)] = e0.c[0];
            cols_lds[wave * 64 + 32 + (lane & 31)] = e0.bias[0];
        } else if ((lane & 31) == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                cols_lds[wave * 64 + 32 * rg + r] = e0.c[r];
                cols_lds[wave * 64 + 32 * rg + 16 + r] = e0.bias[r];
            }
        }
    }
    __syncthreads();

    // ---- gather the lane's weight fragments: filter row kh = bytes [kh*seg, kh*seg + seg) of K ----
    s_v4i wf[SC_CT][KHC];
    {
        const int wrow = epi_weight_slot<EPI>(lane) & 31;
#pragma unroll
        for (int t = 0; t < SC_CT; ++t) {
            const uint8_t *src = wmat + (t * 32 + wrow) * (p.KB * 64);
#pragma unroll
            for (int kh = 0; kh < KHC; ++kh) {
                uint32_t d[4] = {0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int j = 16 * rg + e;
                    const uint32_t b = j < g.seg ? src[kh * g.seg + j] : 0u;
                    d[e >> 2] |= b << (8 * (e & 3));
                }
                wf[t][kh] = s_v4i{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
            }
        }
    }

    // ---- window staging plan: dword q = tid + 256*j of the window's data ------------------------
    int st_lds[SC_NLD], st_goff[SC_NLD];
#pragma unroll
    for (int j = 0; j < SC_NLD; ++j) {
        const int q = tid + 256 * j;
        const int ir = q / g.row_dwords, dw = q - ir * g.row_dwords;
        const bool in = q < g.IR * g.row_dwords;
        st_lds[j] = in ? ir * g.row_stride + g.d0 + 4 * dw : -1;
        st_goff[j] = ir * g.row_bytes + 4 * dw;
    }
    uint32_t stage[SC_NLD];
    auto request = [&](int u) {
        const int b = u / g.RB, rb = u - b * g.RB;
        // the descriptor covers image b only: rows outside it read as zero
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int8_t *>(p.x) + (int64_t)b * g.img_bytes, 0, g.img_bytes, 0x00020000);
        const int unit_off = (rb * g.R * p.stride - p.pad) * g.row_bytes;
#pragma unroll
        for (int j = 0; j < SC_NLD; ++j)
            stage[j] = st_lds[j] >= 0 ? __builtin_amdgcn_raw_buffer_load_b32(rsrc, unit_off + st_goff[j], 0, 0) : 0u;
    };

    // ---- per-lane pixel offsets of the (up to SC_PT) pixel tiles this wave owns in a unit --------
    // pixel tile pt = wave, wave + 4, ...; lane's pixel pl = 32*pt + (lane & 31)
    const int tiles = (g.R * p.Wo + 31) / 32;

    int u = blockIdx.x;
    if (u < g.units) request(u);
    int buf = 0;
    for (; u < g.units; u += gridDim.x, buf ^= 1) {
        uint8_t *win = win0 + buf * g.win_bytes;
#pragma unroll
        for (int j = 0; j < SC_NLD; ++j)
            if (st_lds[j] >= 0) *reinterpret_cast<uint32_t *>(win + st_lds[j]) = stage[j];
        __syncthreads();                                   // window `buf` complete; the other one is free
        const int un = u + gridDim.x;
        if (un < g.units) request(un);                     // travels while this unit is computed

        const int b = u / g.RB, rb = u - b * g.RB;
        const int oh0 = rb * g.R;
        const int pix = min(g.R, p.Ho - oh0) * p.Wo;
        const int64_t m_base = ((int64_t)b * p.Ho + oh0) * p.Wo;
        for (int pt = wave; pt < tiles; pt += 4) {
            int pl = pt * 32 + (lane & 31);
            if (pl >= pix) pl = 0;                         // phantom pixels read a valid one, never stored
            const int r = pl / p.Wo, ow = pl - r * p.Wo;
            // byte address of the lane's 16 bytes of filter row 0
            const int a0 = (r * p.stride) * g.row_stride + g.d0 + (ow * p.stride - p.pad) * p.Cin + 16 * rg;
            const int rows = min(max(pix - pt * 32, 0), 32);
            e_v4i res[SC_CT];
#pragma unroll
            for (int t = 0; t < SC_CT; ++t)
                epi_resid_load<EPI>(p, m_base + pt * 32, rows, (nb0 + t) * 32, lane, res[t]);
            s_v16i acc[SC_CT];
#pragma unroll
            for (int t = 0; t < SC_CT; ++t)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[t][q] = 0;
#pragma unroll
            for (int kh = 0; kh < KHC; ++kh) {
                const int a = a0 + kh * g.row_stride;
                const uint32_t *src = reinterpret_cast<const uint32_t *>(win + (a & ~3));
                const unsigned sh = (unsigned)(a & 3);
                uint32_t q[5];
#pragma unroll
                for (int i = 0; i < 5; ++i) q[i] = src[i];
                s_v4i af;
#pragma unroll
                for (int i = 0; i < 4; ++i) af[i] = (int)__builtin_amdgcn_alignbyte(q[i + 1], q[i], sh);
#pragma unroll
                for (int t = 0; t < SC_CT; ++t) acc[t] = epi_mfma<EPI>(wf[t][kh], af, acc[t]);
            }
#pragma unroll
            for (int t = 0; t < SC_CT; ++t) {
                if ((nb0 + t) * 32 >= p.N) continue;
                EpiCols<EPI> e;
                if constexpr (EPI == EPI_F32) {
                    e.c[0] = cols_lds[t * 64 + (lane & 31)];
                    e.bias[0] = cols_lds[t * 64 + 32 + (lane & 31)];
                } else {
#pragma unroll
                    for (int q2 = 0; q2 < 16; ++q2) {
                        e.c[q2] = cols_lds[t * 64 + 32 * rg + q2];
                        e.bias[q2] = cols_lds[t * 64 + 32 * rg + 16 + q2];
                    }
                }
                epi_tile<EPI>(p, acc[t], SHIFT, e, m_base + pt * 32, rows, (nb0 + t) * 32, lane, res[t]);
            }
        }
    }
}

template <int H, int L>
void launch_nested_conv_smallcin(bool full, const GemmParams &p, const SmallCinGeom &g, hipStream_t st, void *ev_start,
                                 void *ev_stop)
{
    const int ngroups = (p.NB + SC_CT - 1) / SC_CT;
    const dim3 grid((unsigned)g.grid_x, (unsigned)ngroups), block(256);
    const size_t lds = 2 * (size_t)g.win_bytes + (size_t)SC_CT * 32 * p.KB * 64 + SC_CT * 64 * sizeof(float);
    const int mode = epi_mode(p);
#define NQ_SC_LAUNCH(FULLV, EPIV, KHV)                                            \
    do {                                                                          \
        auto k = k_nested_conv_smallcin<H, L, FULLV, EPIV, KHV>;                  \
        static size_t granted = 0;                                                \
        if (lds > granted) {                                                      \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k),          \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            granted = lds;                                                        \
        }                                                                         \
        launch_timed(k, grid, block, lds, st, ev_start, ev_stop, p, g);           \
    } while (0)
#define NQ_SC_KH(FULLV, EPIV)                                    \
    do {                                                         \
        if (p.KH == 7) NQ_SC_LAUNCH(FULLV, EPIV, 7);             \
        else if (p.KH == 3) NQ_SC_LAUNCH(FULLV, EPIV, 3);        \
    } while (0)
#define NQ_SC_MODES(FULLV)                                       \
    do {                                                         \
        if (mode == EPI_ANY) NQ_SC_KH(FULLV, EPI_ANY);           \
        else if (mode == EPI_I8) NQ_SC_KH(FULLV, EPI_I8);        \
        else NQ_SC_KH(FULLV, EPI_F32);                           \
    } while (0)
    if (full && p.low_signed) NQ_SC_MODES(2); else if (full) NQ_SC_MODES(1); else NQ_SC_MODES(0);
}

}  // namespace nq
