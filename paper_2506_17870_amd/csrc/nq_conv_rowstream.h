// Nested-integer convolution for layers with a short reduction (K = KH*KW*Cin of at most
// 9 steps of 64), 32 output channels per block: weights stationary in registers,
// activations streaming through LDS (paper Sec. 3.3 modes, Eq. 4 / Eq. 8; 8-bit
// activations Sec. 4.2).
//
// Such layers (the wide, early layers of a CNN) move far more activation and output bytes
// than weight bytes and run for only a few microseconds, so the kernel is organised around
// the activation stream and around a short prologue.  A block is persistent: it loads and
// decodes the packed weights of its 32 channels ONCE into matrix-core fragments that stay in
// registers, then walks over its share of work units.  A unit is R whole output rows of one
// image (at most 128 pixels, one 32-row tile per wave).  Units are handled in rounds of up to
// rs_round(): the input rows of all units of a round are requested together and copied into RS_G
// LDS windows (pixels padded by 16 bytes against bank conflicts); after one barrier the units
// are computed back to back, each one's output stores overlapping the next one's matrix-core
// work.  The K loop has no barrier and no decoding: 16-byte LDS reads and MFMAs.
//
// Zero padding comes from the hardware range check of buffer loads: the buffer descriptor
// covers exactly one image, rows above or below it fall outside the range and read as zero,
// and halo columns get an offset that is out of range on purpose.  Index arithmetic that does
// not depend on the data (tap offsets, division constants) is done once on the host.  The
// kernel must not spill: a scratch reload would wait for every outstanding store.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int r_v4i __attribute__((ext_vector_type(4)));
typedef int r_v16i __attribute__((ext_vector_type(16)));
typedef unsigned r_v4u __attribute__((ext_vector_type(4)));

constexpr int RS_GMAX = 4;                   // LDS windows a block has room for
// units per round: four, or two where a thread stages eight pieces per unit (registers)
constexpr int rs_round(int ldmax) { return ldmax > 4 ? 2 : 4; }
constexpr int RS_HALO_OFFSET = 0x40000000;   // out of range for any image (host keeps images below 2^29 bytes)

// RS_KCAP: the K steps of 64 of the layer (exact, so the K loop is straight-line code);
// RS_LDMAX: 16-byte window pieces a thread stages per unit.
// RS_CT: 32-channel tiles a block keeps weights for (short reductions leave registers for several:
// the input rows of a unit are then fetched once for all of them).
template <int H, int L, int FULL, int EPI, int RS_KCAP, int RS_LDMAX, int RS_CT>
__global__ void __launch_bounds__(256, 2) k_nested_conv_rowstream(const GemmParams p, const StreamGeom g)
{
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;
    constexpr int WD = H + LP::DW > 8 ? H + LP::DW : 8;   // packed dwords of a K step on arrival (decoded: 8)
    constexpr int RS_G = rs_round(RS_LDMAX);

    extern __shared__ __attribute__((aligned(16))) uint8_t win[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Block id -> (unit slot, 32-channel tile).  Consecutive block ids go to different XCDs (id % 8),
    // each with its own L2.  The blocks that work on the same units for different channel tiles get
    // ids 8 apart: same XCD, dispatched back to back, so the second one finds the input rows in L2.
    const int bid = blockIdx.x, xcd = bid & 7, bj = bid >> 3;
    const int nb0 = (bj % g.nblk) * RS_CT;   // first 32-channel tile of this block (always a real one)
    const int slot = (bj / g.nblk) * 8 + xcd;   // first unit; slots at or past grid_x have no units
    const int CKP = p.Cin + 16;
    const int c16 = p.Cin >> 4;

    // ---- weights: every K step of the channel tile, requested first -----------------------------
    uint32_t W8[RS_CT][RS_KCAP][WD];   // packed dwords on arrival, decoded fragments afterwards
    {
        const int wslot = epi_weight_slot<EPI>(lane);   // channel order that suits the epilogue
#pragma unroll
        for (int c = 0; c < RS_CT; ++c) {
            const int nb = min(nb0 + c, p.NB - 1);      // a tile past N repeats the last one, never stored
            const uint32_t *ph = p.ph + (int64_t)nb * p.KB * (H * 64);
            const uint32_t *pl = FULL ? p.pl + (int64_t)nb * p.KB * (LP::DW * 64) : nullptr;
#pragma unroll
            for (int s = 0; s < RS_KCAP; ++s) {
#pragma unroll
                for (int i = 0; i < H; ++i) W8[c][s][i] = ph[(unsigned)(s * (H * 64) + wslot * H + i)];
                if constexpr (FULL != 0) {
#pragma unroll
                    for (int i = 0; i < LP::DW; ++i)
                        W8[c][s][H + i] = pl[(unsigned)(s * (LP::DW * 64) + wslot * LP::DW + i)];
                }
            }
        }
    }

    // ---- window staging plan of this thread (the same for every unit) --------------------------
    int st_lds[RS_LDMAX], st_goff[RS_LDMAX];
#pragma unroll
    for (int j = 0; j < RS_LDMAX; ++j) {
        const int q = tid + 256 * j;
        const int pos = q >> g.c16_shift, c = q & (c16 - 1);
        const int ir = (int)__umulhi((unsigned)pos, g.wc_magic);   // pos / WC
        const int wc = pos - ir * g.WC;
        const int iw = wc - p.pad;
        const bool in_window = q < g.items;
        const bool in_row = in_window && (unsigned)iw < (unsigned)p.W;
        st_lds[j] = in_window ? pos * CKP + 16 * c : g.win_bytes;   // pieces past the window go to a spare slot
        st_goff[j] = in_row ? (ir * p.W + iw) * p.Cin + 16 * c : RS_HALO_OFFSET;
    }
    r_v4u stage[RS_G][RS_LDMAX];
    auto load_unit = [&](int b, int rb, r_v4u (&stg)[RS_LDMAX]) {
        // the descriptor covers image b only: rows outside it and halo columns read as zero
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int8_t *>(p.x) + (int64_t)b * g.img_bytes, 0, g.img_bytes, 0x00020000);
        const int unit_off = (rb * g.R * p.stride - p.pad) * g.row_bytes;
#pragma unroll
        for (int j = 0; j < RS_LDMAX; ++j)
            stg[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, unit_off + st_goff[j], 0, 0);
    };
    auto store_unit = [&](uint8_t *buf, const r_v4u (&stg)[RS_LDMAX]) {
#pragma unroll
        for (int j = 0; j < RS_LDMAX; ++j) *reinterpret_cast<r_v4u *>(buf + st_lds[j]) = stg[j];
    };

    // units of this block: slot, slot + grid_x, ...; (image, row block) of a unit
    // advance by constants from one unit to the next
    int ub[RS_G], urb[RS_G];
    int nxt_u = slot < g.grid_x ? slot : g.units;
    int nxt_b = nxt_u / g.RB, nxt_rb = nxt_u - nxt_b * g.RB;
    auto request_round = [&]() {
#pragma unroll
        for (int j = 0; j < RS_G; ++j) {
            ub[j] = nxt_b; urb[j] = nxt_rb;
            if (nxt_u < g.units) load_unit(nxt_b, nxt_rb, stage[j]);
            nxt_u += g.grid_x;
            nxt_b += g.step_b; nxt_rb += g.step_rb;
            if (nxt_rb >= g.RB) { nxt_rb -= g.RB; ++nxt_b; }
        }
    };
    int u0 = nxt_u;
    request_round();

    // ---- per-lane constants ---------------------------------------------------------------------
    int a_off;
    {
        int pl = wave * 32 + (lane & 31);
        if (pl >= g.R * p.Wo) pl = 0;                 // phantom rows read a valid pixel, never stored
        const int r = (int)__umulhi((unsigned)pl, g.wo_magic), ow = pl - r * p.Wo;
        a_off = ((r * p.stride) * g.WC + ow * p.stride) * CKP + 32 * (lane >> 5);
    }
    const int rg = lane >> 5;
    // The per-channel constants of the block's tiles wait in LDS behind the windows (64 floats per
    // tile) and are read back for every unit: held in registers for the whole kernel they would push
    // it into scratch.  The first barrier of the unit loop orders the write before the reads.
    float *cols_lds = reinterpret_cast<float *>(win + RS_GMAX * g.win_stride);
    if (wave == 0) {
#pragma unroll
        for (int c = 0; c < RS_CT; ++c) {
            EpiCols<EPI> ec;
            epi_cols<EPI>(p, (nb0 + c) * 32, lane, FULL, ec);
            if constexpr (EPI == EPI_F32) {
                cols_lds[64 * c + (lane & 31)] = ec.c[0];
                cols_lds[64 * c + 32 + (lane & 31)] = ec.bias[0];
            } else if ((lane & 31) == 0) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    cols_lds[64 * c + 32 * rg + r] = ec.c[r];
                    cols_lds[64 * c + 32 * rg + 16 + r] = ec.bias[r];
                }
            }
        }
    }

    // ---- decode the weights in place into matrix-core fragments ---------------------------------
#pragma unroll
    for (int c = 0; c < RS_CT; ++c)
#pragma unroll
        for (int s = 0; s < RS_KCAP; ++s) {
            uint32_t Pk[H], D[8];
#pragma unroll
            for (int i = 0; i < H; ++i) Pk[i] = W8[c][s][i];
            HighCodec<H>::decode(Pk, D);
            if constexpr (FULL != 0) {
                uint32_t Qk[LP::ARR];
#pragma unroll
                for (int i = 0; i < LP::DW; ++i) Qk[i] = W8[c][s][H + i];
                LP::apply(Qk, D);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) W8[c][s][i] = D[i];
        }

    for (; u0 < g.units; u0 += RS_G * g.grid_x) {
        int cur_b[RS_G], cur_rb[RS_G];
#pragma unroll
        for (int j = 0; j < RS_G; ++j) {
            cur_b[j] = ub[j]; cur_rb[j] = urb[j];
            if (u0 + j * g.grid_x < g.units) store_unit(win + j * g.win_stride, stage[j]);
        }
        __syncthreads();
        request_round();                              // the next round travels while this one is computed
#pragma unroll
        for (int j = 0; j < RS_G; ++j) {
            const int u = u0 + j * g.grid_x;
            if (u < g.units) {
                const uint8_t *buf = win + j * g.win_stride;
                // the unit's residual codes travel while its MFMAs run
                const int oh0 = cur_rb[j] * g.R;
                const int pix = min(g.R, p.Ho - oh0) * p.Wo;
                const int64_t m_base = ((int64_t)cur_b[j] * p.Ho + oh0) * p.Wo;
                const int rows = min(max(pix - wave * 32, 0), 32);
#pragma unroll
                for (int c = 0; c < RS_CT; ++c) {
                    const int n0 = (nb0 + c) * 32;
                    if (RS_CT > 1 && n0 >= p.N) continue;         // the block's last tiles may not exist
                    e_v4i res;
                    epi_resid_load<EPI>(p, m_base + wave * 32, rows, n0, lane, res);
                    r_v16i acc;
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[r] = 0;
                    // Activation fragments are read RS_PF reads ahead of the MFMAs that consume them, so
                    // that the LDS latency is covered by matrix-core work; the fences keep that order.
                    constexpr int NFRAG = 2 * RS_KCAP;
                    constexpr int RS_PF = NFRAG < 4 ? NFRAG : 4;
                    r_v4i afrag[RS_PF];
#pragma unroll
                    for (int f = 0; f < RS_PF; ++f)
                        afrag[f] = *reinterpret_cast<const r_v4i *>(buf + a_off + g.tap_off[f >> 1] + 16 * (f & 1));
#pragma unroll
                    for (int f = 0; f < NFRAG; ++f) {
                        const int s = f >> 1, hf = f & 1;
                        const r_v4i a = afrag[f % RS_PF];
                        __builtin_amdgcn_sched_barrier(0);
                        if (f + RS_PF < NFRAG)
                            afrag[f % RS_PF] = *reinterpret_cast<const r_v4i *>(
                                buf + a_off + g.tap_off[(f + RS_PF) >> 1] + 16 * ((f + RS_PF) & 1));
                        const r_v4i bfrag = r_v4i{(int)W8[c][s][4 * hf], (int)W8[c][s][4 * hf + 1],
                                                  (int)W8[c][s][4 * hf + 2], (int)W8[c][s][4 * hf + 3]};
                        acc = epi_mfma<EPI>(bfrag, a, acc);
                        __builtin_amdgcn_sched_barrier(0);
                    }

                    // ---- epilogue (Eq. 2 / Eq. 8) ------------------------------------------------------
                    EpiCols<EPI> eu;
                    if constexpr (EPI == EPI_F32) {
                        eu.c[0] = cols_lds[64 * c + (lane & 31)];
                        eu.bias[0] = cols_lds[64 * c + 32 + (lane & 31)];
                    } else {
                        const e_v4f *cl = reinterpret_cast<const e_v4f *>(cols_lds + 64 * c + 32 * rg);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const e_v4f cc = cl[q], bb = cl[4 + q];
#pragma unroll
                            for (int i = 0; i < 4; ++i) { eu.c[4 * q + i] = cc[i]; eu.bias[4 * q + i] = bb[i]; }
                        }
                    }
                    epi_tile<EPI>(p, acc, SHIFT, eu, m_base + wave * 32, rows, n0, lane, res);
                }
            }
        }
        __syncthreads();   // all windows of the round are free again
    }
}

template <typename K>
inline void rs_grant_lds(K kernel, size_t lds)
{
    static size_t granted = 0;   // one per kernel instantiation
    if (lds > granted) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
        granted = lds;
    }
}

#define NQ_RS_LAUNCH(FULLV, EPIV, KCAP, LDMAX, CTV)                                \
    do {                                                                      \
        auto k = k_nested_conv_rowstream<H, L, FULLV, EPIV, KCAP, LDMAX, CTV>;     \
        rs_grant_lds(k, lds);                                                 \
        launch_timed(k, grid, block, lds, st, ev_start, ev_stop, p, g);       \
    } while (0)

// Instantiated for the K-step counts of 3x3 convolutions with 64 input channels (9) and of 1x1
// convolutions with 64, 128, 256 and 512 input channels (1, 2, 4, 8); the shorter the reduction, the
// more channel tiles a block takes (rs_channel_tiles).
template <int H, int L>
void launch_nested_conv_rowstream(bool full, const GemmParams &p, const StreamGeom &g, int grid_x, hipStream_t st,
                                  void *ev_start, void *ev_stop)
{
    const dim3 grid((unsigned)(((grid_x + 7) / 8) * 8 * g.nblk)), block(256);
    const size_t lds = RS_GMAX * (size_t)g.win_stride + 1024;   // windows + per-channel constants of up to 4 tiles
    const int mode = epi_mode(p);
#define NQ_RS_CASE(FULLV, EPIV)                              \
    switch (g.ksteps) {                                      \
    case 9: NQ_RS_LAUNCH(FULLV, EPIV, 9, 4, 1); break;       \
    case 1: NQ_RS_LAUNCH(FULLV, EPIV, 1, 4, 4); break;       \
    case 2: NQ_RS_LAUNCH(FULLV, EPIV, 2, 8, 4); break;       \
    case 4: NQ_RS_LAUNCH(FULLV, EPIV, 4, 8, 2); break;       \
    case 8: NQ_RS_LAUNCH(FULLV, EPIV, 8, 8, 1); break;       \
    default: break;                                          \
    }
#define NQ_RS_MODES(FULLV)                                            \
    if (mode == EPI_ANY) { NQ_RS_CASE(FULLV, EPI_ANY) }               \
    else if (mode == EPI_I8) { NQ_RS_CASE(FULLV, EPI_I8) }            \
    else { NQ_RS_CASE(FULLV, EPI_F32) }
    if (full && p.low_signed) { NQ_RS_MODES(2) } else if (full) { NQ_RS_MODES(1) } else { NQ_RS_MODES(0) }
}

}  // namespace nq
