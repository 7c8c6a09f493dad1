// Nested-integer convolution with the input window resident in LDS (paper Sec. 3.3 modes,
// Eq. 4 / Eq. 8; 8-bit activations Sec. 4.2).
//
// A block owns R whole output rows of one image and BN output channels.  It first copies
// the input rows those outputs depend on (with the zero halo written explicitly) into LDS,
// one chunk of CK input channels at a time, every pixel padded by 16 bytes so that 16-byte
// reads of neighbouring pixels spread over all banks.  Every filter tap then reads its
// activation fragments from that window with a different offset, so each input byte is
// fetched from memory once per block instead of once per tap, and the K loop has no
// barrier.  Weights stream from the packed pages straight into registers exactly as in the
// generic kernel (lane = slot of a dense tile) and are decoded there.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int w_v4i __attribute__((ext_vector_type(4)));
typedef int w_v16i __attribute__((ext_vector_type(16)));

template <int H, int L, int FULL, int EPI, int WMG, int WNG, int TM, int TN>
__global__ void __launch_bounds__(256) k_nested_conv_window(const GemmParams p, const WindowGeom g)
{
    static_assert(WMG * WNG == 4, "four waves per block");
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;
    constexpr int BN = WNG * TN * 32;

    extern __shared__ __attribute__((aligned(16))) uint8_t win[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WNG, wn = wave % WNG;
    const int rb = blockIdx.x % g.RB;
    const int64_t b = blockIdx.x / g.RB;
    const int n0 = blockIdx.y * BN;
    const int oh0 = rb * g.R;
    const int rows = min(g.R, p.Ho - oh0);       // output rows this block really has
    const int pix = rows * p.Wo;                 // its output pixels, row major
    const int ih_base = oh0 * p.stride - p.pad;  // input row of window row 0
    const int CKP = g.CK + 16;
    const int c16 = g.CK >> 4;                   // 16-byte chunks per pixel and channel chunk

    // LDS offset of the lane's pixel for each of its row tiles (tap (0,0), channel 0)
    int a_off[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int pl = (wm * TM + i) * 32 + (lane & 31);
        if (pl >= pix) pl = 0;                   // phantom rows read a valid pixel, never stored
        const int r = pl / p.Wo, ow = pl - r * p.Wo;
        a_off[i] = ((r * p.stride) * g.WC + ow * p.stride) * CKP + 32 * (lane >> 5);
    }

    // Packed weights of the next PD K steps live in registers: a load issued PD steps ahead
    // has the latency of the cache hierarchy hidden behind PD steps of matrix-core work.
    constexpr int PD = 4;
    const int nb0 = n0 / 32 + wn * TN;
    const int wslot = epi_weight_slot<EPI>(lane);     // channel order that suits the epilogue
    uint32_t P[PD][TN][H];
    uint32_t Q[PD][TN][LP::ARR];
    auto load_b = [&](uint32_t (&Pd)[TN][H], uint32_t (&Qd)[TN][LP::ARR], int kb) {
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int nb = nb0 + t;
            if (nb < p.NB) {
                const int64_t tile = (int64_t)nb * p.KB + kb;
                const uint32_t *src = p.ph + tile * (H * 64) + wslot * H;
#pragma unroll
                for (int i = 0; i < H; ++i) Pd[t][i] = src[i];
                if constexpr (FULL != 0) {
                    const uint32_t *srcl = p.pl + tile * (LP::DW * 64) + wslot * LP::DW;
#pragma unroll
                    for (int i = 0; i < LP::DW; ++i) Qd[t][i] = srcl[i];
                }
            } else {
#pragma unroll
                for (int i = 0; i < H; ++i) Pd[t][i] = 0;
                if constexpr (FULL != 0) {
#pragma unroll
                    for (int i = 0; i < LP::DW; ++i) Qd[t][i] = 0;
                }
            }
        }
    };

    w_v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int cpk = g.CK >> 6;                   // K steps of 64 per tap and channel chunk
    const int cin64 = p.Cin >> 6;
    const int taps = p.KH * p.KW;
    // K step s of a chunk -> (tap, 64-channel block); weight tile index in the (kh,kw,ci) order
    auto kb_of = [&](int ch, int s) {
        const int tap = s / cpk, cb = s - tap * cpk;
        return tap * cin64 + ch * cpk + cb;
    };

    const int8_t *ximg = p.x + b * (int64_t)p.H * p.W * p.Cin;
    const int row_items = g.WC * c16;            // 16-byte items per window row
    const int items = g.IR * row_items;

    const int steps = taps * cpk;                // K steps per channel chunk
    for (int ch = 0; ch < g.NCH; ++ch) {
        if (ch > 0) __syncthreads();             // everyone is done with the previous chunk
        // weights of the first PD steps go out before the window loads and arrive with them
#pragma unroll
        for (int d = 0; d < PD; ++d)
            if (d < steps) load_b(P[d], Q[d], kb_of(ch, d));
        // ---- stage the window chunk: up to 8 loads in flight per thread ----------------------
        // item q = tid + 256*j is 16-byte piece c of window position pos = ir*WC + wc
        {
            int ir = tid / row_items, rem = tid - ir * row_items;
            for (int q0 = tid; q0 < items; q0 += 256 * 8) {
                uint4 v[8];
                int dst[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    v[u] = make_uint4(0, 0, 0, 0);
                    dst[u] = -1;
                    if (q0 + 256 * u < items) {
                        const int wc = rem >> g.c16_shift, c = rem & (c16 - 1);
                        const int ih = ih_base + ir, iw = wc - p.pad;
                        dst[u] = (ir * g.WC + wc) * CKP + 16 * c;
                        if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                            v[u] = *reinterpret_cast<const uint4 *>(ximg + ((int64_t)ih * p.W + iw) * p.Cin +
                                                                    ch * g.CK + 16 * c);
                    }
                    rem += 256;
                    while (rem >= row_items) { rem -= row_items; ++ir; }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (dst[u] >= 0) *reinterpret_cast<uint4 *>(win + dst[u]) = v[u];
            }
        }
        __syncthreads();

        // ---- all taps of this channel chunk, no barrier --------------------------------------
        for (int s0 = 0; s0 < steps; s0 += PD) {
#pragma unroll
            for (int d = 0; d < PD; ++d) {
                const int s = s0 + d;
                if (s < steps) {
                    w_v4i bfrag[TN][2];
#pragma unroll
                    for (int t = 0; t < TN; ++t) {
                        uint32_t D[8];
                        HighCodec<H>::decode(P[d][t], D);
                        LP::apply(Q[d][t], D);
#pragma unroll
                        for (int hf = 0; hf < 2; ++hf)
                            bfrag[t][hf] =
                                w_v4i{(int)D[4 * hf], (int)D[4 * hf + 1], (int)D[4 * hf + 2], (int)D[4 * hf + 3]};
                    }
                    if (s + PD < steps) load_b(P[d], Q[d], kb_of(ch, s + PD));

                    const int tap = s / cpk, cb = s - tap * cpk;
                    const int kh = tap / p.KW, kw = tap - kh * p.KW;
                    const int tap_off = (kh * g.WC + kw) * CKP + cb * 64;
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                        for (int i = 0; i < TM; ++i) {
                            const w_v4i afrag =
                                *reinterpret_cast<const w_v4i *>(win + a_off[i] + tap_off + 16 * hf);
#pragma unroll
                            for (int t = 0; t < TN; ++t)
                                acc[i][t] = epi_mfma<EPI>(bfrag[t][hf], afrag, acc[i][t]);
                        }
                }
            }
        }
    }

    // ---- epilogue (Eq. 2 / Eq. 8): every load first, one wait (see epi_join), then arithmetic and stores -------
    const int64_t m_base = (b * p.Ho + oh0) * (int64_t)p.Wo;   // whole rows: local pixel -> m is an offset
    auto rows_of = [&](int i) {
        const int left = pix - (wm * TM + i) * 32;
        return left > 32 ? 32 : (left < 0 ? 0 : left);
    };
    e_v4i res[TM * TN];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int i = 0; i < TM; ++i)
            epi_resid_load<EPI>(p, m_base + (wm * TM + i) * 32, rows_of(i), n0 + (wn * TN + t) * 32, lane,
                                res[t * TM + i]);
    // (the sixteen-channel constants of the swapped layouts are too many registers to hold for every column tile:
    // those are fetched per column tile, at the price of one wait for the previous tile's stores)
    constexpr bool COLS_FIRST = EPI == EPI_F32;
    EpiCols<EPI> ecols[COLS_FIRST ? TN : 1];
    if constexpr (COLS_FIRST) {
#pragma unroll
        for (int t = 0; t < TN; ++t) epi_cols<EPI>(p, n0 + (wn * TN + t) * 32, lane, FULL, ecols[t]);
    }
    epi_join();
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int nt0 = n0 + (wn * TN + t) * 32;
        EpiCols<EPI> e;
        if constexpr (COLS_FIRST) e = ecols[t];
        else epi_cols<EPI>(p, nt0, lane, FULL, e);
#pragma unroll
        for (int i = 0; i < TM; ++i)
            epi_tile<EPI>(p, acc[i][t], SHIFT, e, m_base + (wm * TM + i) * 32, rows_of(i), nt0, lane, res[t * TM + i]);
    }
}

template <typename K>
inline void allow_large_lds(K kernel, size_t lds_bytes)
{
    // dynamic LDS above the default limit has to be granted once per kernel
    static size_t granted = 0;
    if (lds_bytes > granted) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds_bytes);
        granted = lds_bytes;
    }
}

template <int H, int L>
void launch_nested_conv_window(bool full, int shape, const GemmParams &p, const WindowGeom &g, size_t lds_bytes,
                               hipStream_t st, void *ev_start, void *ev_stop)
{
    (void)shape;  // one shape so far: 2x2 waves, 8 row tiles x 64 channels
    const int64_t images = p.M / ((int64_t)p.Ho * p.Wo);
    const dim3 grid((unsigned)(images * g.RB), (unsigned)((p.N + 63) / 64)), block(256);
    const int mode = epi_mode(p);
#define NQ_WIN_LAUNCH(FULLV, EPIV)                                              \
    do {                                                                        \
        auto k = k_nested_conv_window<H, L, FULLV, EPIV, 2, 2, 4, 1>;           \
        allow_large_lds(k, lds_bytes);                                          \
        launch_timed(k, grid, block, lds_bytes, st, ev_start, ev_stop, p, g);   \
    } while (0)
#define NQ_WIN_MODES(FULLV)                                      \
    do {                                                         \
        if (mode == EPI_ANY) NQ_WIN_LAUNCH(FULLV, EPI_ANY);      \
        else if (mode == EPI_I8) NQ_WIN_LAUNCH(FULLV, EPI_I8);   \
        else NQ_WIN_LAUNCH(FULLV, EPI_F32);                      \
    } while (0)
    if (full && p.low_signed) NQ_WIN_MODES(2); else if (full) NQ_WIN_MODES(1); else NQ_WIN_MODES(0);
}

}  // namespace nq
