// Nested-integer depthwise / grouped convolution (groups of 1, 2 or 4 channels, as many outputs as
// inputs per group): the layers of the lightweight CNNs of the paper's evaluation (Sec. 4, lightweight
// models; modes of Sec. 3.3, Eq. 4 / Eq. 8; 8-bit activations Sec. 4.2).
//
// Per output there are only KH*KW*gs multiply-adds, so the layer is a stream: every activation is read
// once from memory, every output written once.  The multiply-adds still go to the matrix cores, because
// at one byte per operand the vector ALU would be the bottleneck (nine multiply-adds plus the
// dequantisation per output byte is more than it sustains at memory speed): v_mfma_i32_16x16x64_i8
// contracts K = 4 filter taps x 16 input channels against a 16 x 64 weight operand that is zero wherever
// input and output channel are in different groups.  That wastes 15/16 of the matrix core and still
// leaves it far from being the limit.
//
// Roles in one matrix-core step: rows = 16 output channels (weights), columns = 16 output pixels
// (activations).  Lane (n = lane & 15, t = lane >> 4) feeds, for pixel n, the 16 bytes of filter tap
// 4*tg + t; the same lane receives, for pixel n, the sums of rows 4*(lane >> 4) .. + 3.  A wave works on
// 64 channels at once: the lane reads the 64 bytes of its (pixel, tap) as four 16-byte pieces V[0..3],
// and step j (0..3) takes dword j of each of them, i.e. input channels 16*q' + 4*j + i.  With the weight
// rows permuted the same way (row 4*q + i of step j is channel 16*q + 4*j + i) a lane ends up with the 16
// consecutive channels 16*(lane >> 4) .. + 15 of its pixel: one 16-byte store of an int8 output.  Groups
// must not straddle a run of 4 channels, hence gs <= 4.
//
// The activations come through LDS: a block is persistent over work units (image, patch of R x CW output
// pixels) of its 64-channel tile; the input window of a unit is fetched with 16-byte loads whose four
// neighbouring lanes cover the 64 contiguous bytes of one pixel (fetching the fragments straight from
// memory, 16 bytes out of a different cache line per lane, runs at a fraction of the cache's rate), held
// in registers while the previous unit is computed, and written to LDS dword by dword, transposed: the
// 64 bytes of a pixel are stored as dword (j, q') at 16*j + 4*q', so that the operand of step j is one
// 16-byte read.  A pixel takes 80 bytes of LDS: with that stride the 16 lanes that read 16 neighbouring
// pixels hit distinct banks.  Pieces outside the image are fetched through the range check of buffer
// loads and arrive as zeros; taps past the filter read a zero slot behind the window.
//
// Everything that does not depend on the data is worked out once: the weight fragments are built by the
// whole block into a table in LDS from which every wave takes its copy, divisions are multiplications by
// host-made reciprocals, and the (image, patch) of a unit advances by a fixed step per iteration.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "nq_codec.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int g_v4i __attribute__((ext_vector_type(4)));

constexpr int GC_NP = 10;        // 16-byte pieces of a window a thread stages (window <= 640 pixels)
constexpr int GC_PIX = 80;       // LDS bytes per window pixel (64 of data)

// NTG: filter taps / 4, rounded up (3: up to 12 taps, 7: up to 28).
template <int H, int L, int FULL, int EPI, int NTG>
__global__ void __launch_bounds__(256, 2) k_nested_conv_grouped(const GemmParams p, const GroupGeom g)
{
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;
    static_assert(EPI != EPI_F32, "a lane owns 16 channels of a pixel: swapped layouts only");

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];     // the window, then 64 zero bytes
    // before the first window: the decoded weights [channel of the tile][k], k < KB*64 <= 128, and the
    // table of weight fragments [tg][j][lane]
    uint8_t *wmat = lds;
    g_v4i *ftab = reinterpret_cast<g_v4i *>(lds + 8192);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ct = blockIdx.y;                       // 64-channel tile
    const int n = lane & 15, t = lane >> 4;
    const int wk = p.KB * 64;

    // ---- window staging plan: piece i = tid + 256*j is 16-byte piece i & 3 of window pixel i >> 2 --------
    const int sq = tid & 3;
    int st_lds[GC_NP], st_rc[GC_NP];
#pragma unroll
    for (int j = 0; j < GC_NP; ++j) {
        const int pi = (tid + 256 * j) >> 2;
        const int r = (int)(((unsigned)pi * (unsigned)g.icp_magic) >> 20), c = pi - r * g.ICp;
        st_lds[j] = pi < g.IRp * g.ICp ? pi * GC_PIX + 4 * sq : -1;
        st_rc[j] = (r << 16) | c;
    }
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0,
                                                                           (int)g.x_bytes, 0x00020000);
    g_v4i stage[GC_NP];
    auto request = [&](int b, int rb, int cb) {
        const int ih0 = rb * g.R * p.stride - p.pad, iw0 = cb * g.CW * p.stride - p.pad;
#pragma unroll
        for (int j = 0; j < GC_NP; ++j) {
            if (j < g.np) {
                const int ih = ih0 + (st_rc[j] >> 16), iw = iw0 + (st_rc[j] & 0xffff);
                const bool ok = st_lds[j] >= 0 && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                // outside the image: an offset past the tensor, which reads as zero
                const int off = ok ? ((b * p.H + ih) * p.W + iw) * p.N + ct * 64 + 16 * sq : 0x7fff0000;
                const auto v = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off, 0, 0);
                stage[j] = g_v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
            }
        }
    };
    // (image, patch row, patch column) of unit u, advanced by the grid's fixed step
    int u = blockIdx.x;
    int b = u / (g.CB * g.RB), rb = (u - b * g.CB * g.RB) / g.CB, cb = u - (b * g.RB + rb) * g.CB;
    auto advance = [&](int &b_, int &rb_, int &cb_) {
        cb_ += g.step_cb;
        if (cb_ >= g.CB) { cb_ -= g.CB; ++rb_; }
        rb_ += g.step_rb;
        if (rb_ >= g.RB) { rb_ -= g.RB; ++b_; }
        b_ += g.step_b;
    };

    // the first window travels while the weights are set up
    if (u < g.units) request(b, rb, cb);

    // ---- weights of the channel tile -> plain byte matrix in LDS ---------------------------------
    for (int idx = wave; idx < 2 * p.KB; idx += 4) {
        const int half = idx / p.KB, kb = idx - half * p.KB;
        const int nb = 2 * ct + half;
        uint32_t D[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) D[j] = 0;
        if (nb < p.NB) {                              // a tile past N does not exist: zero weights
            const int64_t tile = (int64_t)nb * p.KB + kb;
            uint32_t P[H];
#pragma unroll
            for (int i = 0; i < H; ++i) P[i] = p.ph[tile * (H * 64) + lane * H + i];
            HighCodec<H>::decode(P, D);
            if constexpr (FULL != 0) {
                uint32_t Q[LP::ARR];
#pragma unroll
                for (int i = 0; i < LP::DW; ++i) Q[i] = p.pl[tile * (LP::DW * 64) + lane * LP::DW + i];
                LP::apply(Q, D);
            }
        }
        // slot = 32*g + row holds columns 32*g .. 32*g + 31 of the K step, four per dword
        uint8_t *dst = wmat + (half * 32 + (lane & 31)) * wk + kb * 64 + 32 * (lane >> 5);
        *reinterpret_cast<g_v4i *>(dst) = g_v4i{(int)D[0], (int)D[1], (int)D[2], (int)D[3]};
        *reinterpret_cast<g_v4i *>(dst + 16) = g_v4i{(int)D[4], (int)D[5], (int)D[6], (int)D[7]};
    }
    __syncthreads();

    // ---- weight fragments.  Operand row m = lane & 15 of step j is channel 16*(m>>2) + 4*j + (m&3); its 16
    // bytes are tap 4*tg + (lane >> 4) against input channels 16*(ci>>2) + 4*j + (ci&3), ci < 16: non-zero
    // only inside the row's own group, which lies within dword m >> 2.  Entry (tg, j, lane) of the table is
    // that fragment; the block builds the table together --------------------------------------------------
    for (int idx = tid; idx < NTG * 4 * 64; idx += 256) {
        const int ln = idx & 63, j = (idx >> 6) & 3, tg = idx >> 8;
        const int m = ln & 15, tap = 4 * tg + (ln >> 4);
        const int gfirst = (m & 3) & ~(g.gs - 1);     // first channel of the group within its run of 4 (gs: 1, 2, 4)
        const uint8_t *row = wmat + (16 * (m >> 2) + 4 * j + (m & 3)) * wk + tap * g.gs;
        uint32_t d = 0;
        if (tap < g.taps) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e < g.gs) d |= (uint32_t)row[e] << (8 * (gfirst + e));
        }
        const int dq = m >> 2;
        ftab[idx] = g_v4i{dq == 0 ? (int)d : 0, dq == 1 ? (int)d : 0, dq == 2 ? (int)d : 0, dq == 3 ? (int)d : 0};
    }
    __syncthreads();
    // large filters keep the non-zero dword alone and rebuild the fragment with four selects per step
    constexpr bool COMPACT = NTG > 4;
    g_v4i wf[COMPACT ? 1 : NTG][4];
    int wd[COMPACT ? NTG : 1][4];
    const int mq = (lane & 15) >> 2;
#pragma unroll
    for (int tg = 0; tg < NTG; ++tg)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (COMPACT) wd[tg][j] = reinterpret_cast<const int *>(ftab + (tg * 4 + j) * 64 + lane)[mq];
            else wf[tg][j] = ftab[(tg * 4 + j) * 64 + lane];
        }

    // ---- constants of the lane's sixteen output channels --------------------------------------------
    const int nl0 = ct * 64 + 16 * t;
    EpiCols<EPI> e;
    epi_cols16<EPI>(p, nl0, FULL != 0, e);

    // ---- per-lane filter taps as byte offsets inside the window (the same for every tile) -----------------
    int tap_addr[NTG];
#pragma unroll
    for (int tg = 0; tg < NTG; ++tg) {
        const int tap = 4 * tg + t;
        const int kh = (tap * p.kw_magic) >> 16;
        tap_addr[tg] = tap < g.taps ? (kh * g.ICp + (tap - kh * p.KW)) * GC_PIX : -1;
    }

    __syncthreads();                                   // every wave has its weight fragments: the table may go
    if (tid < 4) *reinterpret_cast<g_v4i *>(lds + g.zero_off + 16 * tid) = g_v4i{0, 0, 0, 0};

    for (; u < g.units; u += gridDim.x) {
#pragma unroll
        for (int j = 0; j < GC_NP; ++j)
            if (j < g.np && st_lds[j] >= 0) {
                int *dst = reinterpret_cast<int *>(lds + st_lds[j]);
                dst[0] = stage[j][0];                  // dword k of piece sq -> 16*k + 4*sq of the pixel
                dst[4] = stage[j][1];
                dst[8] = stage[j][2];
                dst[12] = stage[j][3];
            }
        __syncthreads();                               // the window of unit u is complete
        int bn = b, rbn = rb, cbn = cb;
        advance(bn, rbn, cbn);
        if (u + (int)gridDim.x < g.units) request(bn, rbn, cbn);   // travels while this unit is computed

        // Loads return in order: a wait for a residual load inside the loop is also a wait for the window
        // requested above.  Layers without a residual get a loop with no load in it.
        auto tiles = [&](auto with_resid) {
        for (int tile = wave; tile < g.ptiles; tile += 4) {
            // the lane's pixel (the one it reads fragments for and the one it stores)
            const int idx = tile * 16 + n;
            const int idc = idx < g.R * g.CW ? idx : g.R * g.CW - 1;
            const int r = (int)(((unsigned)idc * (unsigned)g.cw_magic) >> 20), c = idc - r * g.CW;
            const int oh = rb * g.R + r, ow = cb * g.CW + c;
            const bool live = idx < g.R * g.CW && oh < p.Ho && ow < p.Wo;
            const int base = (r * g.ICp + c) * (p.stride * GC_PIX);

            e_v4i res = e_v4i{0, 0, 0, 0};
            const int64_t o = (((int64_t)b * p.Ho + oh) * p.Wo + ow) * p.N + nl0;
            if constexpr (EPI == EPI_I8 && decltype(with_resid)::value) {
                if (live && nl0 < p.N) res = *reinterpret_cast<const e_v4i *>(p.resid + o);
            }

            g_v4i acc[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[j] = g_v4i{0, 0, 0, 0};
            // the taps go through the registers in rounds of at most CH groups of four
            constexpr int CH = NTG <= 4 ? NTG : 4;
#pragma unroll
            for (int c0 = 0; c0 < NTG; c0 += CH) {
                g_v4i V[CH][4];
#pragma unroll
                for (int cc = 0; cc < CH; ++cc) {
                    const int tg = c0 + cc;
                    if (tg < NTG) {
                        const uint8_t *src = lds + (tap_addr[tg] >= 0 ? base + tap_addr[tg] : g.zero_off);
#pragma unroll
                        for (int j = 0; j < 4; ++j) V[cc][j] = *reinterpret_cast<const g_v4i *>(src + 16 * j);
                    }
                }
#pragma unroll
                for (int cc = 0; cc < CH; ++cc) {
                    const int tg = c0 + cc;
                    if (tg < NTG) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            g_v4i a;
                            if constexpr (COMPACT) {
                                int d = wd[tg][j];
                                asm volatile("" : "+v"(d));   // rebuilt here, not hoisted into 4 registers per step
                                a = g_v4i{mq == 0 ? d : 0, mq == 1 ? d : 0, mq == 2 ? d : 0, mq == 3 ? d : 0};
                            } else {
                                a = wf[tg][j];
                            }
                            acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, V[cc][j], acc[j], 0, 0, 0);
                        }
                    }
                }
            }

            if (live) {
                e_v16i a16;
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i) a16[4 * j + i] = acc[j][i];
                epi_row16<EPI>(p, a16, SHIFT, e, o, nl0, res);
            }
        }
        };
        if (p.resid) tiles(std::true_type{});
        else tiles(std::false_type{});
        __syncthreads();                               // every wave is done with the window
        b = bn; rb = rbn; cb = cbn;
    }
}

template <int H, int L>
void launch_nested_conv_grouped(bool full, const GemmParams &p, const GroupGeom &g, hipStream_t st, void *ev_start,
                                void *ev_stop)
{
    const dim3 grid((unsigned)g.grid_x, (unsigned)g.CT), block(256);
    const size_t lds = (size_t)g.lds_bytes;
    const int mode = epi_mode(p) == EPI_I8 ? EPI_I8 : EPI_ANY;   // fp32 outputs take the element-wise epilogue
#define NQ_GC_LAUNCH(FULLV, EPIV)                                                                               \
    do {                                                                                                        \
        if (g.taps <= 12)                                                                                       \
            launch_timed(k_nested_conv_grouped<H, L, FULLV, EPIV, 3>, grid, block, lds, st, ev_start, ev_stop, p, g); \
        else                                                                                                    \
            launch_timed(k_nested_conv_grouped<H, L, FULLV, EPIV, 7>, grid, block, lds, st, ev_start, ev_stop, p, g); \
    } while (0)
#define NQ_GC_MODES(FULLV)                                       \
    do {                                                         \
        if (mode == EPI_I8) NQ_GC_LAUNCH(FULLV, EPI_I8);         \
        else NQ_GC_LAUNCH(FULLV, EPI_ANY);                       \
    } while (0)
    if (full && p.low_signed) NQ_GC_MODES(2); else if (full) NQ_GC_MODES(1); else NQ_GC_MODES(0);
}

}  // namespace nq
