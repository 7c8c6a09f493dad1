// Grouped convolution with groups of any width (the lightweight CNNs of the paper's Sec. 4: the grouped 1x1
// layers of ShuffleNet, whose input and output channel counts differ, and the wider groups of ResNeXt), for the
// shapes the 1 / 2 / 4-channel kernel of nq_conv_grouped.h does not take.  Same two modes as everywhere:
// full-bit w_high * 2^l + w_low recomposed on the fly (Eq. 4), part-bit w_high with the scale s * 2^l (Eq. 8).
//
// Output channel co belongs to group co / (Cout / groups) and sums over the Cin / groups input channels of
// that group; weights are an ordinary nested tensor [Cout][KH*KW*gs_in], k = (kh*KW + kw)*gs_in + ci.
//
// A direct convolution on the vector ALU.  A lane owns one output channel, a wave 64 consecutive channels and
// PIX consecutive output pixels, a block four such pixel runs.  Per 32 values of k the lane decodes the packed
// dwords of its own row of the weight tile (the dense pages give a lane exactly that: slot = row) into eight
// operand dwords and multiplies them, four bytes at a time with the packed dot product, with the input dwords
// of every one of its pixels; the lanes of a group read the same input dwords (one broadcast from the cache), a
// wave a contiguous run of the pixel.  Where a dword of k would straddle two filter taps or start off a dword
// of the input (gs_in or Cin not a multiple of four, unaligned input) the bytes are fetched one by one.  The
// pixel and tap arithmetic is the same for the whole wave and runs on the scalar unit.  The reach of this kernel
// is generality, not speed: about half a vector instruction per multiply-add.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_epilogue.h"
#include "nq_gemm_kernel.h"

namespace nq {

constexpr int GA_PIX = 8;                    // output pixels per wave

// FULL: 0 part-bit, 1 full-bit (unsigned lower part), 2 full-bit (compensated signed lower part).
template <int H, int L, int FULL>
__global__ void __launch_bounds__(256) k_nested_conv_grouped_any(const GemmParams p, int gs_in, int gs_out, int quads)
{
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = blockIdx.y * 64 + lane;                 // the lane's output channel
    const bool n_ok = n < p.N;
    const int nc = n_ok ? n : p.N - 1;                    // lanes past N compute channel N-1 again and store nothing
    const int x_first = (nc / gs_out) * gs_in;            // first input channel of the lane's group
    const int64_t m_first = ((int64_t)blockIdx.x * 4 + wave) * GA_PIX;
    if (m_first >= p.M) return;                           // whole wave

    // the wave's pixels: offset of input pixel (ih0, iw0) and the pair itself, the same for every lane
    int pix_off[GA_PIX], pix_ih0[GA_PIX], pix_iw0[GA_PIX];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int q = 0; q < GA_PIX; ++q) {
        const int64_t m = m_first + q;
        const int mm = m < p.M ? (int)m : 0;
        const int b = mm / HoWo, rem = mm - b * HoWo;
        const int oh = rem / p.Wo, ow = rem - oh * p.Wo;
        const int ih0 = oh * p.stride - p.pad, iw0 = ow * p.stride - p.pad;
        pix_off[q] = ((b * p.H + ih0) * p.W + iw0) * p.Cin;
        pix_ih0[q] = m < p.M ? ih0 : -(1 << 20);          // a pixel past M: no tap ever lands in the image
        pix_iw0[q] = iw0;
    }

    int acc[GA_PIX];
#pragma unroll
    for (int q = 0; q < GA_PIX; ++q) acc[q] = 0;

    const int taps = p.KH * p.KW;
    const int64_t tile_row = (int64_t)(nc >> 5) * p.KB;   // first tile of the lane's row of tiles
    const int r = nc & 31;
    for (int k32 = 0; k32 * 32 < p.K; ++k32) {
        // the lane's 32 weights k32*32 .. +31 of its row: slot 32*g + r of tile (n / 32, k32 / 2), g = k32 & 1
        const int64_t tile = tile_row + (k32 >> 1);
        const int slot = 32 * (k32 & 1) + r;
        uint32_t P[H], Q[LP::ARR], D[8];
#pragma unroll
        for (int i = 0; i < H; ++i) P[i] = p.ph[tile * (H * 64) + slot * H + i];
        if constexpr (FULL != 0) {
#pragma unroll
            for (int i = 0; i < LP::DW; ++i) Q[i] = p.pl[tile * (LP::DW * 64) + slot * LP::DW + i];
        }
        HighCodec<H>::decode(P, D);
        LP::apply(Q, D);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k0 = k32 * 32 + 4 * j;              // the four weights of D[j] are k0 .. k0 + 3
            if (k0 >= p.K) break;                         // (the pages hold zeros there)
            if (quads) {
                // gs_in, Cin and the input pointer are multiples of four: the four k are four consecutive channels of
                // one tap, one aligned dword of the input
                const int tap = k0 / gs_in, ci = k0 - tap * gs_in;
                const int kh = tap / p.KW, kw = tap - kh * p.KW;
                const int toff = (kh * p.W + kw) * p.Cin + ci + x_first;
                // all pixels' dwords are requested before the first is used (a pixel whose tap lies outside the image
                // reads the tensor's first dword of the group instead and contributes zero): eight loads in flight
                // instead of one
                int xv[GA_PIX];
#pragma unroll
                for (int q = 0; q < GA_PIX; ++q) {
                    const int ih = pix_ih0[q] + kh, iw = pix_iw0[q] + kw;
                    const bool in = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                    xv[q] = *reinterpret_cast<const int *>(p.x + (in ? pix_off[q] + toff : x_first));
                    if (!in) xv[q] = 0;
                }
#pragma unroll
                for (int q = 0; q < GA_PIX; ++q) acc[q] = __builtin_amdgcn_sdot4(xv[q], (int)D[j], acc[q], false);
            } else {
#pragma unroll
                for (int bb = 0; bb < 4; ++bb) {
                    const int k = k0 + bb;
                    if (k >= p.K) break;
                    const int tap = k / gs_in, ci = k - tap * gs_in;
                    const int kh = tap / p.KW, kw = tap - kh * p.KW;
                    const int toff = (kh * p.W + kw) * p.Cin + ci + x_first;
                    const int wv = (int)(int8_t)(D[j] >> (8 * bb));
                    int xb[GA_PIX];
#pragma unroll
                    for (int q = 0; q < GA_PIX; ++q) {
                        const int ih = pix_ih0[q] + kh, iw = pix_iw0[q] + kw;
                        const bool in = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                        xb[q] = (int)p.x[in ? pix_off[q] + toff : x_first];
                        if (!in) xb[q] = 0;
                    }
#pragma unroll
                    for (int q = 0; q < GA_PIX; ++q) acc[q] += xb[q] * wv;
                }
            }
        }
    }
    (void)taps;

    // ---- epilogue (Eq. 2 / Eq. 8), element by element: the order of operations of epi_row16's general path ----
    if (!n_ok) return;
    const float lo = p.relu ? 0.0f : -__builtin_inff();
    float c = p.act_scale * p.scale[n];
    if (FULL == 0) c = c * p.part_mul;
    const float bias = p.bias ? p.bias[n] : 0.0f;
#pragma unroll
    for (int q = 0; q < GA_PIX; ++q) {
        const int64_t m = m_first + q;
        if (m >= p.M) break;
        const int64_t o = m * p.N + n;
        const int a = acc[q] >> SHIFT;
        if (p.acc_dump) p.acc_dump[o] = a;
        float y = (float)a * c;
        y = y + bias;
        if (p.resid) {
            const float rv = p.resid_scale * (float)p.resid[o];
            y = y + rv;
        }
        y = fmaxf(y, lo);
        if (p.out_int8)
            reinterpret_cast<int8_t *>(p.y)[o] = (int8_t)(int)epi_quantise(y, p.inv_out_scale);
        else
            reinterpret_cast<float *>(p.y)[o] = y;
    }
}

template <int H, int L>
void launch_nested_conv_grouped_any(bool full, const GemmParams &p, int gs_in, int gs_out, int quads, hipStream_t st,
                                    void *ev_start, void *ev_stop)
{
    const dim3 grid((unsigned)((p.M + 4 * GA_PIX - 1) / (4 * GA_PIX)), (unsigned)((p.N + 63) / 64));
    if (full && p.low_signed)
        launch_timed(k_nested_conv_grouped_any<H, L, 2>, grid, dim3(256), 0, st, ev_start, ev_stop, p, gs_in, gs_out, quads);
    else if (full)
        launch_timed(k_nested_conv_grouped_any<H, L, 1>, grid, dim3(256), 0, st, ev_start, ev_stop, p, gs_in, gs_out, quads);
    else
        launch_timed(k_nested_conv_grouped_any<H, L, 0>, grid, dim3(256), 0, st, ev_start, ev_stop, p, gs_in, gs_out, quads);
}

}  // namespace nq
