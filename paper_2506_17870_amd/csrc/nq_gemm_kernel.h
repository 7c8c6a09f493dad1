// Nested-integer GEMM / implicit-GEMM convolution for gfx950 (paper Sec. 3.3: full-bit
// model = w_high * 2^l + w_low recomposed at run time, Eq. 4; part-bit model = w_high
// alone with the scale s * 2^l, Eq. 8; 8-bit activations, Sec. 4.2).
//
// Work split.  A block of four waves owns a BM x BN tile of the output and walks K in
// steps of 64.  Activations (the A operand) go global -> registers -> LDS (double
// buffered, rows padded to 80 bytes so that 16-byte LDS reads of eight neighbouring rows
// cover all banks) and are read back as 16-byte fragments.  Weights (the B operand) never
// touch LDS: a lane loads the packed dwords of its own slot of a dense tile (the page
// layout is made for this: lane = slot, 256 contiguous bytes per wave load), decodes them
// in registers into the two 16-byte fragments the matrix core wants and reuses them for
// every row tile of the wave.  Which of the two is the matrix core's row operand depends on
// the epilogue layout of the instantiation.  v_mfma_i32_32x32x32_i8 accumulates in int32; because
// integer addition is associative any consistent assignment of k to fragment bytes gives
// the exact sum.  The weight byte fed to the matrix core is w * 2^(8-n) (full-bit) or
// w_high * 2^(8-h) (part-bit, lower field cleared); the accumulator is an exact multiple
// of that power of two and is shifted back before the epilogue.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_epilogue.h"
#include "nq_gemm_params.h"

namespace nq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int A_STRIDE = 80;  // bytes per LDS row of the activation tile (64 + 16 padding)

// FULL: 0 part-bit, 1 full-bit with the unsigned l-bit lower part (concatenation), 2 full-bit with the
// compensated signed (l+1)-bit lower part (shift-add, Sec. 3.3.3).
template <int H, int L, int FULL, int EPI, int BM, int BN, int WM, int WN>
__global__ void __launch_bounds__(256) k_nested_gemm(const GemmParams p)
{
    static_assert(WM * WN == 4, "four waves per block");
    constexpr int S = 8 - H;
    constexpr int TM = BM / WM / 32;   // 32-row tiles per wave
    constexpr int TN = BN / WN / 32;   // 32-column tiles per wave
    constexpr int RPT = BM / 64;       // activation rows a thread stages per K step
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    constexpr int LD = FULL == 2 ? L + 1 : L;   // dwords of the lower-bit page per slot

    __shared__ __attribute__((aligned(16))) uint8_t As[2][BM * A_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;

    // ---- activation staging: thread -> (row, 16-byte chunk) -----------------------------
    const int a_chunk = tid & 3;
    int64_t a_base[RPT];
    int a_ih0[RPT], a_iw0[RPT];
    bool a_ok[RPT];
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int64_t m = m0 + (tid >> 2) + 64 * i;
        a_ok[i] = m < p.M;
        const int64_t mm = a_ok[i] ? m : 0;
        const int64_t b = mm / HoWo;
        const int rem = (int)(mm - b * HoWo);
        const int oh = rem / p.Wo, ow = rem - oh * p.Wo;
        a_ih0[i] = oh * p.stride - p.pad;
        a_iw0[i] = ow * p.stride - p.pad;
        a_base[i] = b * (int64_t)p.H * p.W * p.Cin;
    }
    // position of this thread's chunk inside the (kh, kw, ci) ordering of K
    int k16 = 16 * a_chunk;
    int a_ci, a_kh, a_kw;
    {
        const int tap = k16 / p.Cin;
        a_ci = k16 - tap * p.Cin;
        a_kh = tap / p.KW;
        a_kw = tap - a_kh * p.KW;
    }

    auto load_a = [&](uint4 (&ra)[RPT]) {
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (a_ok[i] && k16 < p.K) {
                if (p.fast_a) {
                    const int ih = a_ih0[i] + a_kh, iw = a_iw0[i] + a_kw;
                    if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                        v = *reinterpret_cast<const uint4 *>(p.x + a_base[i] +
                                                             ((int64_t)ih * p.W + iw) * p.Cin + a_ci);
                } else {
                    uint32_t w[4] = {0, 0, 0, 0};
                    for (int e = 0; e < 16; ++e) {
                        const int k = k16 + e;
                        if (k < p.K) {
                            const int tap = k / p.Cin, ci = k - tap * p.Cin;
                            const int kh = tap / p.KW, kw = tap - kh * p.KW;
                            const int ih = a_ih0[i] + kh, iw = a_iw0[i] + kw;
                            if ((unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W) {
                                const uint32_t byte =
                                    (uint8_t)p.x[a_base[i] + ((int64_t)ih * p.W + iw) * p.Cin + ci];
                                w[e >> 2] |= byte << (8 * (e & 3));
                            }
                        }
                    }
                    v = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            ra[i] = v;
        }
    };
    auto advance_a = [&]() {
        k16 += 64;
        if (p.fast_a) {
            a_ci += 64;
            while (a_ci >= p.Cin) {
                a_ci -= p.Cin;
                if (++a_kw == p.KW) { a_kw = 0; ++a_kh; }
            }
        }
    };

    // ---- weight staging: lane -> slot of a dense tile -------------------------------------
    const int nb0 = n0 / 32 + wn * TN;
    const int wslot = epi_weight_slot<EPI>(lane);             // channel order that suits the epilogue
    uint32_t P[TN][H];
    uint32_t Q[TN][FULL ? LD : 1];
    auto load_b = [&](int kb) {
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int nb = nb0 + t;
            if (nb < p.NB) {
                const int64_t tile = (int64_t)nb * p.KB + kb;
                const uint32_t *src = p.ph + tile * (H * 64) + wslot * H;
#pragma unroll
                for (int i = 0; i < H; ++i) P[t][i] = src[i];
                if constexpr (FULL != 0) {
                    const uint32_t *srcl = p.pl + tile * (LD * 64) + wslot * LD;
#pragma unroll
                    for (int i = 0; i < LD; ++i) Q[t][i] = srcl[i];
                }
            } else {
#pragma unroll
                for (int i = 0; i < H; ++i) P[t][i] = 0;
                if constexpr (FULL != 0) {
#pragma unroll
                    for (int i = 0; i < LD; ++i) Q[t][i] = 0;
                }
            }
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    uint4 ra[RPT];
    load_a(ra);
    load_b(0);

    const int a_write = (tid >> 2) * A_STRIDE + 16 * a_chunk;
    const int a_read = (wm * (BM / WM) + (lane & 31)) * A_STRIDE + 32 * (lane >> 5);

    for (int kb = 0; kb < p.KB; ++kb) {
        uint8_t *as = As[kb & 1];
#pragma unroll
        for (int i = 0; i < RPT; ++i)
            *reinterpret_cast<uint4 *>(as + a_write + 64 * i * A_STRIDE) = ra[i];
        __syncthreads();

        // decode this step's weights into matrix-core fragments
        v4i bfrag[TN][2];
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            uint32_t D[8];
            HighCodec<H>::decode(P[t], D);
            if constexpr (FULL == 1) LowCodec<L, S>::decode_or(Q[t], D);
            if constexpr (FULL == 2) SignedLowCodec<L, S>::decode_add(Q[t], D);
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
                bfrag[t][hf] = v4i{(int)D[4 * hf], (int)D[4 * hf + 1], (int)D[4 * hf + 2], (int)D[4 * hf + 3]};
        }
        // prefetch the next step while the matrix cores run
        if (kb + 1 < p.KB) {
            advance_a();
            load_a(ra);
            load_b(kb + 1);
        }
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const v4i afrag = *reinterpret_cast<const v4i *>(as + a_read + i * 32 * A_STRIDE + 16 * hf);
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    acc[i][t] = epi_mfma<EPI>(bfrag[t][hf], afrag, acc[i][t]);
            }
    }

    // ---- epilogue (Eq. 2 / Eq. 8): every load first, one wait (see epi_join), then arithmetic and stores -------
    const int64_t mw0 = m0 + wm * (BM / WM);
    auto rows_of = [&](int i) {
        const int64_t left = p.M - (mw0 + i * 32);
        return left > 32 ? 32 : (left < 0 ? 0 : (int)left);
    };
    e_v4i res[TM * TN];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int i = 0; i < TM; ++i)
            epi_resid_load<EPI>(p, mw0 + i * 32, rows_of(i), n0 + (wn * TN + t) * 32, lane, res[t * TM + i]);
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
            epi_tile<EPI>(p, acc[i][t], SHIFT, e, mw0 + i * 32, rows_of(i), nt0, lane, res[t * TM + i]);
    }
}

// Launches `kernel`; with events the dispatch itself is time stamped (begin and end of the kernel).
template <typename F, typename... Args>
inline void launch_timed(F kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, void *ev_start, void *ev_stop,
                         Args... args)
{
    if (ev_start || ev_stop)
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, (hipEvent_t)ev_start, (hipEvent_t)ev_stop, 0,
                              args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, args...);
}

#define NQ_LAUNCH_TILE(FULLV, EPIV, BM, BN, WM, WN)                                                       \
    launch_timed(k_nested_gemm<H, L, FULLV, EPIV, BM, BN, WM, WN>,                                        \
                 dim3((unsigned)((p.M + BM - 1) / BM), (unsigned)((p.N + BN - 1) / BN)), dim3(256), 0, st, \
                 ev_start, ev_stop, p)

#define NQ_LAUNCH_TILES(FULLV, EPIV)                                  \
    do {                                                              \
        if (tile == 0) NQ_LAUNCH_TILE(FULLV, EPIV, 256, 64, 4, 1);    \
        else if (tile == 1) NQ_LAUNCH_TILE(FULLV, EPIV, 128, 256, 1, 4); \
        else NQ_LAUNCH_TILE(FULLV, EPIV, 64, 256, 1, 4);              \
    } while (0)

template <int H, int L>
void launch_nested_gemm(bool full, int tile, const GemmParams &p, hipStream_t st, void *ev_start, void *ev_stop)
{
    const int mode = epi_mode(p);
#define NQ_LAUNCH_MODES(FULLV)                                     \
    do {                                                           \
        if (mode == EPI_ANY) NQ_LAUNCH_TILES(FULLV, EPI_ANY);      \
        else if (mode == EPI_I8) NQ_LAUNCH_TILES(FULLV, EPI_I8);   \
        else NQ_LAUNCH_TILES(FULLV, EPI_F32);                      \
    } while (0)
    if (full && p.low_signed) NQ_LAUNCH_MODES(2);
    else if (full) NQ_LAUNCH_MODES(1);
    else NQ_LAUNCH_MODES(0);
}

}  // namespace nq
