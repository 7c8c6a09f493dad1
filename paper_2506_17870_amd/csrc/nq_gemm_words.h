// Nested-integer GEMM that reads the paper's own pages (Sec. 3.3.4: 64 / k fields of k bits per unsigned
// 64-bit word, every row starting a new word), so that a model stored exactly as the paper packs it runs
// without being repacked: full-bit w_high * 2^l + w_low (Eq. 4) or part-bit w_high with s * 2^l (Eq. 8).
//
// The two pages cut a row into words of different lengths (12 five-bit fields against 21 three-bit ones), so
// the parts are not recomposed element by element.  The sum over k is split instead:
//     sum_k x[k] * (high[k] * 2^l + low[k])  =  2^l * sum_k x[k] * high[k]  +  sum_k x[k] * low[k],
// one pass of the matrix core over each page, each with its own order of k, joined in int32 at the end (exact:
// integers).  Within a page a matrix-core step takes sixteen operand slots per half-wave; a lane fills them
// with the fields of one word (k >= 4: one word per half-wave, slots past the 64 / k fields are zero) or with
// one sixteen-field group of a word (k <= 3).  The activations of a step are the sixteen bytes of the lane's
// row that start at the first field's k, whatever its alignment; what they hold past the word's last field
// meets a zero weight.  Signed fields are decoded to the top of their byte (value * 2^(8-k), no sign extension
// needed) and the page's sum is shifted back, unsigned ones to the bottom.
//
// One block per 32 rows x 32 columns; its four or eight waves split the steps of a page (wave w takes steps w,
// w + NW, ...) and keep eight of them requested ahead; the partial sums meet in LDS and wave 0 runs the
// epilogue.  Like the kernel for few rows it is made for the regime in which the packed weights are the
// traffic; it takes any M, reading the pages once per 32 rows.  What bounds it is the vector ALU: about two
// instructions per field to move it, four per weight with everything else of a step.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_epilogue.h"
#include "nq_gemm_kernel.h"

namespace nq {

// Fields of one word of k = KB bits, as bytes of the matrix core's operand.
template <int KB, bool SGN>
struct WordFields {
    static constexpr int F = 64 / KB;               // fields per word
    static constexpr int G = (F + 15) / 16;         // groups of sixteen fields per word: 1, 2 or 4
    static constexpr int NF = F < 16 ? F : 16;      // fields of a group
    static constexpr int UP = SGN ? 8 - KB : 0;     // a byte holds field << UP
    static constexpr int SPW = G > 1 ? G / 2 : 1;   // matrix-core steps per word when both half-waves share it

    // (lo, hi): the word, shifted down so that the group's first field is at bit 0, nothing but fields above
    __device__ __forceinline__ static e_v4i bytes(uint32_t lo, uint32_t hi)
    {
        uint32_t D[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            const int b = j * KB;                   // where the field is
            const int tb = 8 * (j & 3) + UP;        // where it goes
            const uint32_t mask = ((1u << KB) - 1u) << tb;
            uint32_t src;
            int sb;
            if (b + KB <= 32) { src = lo; sb = b; }
            else if (b >= 32) { src = hi; sb = b - 32; }
            else { src = __builtin_amdgcn_alignbit(hi, lo, b); sb = 0; }
            const uint32_t moved = sb >= tb ? src >> (sb - tb) : src << (tb - sb);
            D[j >> 2] |= moved & mask;
        }
        return e_v4i{(int)D[0], (int)D[1], (int)D[2], (int)D[3]};
    }

    // Operand bytes of group `group` of the word (lo, hi).
    __device__ __forceinline__ static e_v4i decode(uint32_t lo, uint32_t hi, int group)
    {
        if constexpr (G > 1) {
            if constexpr (F * KB < 64) hi &= (1u << (F * KB - 32)) - 1u;     // spare top bits are no field
            const uint64_t v = (((uint64_t)hi << 32) | lo) >> (16 * KB * group);
            return bytes((uint32_t)v, (uint32_t)(v >> 32));
        } else {
            return bytes(lo, hi);
        }
    }
};

// Geometry of the activation chunks in LDS for pages of KB-bit fields and NW waves per block.  A chunk is what
// 8 * NW consecutive steps of a page read: 8 steps per wave.
template <int KB, int NW>
struct WordChunk {
    static constexpr int F = 64 / KB, G = (F + 15) / 16, SPW = G > 1 ? G / 2 : 1;
    // Step t of the page (wave w takes t = w, w + NW, ...).  Byte offsets of its word and of the first
    // activation of its sixteen slots are linear in t:
    //   one word per half-wave (k >= 4):   word 2t + g,  k = (2t + g) * F
    //   one word per step (k = 2, 3):      word t,       k = t * F + 16 g          (group g)
    //   two steps per word (k = 1):        word t >> 1,  k = 32 t + 16 g           (group 2 (t & 1) + g)
    static constexpr int WSTEP = G == 1 ? 16 : 8 / SPW;
    static constexpr int XSTEP = G == 1 ? 2 * F : F / SPW;
    static constexpr int SC = 8 * NW;                    // steps of a chunk
    static constexpr int SPAN = XSTEP * SC;              // activation bytes a chunk advances by
    // bytes of a row in LDS: the span, the last step's reach past it (less than a step, plus up to 3 bytes
    // of alignment and 20 bytes read), in 16-byte pieces, an odd number of them (rows fall on different banks)
    static constexpr int PPR = ((SPAN + 32 + 15) / 16) | 1;
    static constexpr int RS = 16 * PPR;
    static constexpr int BUF = 32 * RS + 16;             // one buffer; the last 16 bytes take pieces of no row
    static constexpr int NPT = (32 * PPR + 64 * NW - 1) / (64 * NW);   // pieces a thread stages per chunk
};

// LDS bytes of the kernel: two chunk buffers of the page with the longest rows, or the partial sums.
template <int HB, int LB, int NW>
constexpr int words_lds_bytes()
{
    int b = 2 * WordChunk<HB, NW>::BUF;
    if (LB > 0 && 2 * WordChunk<(LB > 0 ? LB : 1), NW>::BUF > b) b = 2 * WordChunk<(LB > 0 ? LB : 1), NW>::BUF;
    return b > (NW - 1) * 4096 ? b : (NW - 1) * 4096;
}

// Barrier of the block that orders LDS accesses only (a __syncthreads would also wait for every global load in
// flight).
__device__ __forceinline__ void words_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// acc += X[32 rows] * page[32 columns]^T over the whole row of one page.  wrs: the 32 weight rows of the block
// (rows past N are out of its range and read as zero), row_off: byte offset of the lane's row in it, W: words
// per row.  xrs: the activations; x_row0: byte offset of the block's first row, x_rows: how many of its 32 rows
// exist.  lds: two chunk buffers.  The result holds the fields times 2^UP.
//
// Activations go through LDS.  Fetched straight from memory, the sixteen bytes of a step are one cache line per
// lane for nine to sixteen weights.  Instead the block copies, chunk by chunk, a run of every row into LDS with
// whole-line loads (each row from the dword its run starts in, so every load is dword aligned whatever K is),
// and a step reads four or five dwords of its row there and shifts the sixteen bytes into place.  Bytes past
// the end of a row belong to the next row (or read as zero past the last one) and meet zero weights: the
// row's last word is zero padded.  The words themselves stream from memory, eight steps ahead per wave, across
// the chunks.
// FIFTH: the sixteen bytes may start inside a dword and reach into a fifth one.
// CONV: the rows are the output pixels of a convolution and k runs over (kh, kw, ci) of the NHWC input (Sec. 4.1's
// CNN layers from the paper's own pages): a row is not contiguous in memory, so the staging gathers it, dword by
// dword when the number of input channels is a multiple of four (a dword then lies inside one filter tap), else
// byte by byte; taps outside the image and k >= K are requested out of range and read as zero.  Every row then
// starts at k = 0 of its own (no alignment to inherit from memory): x_row0 is not used, cv is the geometry.
template <int KB, bool SGN, bool FIFTH, int NW, bool CONV>
__device__ __forceinline__ void words_page_steps(const __amdgpu_buffer_rsrc_t wrs, int row_off, int W,
                                                 const __amdgpu_buffer_rsrc_t xrs, uint32_t x_row0, int x_rows, int K,
                                                 uint8_t *lds, int tid, int wave, int g, e_v16i &acc,
                                                 const GemmParams &cv, int64_t m0)
{
    using WF = WordFields<KB, SGN>;
    using WC = WordChunk<KB, NW>;
    constexpr int F = WF::F, G = WF::G, SPW = WF::SPW;
    constexpr int WSTEP = WC::WSTEP, XSTEP = WC::XSTEP, RS = WC::RS, PPR = WC::PPR, NPT = WC::NPT;
    constexpr uint32_t NOWHERE = 0x7fff0000u;     // past every buffer: reads as zero
    const int lane = tid & 63;
    const int T = G == 1 ? (W + 1) / 2 : W * SPW;      // steps of the page
    const int chunks = (T + WC::SC - 1) / WC::SC;      // steps past T read zero words
    const int group = G == 1 ? 0 : 2 * (wave % SPW) + g;
    const uint32_t w_end = (uint32_t)(row_off + 8 * W);
    uint32_t w_at = (uint32_t)(row_off + WSTEP * wave + (G == 1 ? 8 * g : -(8 / SPW) * (wave % SPW)));

    // ---- staging plan of this thread: piece q of the chunk is piece q % PPR of row q / PPR ----------------
    uint32_t st_x[NPT];     // byte offset of the piece's row in the activations (NOWHERE past M)
    int st_lds[NPT];        // where the piece goes in a buffer
    int st_base[CONV ? NPT : 1], st_hw[CONV ? NPT : 1];   // CONV: offset of tap (0,0) of the row's pixel, (ih0 << 16) | (iw0 & 0xffff)
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        const int q = tid + 64 * NW * i;
        const int r = q / PPR, pi = q - r * PPR;
        const bool real = r < 32;
        st_x[i] = real && r < x_rows ? x_row0 + (uint32_t)(r * K) : NOWHERE;
        st_lds[i] = real ? r * RS + 16 * pi : 32 * RS;
        if constexpr (CONV) {
            const int64_t m = m0 + r;
            const bool row_ok = real && r < x_rows;
            const int HoWo = cv.Ho * cv.Wo;
            const int mm = row_ok ? (int)m : 0;
            const int b = mm / HoWo, rem = mm - b * HoWo;
            const int oh = rem / cv.Wo, ow = rem - oh * cv.Wo;
            const int ih0 = oh * cv.stride - cv.pad, iw0 = ow * cv.stride - cv.pad;
            st_base[i] = ((b * cv.H + ih0) * cv.W + iw0) * cv.Cin;
            // a row that does not exist gets a pixel row that no tap brings into the image
            st_hw[i] = (row_ok ? ih0 : -16384) * 65536 + (iw0 & 0xffff);
        }
    }
    e_v4i stage[NPT];
    auto stage_load = [&](int c) {
        const uint32_t k_lo = (uint32_t)(c * WC::SPAN);
#pragma unroll
        for (int i = 0; i < NPT; ++i) {
            const int q = tid + 64 * NW * i;
            const int pi = q % PPR;
            if constexpr (!CONV) {
                // the row's run starts in the dword that holds its byte k_lo
                const uint32_t at = st_x[i] == NOWHERE ? NOWHERE : ((st_x[i] + k_lo) & ~3u) + (uint32_t)(16 * pi);
                const auto v = __builtin_amdgcn_raw_buffer_load_b128(xrs, at, 0, 0);
                stage[i] = e_v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
            } else {
                // the sixteen bytes k0 .. k0 + 15 of the pixel's row of the implicit GEMM
                const int k0 = (int)(k_lo & ~3u) + 16 * pi;
                const int ih0 = st_hw[i] >> 16, iw0 = (int)(int16_t)(st_hw[i] & 0xffff);
                const int kwc = cv.KW * cv.Cin;
                int kh = k0 / kwc;
                const int rem = k0 - kh * kwc;
                int kw = rem / cv.Cin;
                int ci = rem - kw * cv.Cin;
                auto where = [&](int k) -> uint32_t {
                    const bool in = k < K && (unsigned)(ih0 + kh) < (unsigned)cv.H && (unsigned)(iw0 + kw) < (unsigned)cv.W;
                    return in ? (uint32_t)(st_base[i] + (kh * cv.W + kw) * cv.Cin + ci) : NOWHERE;
                };
                auto advance = [&](int by) {
                    ci += by;
                    if (ci >= cv.Cin) {
                        ci -= cv.Cin;
                        if (++kw == cv.KW) { kw = 0; ++kh; }
                    }
                };
                uint32_t d[4];
                if ((cv.Cin & 3) == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        d[j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xrs, where(k0 + 4 * j), 0, 0);
                        advance(4);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        d[j] = 0u;
#pragma unroll
                        for (int bb = 0; bb < 4; ++bb) {
                            const uint32_t v = (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(xrs, where(k0 + 4 * j + bb), 0, 0) & 0xffu;
                            d[j] |= v << (8 * bb);
                            advance(1);
                        }
                    }
                }
                stage[i] = e_v4i{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
            }
        }
    };
    // the lane's own row: where its bytes are in a buffer
    const int xr = lane & 31;
    const uint32_t x_mine = CONV ? 0u : (xr < x_rows ? x_row0 + (uint32_t)(xr * K) : 0u);
    uint32_t x_use = x_mine + (uint32_t)(XSTEP * wave + (G == 1 ? F * g : 16 * g));   // first byte of the next step

    uint2 Wd[8];
    auto request = [&](int slot) {
        const auto wv = __builtin_amdgcn_raw_buffer_load_b64(wrs, w_at < w_end ? w_at : NOWHERE, 0, 0);
        Wd[slot] = uint2{(uint32_t)wv[0], (uint32_t)wv[1]};
        w_at += (uint32_t)(WSTEP * NW);
    };

    stage_load(0);
#pragma unroll
    for (int d = 0; d < 8; ++d) {
        request(d);
        __builtin_amdgcn_sched_barrier(0);     // oldest first, as the loop expects them to arrive
    }
    for (int c = 0; c < chunks; ++c) {
        uint8_t *buf = lds + (c & 1) * WC::BUF;
        // The buffer was last read two chunks ago, and every wave has passed the barrier of the chunk in
        // between since: one barrier per chunk is enough.
#pragma unroll
        for (int i = 0; i < NPT; ++i) *reinterpret_cast<e_v4i *>(buf + st_lds[i]) = stage[i];
        if (c + 1 < chunks) stage_load(c + 1);         // travels while this chunk is computed
        words_lds_barrier();
        const uint8_t *mine = buf + xr * RS;
        const uint32_t run0 = (x_mine + (uint32_t)(c * WC::SPAN)) & ~3u;      // first byte of the row's run
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            const uint32_t pos = x_use - run0;
            x_use += (uint32_t)(XSTEP * NW);
            const uint32_t sh = pos & 3u;
            const uint32_t *src = reinterpret_cast<const uint32_t *>(mine + (pos & ~3u));
            const uint32_t x0 = src[0], x1 = src[1], x2 = src[2], x3 = src[3];
            const uint32_t x4 = FIFTH ? src[4] : 0u;
            const e_v4i a = e_v4i{(int)__builtin_amdgcn_alignbyte(x1, x0, sh), (int)__builtin_amdgcn_alignbyte(x2, x1, sh),
                                  (int)__builtin_amdgcn_alignbyte(x3, x2, sh), (int)__builtin_amdgcn_alignbyte(x4, x3, sh)};
            const e_v4i b = WF::decode(Wd[d].x, Wd[d].y, group);
            // the slot's registers are free again: the new request lands in them
            __builtin_amdgcn_sched_barrier(0);
            request(d);
            acc = epi_mfma<EPI_ANY>(b, a, acc);
            // keeps the steps in this order: request, wait for the oldest, compute
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    words_lds_barrier();      // the buffers are free for the next page or for the partial sums
}

template <int KB, bool SGN, int NW, bool CONV>
__device__ __forceinline__ void words_page(const __amdgpu_buffer_rsrc_t wrs, int row_off, int W,
                                           const __amdgpu_buffer_rsrc_t xrs, uint32_t x_row0, int x_rows, int K,
                                           uint8_t *lds, int tid, int wave, int g, e_v16i &acc, const GemmParams &cv,
                                           int64_t m0)
{
    using WF = WordFields<KB, SGN>;
    // No fifth dword where a step has at most thirteen fields (up to three bytes are lost to the alignment),
    // nor where every step starts on a multiple of sixteen bytes of a row and the rows start on dwords.
    constexpr bool on16 = KB == 1 || KB == 2 || KB == 4;
    if constexpr (WF::NF <= 13) {
        words_page_steps<KB, SGN, false, NW, CONV>(wrs, row_off, W, xrs, x_row0, x_rows, K, lds, tid, wave, g, acc, cv, m0);
    } else {
        // (the gathered rows of a convolution all start at k = 0 of a buffer row)
        if (on16 && (CONV || (K & 3) == 0))
            words_page_steps<KB, SGN, false, NW, CONV>(wrs, row_off, W, xrs, x_row0, x_rows, K, lds, tid, wave, g, acc, cv, m0);
        else
            words_page_steps<KB, SGN, true, NW, CONV>(wrs, row_off, W, xrs, x_row0, x_rows, K, lds, tid, wave, g, acc, cv, m0);
    }
}

// HB: bits of the higher-bit fields.  MODE 0: part-bit; 1: unsigned lower-bit fields of LB = l bits; 2: signed
// lower-bit fields of LB = l + 1 bits (compensated format, Sec. 3.3.3).  WH, WL: words per row of the pages.
// NW: waves per block (4, or 8 where a layer has few blocks).
template <int HB, int LB, int MODE, int NW, bool CONV>
__global__ void __launch_bounds__(64 * NW) k_nested_gemm_words(const GemmParams p, int WH, int WL)
{
    constexpr int EPI = EPI_ANY;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // chunk buffers, then the partial sums

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5;
    const int nb = blockIdx.x;
    const int64_t m0 = (int64_t)blockIdx.y * 32;

    // the block's 32 weight rows of either page and the activations as range-checked buffers: rows past N or
    // M read as zero (and are not stored)
    const int cols = p.N - nb * 32 < 32 ? p.N - nb * 32 : 32;
    const int cn = epi_weight_slot<EPI>(lane) & 31;
    // The range ends with the dword that holds the last activation (the host checks that they start on one):
    // what that dword holds behind it stands at k >= K of the last row and meets zero weights.
    // CONV: the whole input tensor (the host keeps it below 2 GiB)
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(p.x), 0,
        CONV ? (int)(((p.M / ((int64_t)p.Ho * p.Wo)) * p.H * p.W * p.Cin + 3) & ~int64_t(3)) : (int)((p.M * p.K + 3) & ~int64_t(3)),
        0x00020000);
    const uint32_t x_row0 = (uint32_t)(m0 * p.K);
    const int x_rows = p.M - m0 < 32 ? (int)(p.M - m0) : 32;

    e_v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
    {
        const uint2 *rows_h = reinterpret_cast<const uint2 *>(p.ph) + (int64_t)nb * 32 * WH;
        const __amdgpu_buffer_rsrc_t wrs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint2 *>(rows_h), 0, cols * WH * 8, 0x00020000);
        words_page<HB, true, NW, CONV>(wrs, cn * WH * 8, WH, xrs, x_row0, x_rows, p.K, lds, tid, wave, g, acc, p, m0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] >>= 8 - HB;
    if constexpr (MODE != 0) {
        constexpr int L = MODE == 2 ? LB - 1 : LB;
        e_v16i acl;
#pragma unroll
        for (int r = 0; r < 16; ++r) acl[r] = 0;
        const uint2 *rows_l = reinterpret_cast<const uint2 *>(p.pl) + (int64_t)nb * 32 * WL;
        const __amdgpu_buffer_rsrc_t wrs =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint2 *>(rows_l), 0, cols * WL * 8, 0x00020000);
        words_page<LB, MODE == 2, NW, CONV>(wrs, cn * WL * 8, WL, xrs, x_row0, x_rows, p.K, lds, tid, wave, g, acl, p, m0);
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = acc[r] * (1 << L) + (acl[r] >> (MODE == 2 ? 8 - LB : 0));
    }

    // ---- add the partial sums of the waves ----------------------------------------------------------
    int *red = reinterpret_cast<int *>(lds);          // [NW - 1][16][64]
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) red[((wave - 1) * 16 + r) * 64 + lane] = acc[r];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += red[(w * 16 + r) * 64 + lane];

    // ---- epilogue (Eq. 2 / Eq. 8) ----------------------------------------------------------------
    EpiCols<EPI> e;
    epi_cols<EPI>(p, nb * 32, lane, MODE != 0, e);
    const int64_t left = p.M - m0;
    const int rows = left > 32 ? 32 : (int)left;
    e_v4i res;
    epi_resid_load<EPI>(p, m0, rows, nb * 32, lane, res);
    epi_tile<EPI>(p, acc, 0, e, m0, rows, nb * 32, lane, res);
}

}  // namespace nq
