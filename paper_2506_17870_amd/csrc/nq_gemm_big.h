// Nested-integer GEMM main loop for large problems (paper Sec. 3.3: full-bit = w_high * 2^l +
// w_low recomposed on the fly, Eq. 4; part-bit = w_high with the scale s * 2^l, Eq. 8).  Also
// serves convolutions: 1x1 stride 1 is a GEMM over the NHWC pixels as it stands, and with CONV
// any filter over a power-of-two number of input channels (>= 16) is an implicit GEMM in which
// every 16-byte piece of an activation row is fetched from the input pixel its filter tap points
// at (or from out of range, which reads as zero, for the padding and for the tail of K).
//
// Block tile (32*TM) x 256, four waves side by side along N (wave tile 32*TM x 64: TM x 2 MFMA
// tiles of 32 x 32).  The K loop advances 256 at a time: one barrier per four K steps of 64.
// Activations travel global -> LDS directly (buffer loads with the LDS bit: no registers, no
// store instructions; rows past M read as zero through the range check), one iteration ahead,
// into one of two panels of 128 rows x 256 bytes.  A wave-wide LDS-direct load writes 1024
// contiguous bytes, so rows cannot be padded; instead the sixteen 16-byte pieces of row r are
// stored at position c ^ (r & 15): a panel row is 256 bytes, once round the 64 banks, so without
// the exchange the same piece of every row would sit in the same four banks, and with it sixteen
// neighbouring rows are read without bank conflicts.
// Weights: the packed dwords of a lane's own slot, requested four K steps (one iteration) ahead
// in a rolling register pipeline, decoded in registers and reused for the four row tiles.  All
// weight loads consumed in an iteration are older than that iteration's activation request, so
// waiting for them never waits for the slower activation loads.  LDS reads run four fragments
// ahead of the MFMAs that use them.  With TM <= 4 the kernel stays within 256 registers so that
// two blocks share a compute unit: one block's prologue, barrier waits and output stores hide
// behind the other's matrix-core work.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_epilogue.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int g_v4i __attribute__((ext_vector_type(4)));
typedef int g_v16i __attribute__((ext_vector_type(16)));
typedef unsigned g_v4u __attribute__((ext_vector_type(4)));

constexpr int GB_BN = 256, GB_KI = 4;                    // K steps of 64 per iteration
constexpr int GB_ROW = GB_KI * 64;                       // LDS bytes per panel row (swizzled, not padded)

// Slot m of a woven K step decodes dword m % 8 of a tile; the dwords past the H-th are gathered from the spare bits of
// the others and cost three times as many instructions.  gb_pref(H, n, i): the i-th of the n slots in the order in
// which they should take the step's other work (LDS reads, memory requests): the slots with a cheap dword first.
constexpr int gb_pref(int H, int n, int i)
{
    int seen = 0;
    for (int pass = 0; pass < 2; ++pass)
        for (int m = 0; m < n; ++m)
            if (((m % 8) < H) == (pass == 0)) {
                if (seen == i) return m;
                ++seen;
            }
    return i % n;
}

constexpr int gb_light(int H, int n)                      // how many of the n slots decode a cheap dword
{
    int c = 0;
    for (int m = 0; m < n; ++m) c += (m % 8) < H;
    return c;
}

typedef unsigned g_v2u __attribute__((ext_vector_type(2)));
typedef unsigned g_v3u __attribute__((ext_vector_type(3)));

// Dwords [4 * c, min(4 * c + 4, n_all)) of a slot's n_all packed dwords into dst, as one request.  (A function and not
// a lambda of the kernel: a lambda called from another lambda there makes the host pass drop the kernel's stub.)
__device__ __forceinline__ void gb_fetch(uint32_t *dst, const __amdgpu_buffer_rsrc_t &rs, int n_all, int c, int voff, int soff)
{
    const int n = n_all - 4 * c >= 4 ? 4 : n_all - 4 * c;
    if (n == 4) {
        const g_v4u v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 16 * c, soff, 0);
        dst[4 * c] = v[0]; dst[4 * c + 1] = v[1]; dst[4 * c + 2] = v[2]; dst[4 * c + 3] = v[3];
    } else if (n == 3) {
        const g_v3u v = __builtin_amdgcn_raw_buffer_load_b96(rs, voff + 16 * c, soff, 0);
        dst[4 * c] = v[0]; dst[4 * c + 1] = v[1]; dst[4 * c + 2] = v[2];
    } else if (n == 2) {
        const g_v2u v = __builtin_amdgcn_raw_buffer_load_b64(rs, voff + 16 * c, soff, 0);
        dst[4 * c] = v[0]; dst[4 * c + 1] = v[1];
    } else {
        dst[4 * c] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff + 16 * c, soff, 0);
    }
}

// TM: 32-row tiles per wave (block tile 32*TM x 256); the host picks TM so that the number of
// blocks fits the 256 compute units with little left over.  TM <= 4 fits two blocks per unit
// (the element-wise epilogue needs more registers and runs one block per unit rather than spill).
// FULL: 0 part-bit, 1 full-bit (unsigned lower part), 2 full-bit (compensated signed lower part).
// TMX: 2..5 = TM; 6 = TM 4 with the compute unit to itself (SOLO: 512 registers, the deep weight pipeline);
// 7 = TM 4 with one column tile per wave (NARROW: block tile 128 x 128, for layers of up to 128 output channels whose
// 256-column tile would be half empty; half the registers, so the deep pipeline and the woven K step fit two blocks per unit).
template <int H, int L, int FULL, int EPI, int TMX, bool CONV>
__global__ void __launch_bounds__(256, ((TMX <= 4 || TMX == 7) && EPI != EPI_ANY ? 2 : 1)) k_nested_gemm_big(const GemmParams p)
{
    constexpr int TM = TMX >= 6 ? 4 : TMX;
    constexpr bool SOLO = TMX == 5 || TMX == 6, NARROW = TMX == 7;
    constexpr int TN = NARROW ? 1 : 2, BN = 128 * TN;        // column tiles per wave, columns per block
    constexpr int GB_BM = 32 * TM;
    constexpr int GB_PANEL = GB_BM * GB_ROW;             // bytes per LDS panel
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;
    // weights are requested PD K steps ahead (registers permitting: TM = 4 shares the compute unit with a
    // second block and has 256 registers, TM >= 5 has 512)
    constexpr int PD = NARROW ? 4 : (TM == 4 && !SOLO && (FULL || H == 7) ? 2 : 4);
    constexpr int APT = 2 * TM;                          // LDS-direct loads per wave and iteration (4 rows each)

    extern __shared__ __attribute__((aligned(16))) uint8_t panel[];

    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index is the same for every lane of a wave: tell the compiler, so that everything
    // derived from it (tile numbers, page addresses) lives in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // n tiles vary fastest so that blocks running together share their activation rows
    const int nblocks = (p.N + BN - 1) / BN;
    const int bm = blockIdx.x / nblocks, bn = blockIdx.x - bm * nblocks;
    const int64_t m0 = (int64_t)bm * GB_BM;
    const int n0 = bn * BN;

    const int iters = (p.KB + GB_KI - 1) / GB_KI;

    // ---- first touch of the packed pages ----------------------------------------------------------
    // In a network every launch meets weights that no cache holds.  The K loop asks for them four steps
    // ahead, which covers the latency of L2 but not that of memory, and the blocks of a launch move in step:
    // each new K step would wait for memory once more.  So every wave first touches one dword in each of up to
    // 4 x 64 cache lines of either page, the waves that share an L2 (blocks 8 apart run on the same XCD) covering
    // the pages between them as far as they reach (3 MB per XCD with 24 blocks: the 2.4 MB pages of the 512-channel
    // 3x3 layers, which have few rows and therefore few blocks, took 36 us inside the forward and 30 us warm with a
    // single round of 64 lines); the values are not used.
    uint32_t touch_h = 0, touch_l = 0;
    {
        const int64_t waves_xcd = (int64_t)((gridDim.x + 7) >> 3) * 4;
        const int64_t dwords_h = (int64_t)p.NB * p.KB * (H * 64), dwords_l = (int64_t)p.NB * p.KB * (LP::DW * 64);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t line = (r * waves_xcd + (int64_t)(blockIdx.x >> 3) * 4 + wave) * 64 + lane;
            if (line * 32 < dwords_h) touch_h ^= p.ph[line * 32];
            if (FULL != 0 && line * 32 < dwords_l) touch_l ^= p.pl[line * 32];
        }
    }

    // ---- activations -------------------------------------------------------------------------
    // LDS-direct load k of wave w fills panel slots [(APT*w + k)*64, +64) (16 bytes each): lane l
    // writes row 4*(APT*w + k) + (l >> 4), position l & 15, and therefore fetches piece
    // c = (l & 15) ^ (row & 15) of that row, row & 15 = 4*((APT*w + k) & 3) + (l >> 4): four variants,
    // kept in the order in which this wave's loads k = 0, 1, 2, 3 (mod 4) need them.
    typedef __attribute__((address_space(3))) void *lds_ptr;
    constexpr int OOR = 0x7fff0000;                      // beyond every descriptor range: moves no data
    int piece[4];
#pragma unroll
    for (int par = 0; par < 4; ++par) piece[par] = (lane & 15) ^ (4 * ((APT * wave + par) & 3) + (lane >> 4));
    // GEMM: descriptor over the rows of this block; rows past M are out of range.
    // CONV: descriptor over the whole input tensor (the host keeps it below 2 GiB).
    const int64_t rows_here = (p.M - m0) < GB_BM ? (p.M - m0) : GB_BM;
    // (descriptors go through readfirstlane: one that the compiler believes to differ between lanes, e.g. because a
    // 64-bit product was computed on the vector ALU, is served by a loop over its distinct values at every use)
    auto uniform_ptr = [](const void *q) {
        const uint64_t a = reinterpret_cast<uint64_t>(q);
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
        return reinterpret_cast<void *>(((uint64_t)hi << 32) | lo);
    };
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        uniform_ptr(p.x + (CONV ? 0 : m0 * p.K)), 0,
        __builtin_amdgcn_readfirstlane(CONV ? (int)((int64_t)(p.M / ((int64_t)p.Ho * p.Wo)) * p.H * p.W * p.Cin)
                                            : (int)(rows_here * p.K)),
        0x00020000);
    int a_goff[4];                                       // GEMM: offset of the lane's piece in rows 0..3
    // CONV: per row of the block, the byte offset of filter tap (0,0) and the set of taps that fall into the
    // image for the pixel, worked out once, one row per thread, and handed to the lanes that request the row through a
    // small LDS table behind the panels
    int2 *rowtab = reinterpret_cast<int2 *>(panel + 2 * GB_PANEL);
    // with 96 or 128 rows per block (two blocks share the unit's registers) there is no room for them
    constexpr bool ROWREG = CONV && (TM <= 2 || SOLO || NARROW);
    int2 rowreg[ROWREG ? APT : 1];
    if constexpr (CONV) {
        if (tid < GB_BM) {
            const int HoWo = p.Ho * p.Wo;
            const int64_t m = m0 + tid;
            const int mm = m < p.M ? (int)m : 0;
            const int b = mm / HoWo, rem = mm - b * HoWo;
            const int oh = rem / p.Wo, ow = rem - oh * p.Wo;
            const int ih0 = oh * p.stride - p.pad, iw0 = ow * p.stride - p.pad;
            // which taps fall into the image for this pixel: bit kh (filter rows) and bit 16 + kw (filter
            // columns); rows past M get no bit at all
            const int h_lo = max(0, -ih0), h_hi = min(p.KH - 1, p.H - 1 - ih0);
            const int w_lo = max(0, -iw0), w_hi = min(p.KW - 1, p.W - 1 - iw0);
            const uint32_t hbits = h_hi >= h_lo ? (2u << h_hi) - (1u << h_lo) : 0u;
            const uint32_t wbits = w_hi >= w_lo ? (2u << w_hi) - (1u << w_lo) : 0u;
            rowtab[tid] = make_int2(((b * p.H + ih0) * p.W + iw0) * p.Cin,
                                    m < p.M ? (int)(hbits | (wbits << 16)) : 0);
        }
        __syncthreads();
        // a lane requests the same APT rows in every iteration: their entries move to registers once (read
        // from LDS inside the K loop, every request would wait for the table and, with it, for every
        // fragment read in flight)
        if constexpr (ROWREG) {
#pragma unroll
            for (int k = 0; k < APT; ++k) rowreg[k] = rowtab[4 * (wave * APT + k) + (lane >> 4)];
        }
    } else {
#pragma unroll
        for (int par = 0; par < 4; ++par)
            a_goff[par] = (wave * (4 * APT) + (lane >> 4)) * p.K + 16 * piece[par];
    }
    // CONV: where the lane's four pieces of iteration `it` come from: the k index of a piece -> filter tap
    // and channel (Cin is a power of two).  Worked out once per iteration, used by all its requests.
    // (24-bit multiplications: full rate on the vector ALU, where a 32-bit one takes four issue slots; a filter has
    // at most 15 x 16 taps and the image at most 8192 columns)
    int tap_off[4], tap_hw[4];
    auto set_taps = [&](int it) {
#pragma unroll
        for (int par = 0; par < 4; ++par) {
            const int kk = it * (GB_KI * 64) + 16 * piece[par];
            const int tap = kk >> p.cin_shift, ci = kk & (p.Cin - 1);
            const int kh = __mul24(tap, p.kw_magic) >> 16, kw = tap - __mul24(kh, p.KW);
            tap_off[par] = ((__mul24(kh, p.W) + kw) << p.cin_shift) + ci;
            // the tap's bits in a pixel's table entry; a piece past the end of K gets bit 15, which no pixel has
            tap_hw[par] = kk < p.K ? (int)((1u << kh) | (0x10000u << kw)) : 0x8000;
        }
    };
    // requests the loads k0 <= k < k1 of iteration `it` (all of them: k0 = 0, k1 = APT); CONV: rows[k - kbase] is
    // the table entry of the row load k fetches
    auto load_a = [&](int it, uint8_t *dst, int k0, int k1, const int2 *rows, int kbase) {
        // An iteration that does not exist is requested out of range, which moves no data.  No branch:
        // the loop body is the same straight-line code every time, which lets the compiler count
        // outstanding loads exactly instead of waiting conservatively.
        if constexpr (CONV) {
#pragma unroll
            for (int k = 0; k < APT; ++k) {
                if (k < k0 || k >= k1) continue;
                const int2 row = rows[k - kbase];
                const bool in = (row.y & tap_hw[k & 3]) == tap_hw[k & 3];
                const int off = in ? row.x + tap_off[k & 3] : OOR;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (lds_ptr)(dst + (wave * APT + k) * 1024), 16, off, 0, 0,
                                                         0);
            }
        } else {
            const int koff = it < iters ? it * (GB_KI * 64) : OOR;
#pragma unroll
            for (int k = 0; k < APT; ++k) {
                if (k < k0 || k >= k1) continue;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (lds_ptr)(dst + (wave * APT + k) * 1024), 16,
                                                         a_goff[k & 3] + k * 4 * p.K + koff, 0, 0, 0);
            }
        }
    };

    // ---- weights: rolling pipeline of packed dwords, PD K steps deep --------------------------
    const int nb0 = n0 / 32 + wave * TN;
    const int wslot = epi_weight_slot<EPI>(lane);             // channel order that suits the epilogue
    uint32_t P[PD][TN][H];
    uint32_t Q[PD][TN][LP::ARR];
    // K steps past the last one (K not a multiple of 256) read the last real tile: their activations
    // are zero.  Column tiles past N read the last real tile as well: their accumulators are never
    // stored.  So no masking is needed.
    int64_t tile0[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) tile0[t] = (int64_t)min(nb0 + t, p.NB - 1) * p.KB;
    // The wave's rows of tiles are read through buffer descriptors whose base is the wave's first tile: what varies
    // from request to request is then a small scalar offset (tile and K step) next to a constant lane offset, and
    // no address arithmetic is left for the vector ALU.  A K step that does not exist is requested out of range:
    // it returns zeros at once and moves nothing.
    const int tspan = __builtin_amdgcn_readfirstlane((int)(tile0[TN - 1] - tile0[0] + p.KB));
    const __amdgpu_buffer_rsrc_t hrsrc =
        __builtin_amdgcn_make_buffer_rsrc(uniform_ptr(p.ph + tile0[0] * (H * 64)), 0, tspan * (H * 256), 0x00020000);
    const __amdgpu_buffer_rsrc_t lrsrc = __builtin_amdgcn_make_buffer_rsrc(
        uniform_ptr(FULL != 0 ? p.pl + tile0[0] * (LP::DW * 64) : p.ph), 0, FULL != 0 ? tspan * (LP::DW * 256) : 0,
        0x00020000);
    int trel[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) trel[t] = __builtin_amdgcn_readfirstlane((int)(tile0[t] - tile0[0]));
    // The packed dwords of a slot are contiguous in the page (slot-major tiles), so a lane fetches them four at a
    // time: the address unit takes as long over a wave's request for one dword per lane as over one for four, and
    // with one request per dword it, not the matrix core, set the pace of the K loop.  A pipeline slot of a K step is
    // NBL requests: for each column tile the pieces of the higher-bit dwords, then those of the lower-bit dwords;
    // load_b issues the requests j0 <= j < j1 of K step kb.
    constexpr int CH = (H + 3) / 4, CL = (LP::DW + 3) / 4;          // requests per tile and page
    constexpr int NBL = TN * (CH + CL);
    auto load_b = [&](uint32_t (&Pd)[TN][H], uint32_t (&Qd)[TN][LP::ARR], int kb, int j0, int j1) {
        // (the last PD refills ask for K steps that do not exist and read the last real tile again: it is in the
        // cache, and turning them into out-of-range requests costs four instructions per refill all loop long)
        const int voff_h = wslot * (H * 4), voff_l = wslot * (LP::DW * 4);
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int tk = trel[t] + min(kb, p.KB - 1);
#pragma unroll
            for (int c = 0; c < CH; ++c)
                if (t * (CH + CL) + c >= j0 && t * (CH + CL) + c < j1) gb_fetch(Pd[t], hrsrc, H, c, voff_h, tk * (H * 256));
            if constexpr (FULL != 0) {
#pragma unroll
                for (int c = 0; c < CL; ++c)
                    if (t * (CH + CL) + CH + c >= j0 && t * (CH + CL) + CH + c < j1)
                        gb_fetch(Qd[t], lrsrc, LP::DW, c, voff_l, tk * (LP::DW * 256));
            }
        }
    };

    // With the compute unit's whole register file the per-channel constants of the epilogue are fetched here, behind
    // the first panel's latency, instead of after the K loop, where nothing would hide theirs.
    constexpr bool COLS_FIRST = SOLO || EPI == EPI_F32;       // constants of all column tiles before the first store
    EpiCols<EPI> ecols[COLS_FIRST ? TN : 1];
    if constexpr (SOLO) {
#pragma unroll
        for (int t = 0; t < TN; ++t) epi_cols<EPI>(p, n0 + (wave * TN + t) * 32, lane, FULL, ecols[t]);
    }

    g_v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][t][r] = 0;

    // in this order (the fences keep it): the loop's waits count on the panel being requested before
    // the weights, and on the weights of K step d before those of d + 1
    if constexpr (CONV) set_taps(0);
    if constexpr (CONV && !ROWREG) {
        int2 rows0[APT];
#pragma unroll
        for (int k = 0; k < APT; ++k) rows0[k] = rowtab[4 * (wave * APT + k) + (lane >> 4)];
        load_a(0, panel, 0, APT, rows0, 0);
    } else {
        load_a(0, panel, 0, APT, rowreg, 0);
    }
#pragma unroll
    for (int d = 0; d < PD; ++d) {
        __builtin_amdgcn_sched_barrier(0);
        load_b(P[d], Q[d], d, 0, NBL);
    }
    __builtin_amdgcn_sched_barrier(0);

    // LDS address of the lane's fragment for K step d and half hf: piece c = 4*d + 2*g + hf of row
    // r sits at position c ^ (r & 15); the row tiles are multiples of 32 rows, so r & 15 = lane & 15.
    int a_read[4][2];
    {
        const int r15 = lane & 15, g = lane >> 5;
#pragma unroll
        for (int d0 = 0; d0 < 4; ++d0)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
                a_read[d0][hf] = (lane & 31) * GB_ROW + 16 * ((4 * d0 + 2 * g + hf) ^ r15);
    }

    // Memory instructions are spread through the matrix-core stream: a burst of them would hold the
    // wave at the issue port (the address unit takes one at a time) while the matrix cores run dry.
    // Per K step the wave issues its share of the next panel's LDS-direct loads (first three K steps of
    // an iteration) and the refill of the weight slot whose dwords it has already decoded, a few after
    // every pair of MFMAs.  Where the weight pipeline is four K steps deep (AHEAD) the decoding is
    // spread the same way, one K step ahead: while the MFMAs of step d run, the wave decodes the weights
    // of step d + 1 in four slices (higher-bit fields, then lower-bit fields, of each of its two column
    // tiles), so that VALU and matrix cores work at the same time even when the wave has the SIMD to
    // itself.  With the two-step pipeline that would leave the loads a single K step to arrive; there
    // the weights of a step are decoded at its start.
    constexpr bool AHEAD = PD >= 4;
    g_v4i bfrag[TN][2];                                   // decoded weights of the current K step
    constexpr bool WOVEN = (SOLO && TM == 4) || NARROW;
    g_v4i bfr[WOVEN ? 2 : 1][TN][2];                      // woven K step: of the current and of the next step
    if constexpr (AHEAD) {
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            uint32_t D[8];
            HighCodec<H>::decode(P[0][t], D);
            LP::apply(Q[0][t], D);
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                bfrag[t][hf] = g_v4i{(int)D[4 * hf], (int)D[4 * hf + 1], (int)D[4 * hf + 2], (int)D[4 * hf + 3]};
                bfr[0][t][hf] = bfrag[t][hf];
                if constexpr (WOVEN) bfr[1][t][hf] = bfrag[t][hf];
            }
        }
    }
    // keeps the first-touch loads alive up to here and no further: loads complete in order and the first panel was
    // requested after them, so the loop's first wait covers them anyway, and their registers are free for the loop
    asm volatile("" ::"v"(touch_h), "v"(touch_l));
    for (int it = 0; it < iters; ++it) {
        uint8_t *cur = panel + (it & 1) * GB_PANEL;
        uint8_t *nxt = panel + ((it + 1) & 1) * GB_PANEL;
        // Every wave must have its own share of panel `cur` in LDS before anyone reads it.  Loads complete
        // in order and at least NBL weight loads follow a wave's last panel load (the prologue and the
        // last K step of an iteration request weights only), so "at most NBL loads outstanding" means
        // that the panel loads are done; the newest weight loads stay in flight.
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt((NBL & 15) | (7 << 4) | (15 << 8) | ((NBL >> 4) << 14));
        __syncthreads();                                  // panel `cur` has arrived, the other one is free
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (CONV) set_taps(it + 1);

        if constexpr (WOVEN) {
            // One wave per SIMD: nothing hides a stall, and whatever the wave issues between two MFMAs beyond what
            // fits in the shadow of the first delays the second.  So the K step is woven by hand, one fenced slot
            // per MFMA: the MFMA, the decoding of ONE dword of step d + 1's weights (the codec is called whole and
            // everything but that dword is dead code), and, in the slots whose dword is cheap to decode, the LDS read
            // of one fragment of step d + 1 or a refill of the pipeline slot decoded during the previous step; now and
            // then one of the next panel's requests.  Left to the scheduler the same work came out in bursts of sixty
            // instructions between two MFMAs (3950 -> 3440 clocks per four K steps on a 1024 -> 256 layer).
            constexpr int NF = 2 * TM, NM = NF * TN;
            g_v4i af[2][NF];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                af[0][f] = *reinterpret_cast<const g_v4i *>(cur + a_read[0][f / TM] + (f % TM) * 32 * GB_ROW);
#pragma unroll
            for (int d = 0; d < GB_KI; ++d) {
                const int kb = it * GB_KI + d;
                const int k0 = d * APT / (GB_KI - 1), k1 = (d + 1) * APT / (GB_KI - 1);   // this step's panel requests
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    const int f = m / TN, t = m % TN;
                    __builtin_amdgcn_sched_barrier(0);
                    acc[f % TM][t] = epi_mfma<EPI>(bfr[d & 1][t][f / TM], af[d & 1][f], acc[f % TM][t]);
                    if (d + 1 < GB_KI) {
#pragma unroll
                        for (int fr = 0; fr < NF; ++fr)       // fragment fr of step d + 1, in a slot with cheap decoding
                            if (gb_pref(H, NM, fr) == m)
                                af[(d + 1) & 1][fr] = *reinterpret_cast<const g_v4i *>(cur + a_read[d + 1][fr / TM] +
                                                                                       (fr % TM) * 32 * GB_ROW);
                    }
#pragma unroll
                    for (int q = m * 8 * TN / NM; q < (m + 1) * 8 * TN / NM; ++q) {   // one dword (TM = 4), or none
                        uint32_t Dn[8];
                        HighCodec<H>::decode(P[(d + 1) % PD][q / 8], Dn);
                        LP::apply(Q[(d + 1) % PD][q / 8], Dn);
                        bfr[(d + 1) & 1][q / 8][(q % 8) / 4][q % 4] = (int)Dn[q % 8];
                    }
#pragma unroll
                    for (int j = 0; j < NBL; ++j)             // refills in the cheap slots after those of the reads
                        if (gb_pref(H, NM, (NF + j) % gb_light(H, NM)) == m) load_b(P[d % PD], Q[d % PD], kb + PD, j, j + 1);
                    if (d < GB_KI - 1) {
#pragma unroll
                        for (int k = 0; k < APT; ++k)
                            if (k >= k0 && k < k1 && (k - k0) * NM / (k1 - k0) + 1 == m) load_a(it + 1, nxt, k, k + 1, rowreg, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else if constexpr (SOLO) {
            // (160-row blocks: the hand-woven form above runs out of registers)  The K step is written as plain data flow and the
            // instruction scheduler is told the pattern to weave: after every MFMA a handful of vector
            // instructions (the next step's decoding, addresses), every second one an LDS read, and the
            // step's memory requests spread evenly.  The fragments of step d + 1 are read during step d, so
            // that no MFMA waits for LDS inside an iteration; only the first step after the barrier does.
            constexpr int NF = 2 * TM;
            g_v4i af[2][NF];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                af[0][f] = *reinterpret_cast<const g_v4i *>(cur + a_read[0][f / TM] + (f % TM) * 32 * GB_ROW);
#pragma unroll
            for (int d = 0; d < GB_KI; ++d) {
                const int kb = it * GB_KI + d;
                __builtin_amdgcn_sched_barrier(0);
                if (d + 1 < GB_KI) {
#pragma unroll
                    for (int f = 0; f < NF; ++f)
                        af[(d + 1) & 1][f] =
                            *reinterpret_cast<const g_v4i *>(cur + a_read[d + 1][f / TM] + (f % TM) * 32 * GB_ROW);
                }
#pragma unroll
                for (int f = 0; f < NF; ++f)
#pragma unroll
                    for (int t = 0; t < TN; ++t)
                        acc[f % TM][t] = epi_mfma<EPI>(bfrag[t][f / TM], af[d & 1][f], acc[f % TM][t]);
                g_v4i bnext[TN][2];
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    uint32_t Dn[8];
                    HighCodec<H>::decode(P[(d + 1) % PD][t], Dn);
                    LP::apply(Q[(d + 1) % PD][t], Dn);
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2)
                        bnext[t][h2] = g_v4i{(int)Dn[4 * h2], (int)Dn[4 * h2 + 1], (int)Dn[4 * h2 + 2],
                                             (int)Dn[4 * h2 + 3]};
                }
                if (d < GB_KI - 1)
                    load_a(it + 1, nxt, d * APT / (GB_KI - 1), (d + 1) * APT / (GB_KI - 1), rowreg, 0);
                load_b(P[d % PD], Q[d % PD], kb + PD, 0, NBL);
#pragma unroll
                for (int m = 0; m < NF * TN; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);           // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);           // vector ALU in its shadow
                    if (m % 2 == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // an LDS read
                    if (m % 4 == 3) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);   // memory requests
                    else __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) bfrag[t][h2] = bnext[t][h2];
            }
        } else {
#pragma unroll
        for (int d = 0; d < GB_KI; ++d) {
            const int kb = it * GB_KI + d;
            constexpr int NF = 2 * TM, PF = 4;
            g_v4i bnext[TN][2];                           // the next K step's weights, decoded on the way
            uint32_t Dn[8];
            if constexpr (!AHEAD) {
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    HighCodec<H>::decode(P[d % PD][t], Dn);
                    LP::apply(Q[d % PD][t], Dn);
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2)
                        bfrag[t][h2] = g_v4i{(int)Dn[4 * h2], (int)Dn[4 * h2 + 1], (int)Dn[4 * h2 + 2],
                                             (int)Dn[4 * h2 + 3]};
                }
            }

            // CONV without room for the whole row table in registers: the entries this K step's requests need
            // are read with the step's first fragments, so that no request waits for the table in mid-step
            constexpr int RS = (APT + GB_KI - 2) / (GB_KI - 1);
            const int rs_k0 = d * APT / (GB_KI - 1);
            int2 rowstep[RS];
            if constexpr (CONV && !ROWREG) {
                if (d < GB_KI - 1) {
#pragma unroll
                    for (int k = 0; k < RS; ++k)
                        rowstep[k] = rowtab[4 * (wave * APT + min(rs_k0 + k, APT - 1)) + (lane >> 4)];
                }
            }
            // fragment f = (hf, i): LDS reads four fragments ahead of their MFMAs
            g_v4i af[PF];
#pragma unroll
            for (int f = 0; f < PF; ++f)
                af[f] = *reinterpret_cast<const g_v4i *>(cur + a_read[d][f / TM] + (f % TM) * 32 * GB_ROW);
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const int i = f % TM, hf = f / TM;
                const g_v4i a = af[f % PF];
                __builtin_amdgcn_sched_barrier(0);
                if (f + PF < NF)
                    af[f % PF] = *reinterpret_cast<const g_v4i *>(cur + a_read[d][(f + PF) / TM] +
                                                                  ((f + PF) % TM) * 32 * GB_ROW);
#pragma unroll
                for (int t = 0; t < TN; ++t) acc[i][t] = epi_mfma<EPI>(bfrag[t][hf], a, acc[i][t]);
                // a slice of the next step's decoding
#pragma unroll
                for (int t = 0; t < TN && AHEAD; ++t) {
                    if (f == t * NF / TN) HighCodec<H>::decode(P[(d + 1) % PD][t], Dn);
                    if (f == t * NF / TN + 1) {
                        LP::apply(Q[(d + 1) % PD][t], Dn);
#pragma unroll
                        for (int h2 = 0; h2 < 2; ++h2)
                            bnext[t][h2] = g_v4i{(int)Dn[4 * h2], (int)Dn[4 * h2 + 1], (int)Dn[4 * h2 + 2],
                                                 (int)Dn[4 * h2 + 3]};
                    }
                }
                // this step's share of the memory requests; the slot refilled has been decoded (during the
                // previous step, or at the start of this one)
                if (d < GB_KI - 1)
                    load_a(it + 1, nxt, (d * NF + f) * APT / ((GB_KI - 1) * NF),
                           (d * NF + f + 1) * APT / ((GB_KI - 1) * NF), ROWREG ? rowreg : rowstep, ROWREG ? 0 : rs_k0);
                load_b(P[d % PD], Q[d % PD], kb + PD, f * NBL / NF, (f + 1) * NBL / NF);
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (AHEAD) {
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) bfrag[t][h2] = bnext[t][h2];
            }
        }
        }
    }

    // ---- epilogue (Eq. 2 / Eq. 8): every load first, then one wait, then arithmetic and stores -------
    // Loads and stores share one counter and it counts in order: a wait for a load that the compiler places
    // after a store has been issued is a wait for that store's acknowledgement as well.  It places one
    // wherever a register is reused that a load may still be writing, and the residual requests below are
    // conditional, so on the path without a residual they stay "pending" in its books for good: every tile's
    // arithmetic then waited for the previous tile's store to come back from memory (half of the epilogue's
    // time).  Hence the order here: per-channel constants and residual codes of all tiles are requested,
    // epi_join() waits for everything once, and from there to the end nothing is loaded.
    auto rows_of = [&](int i) {
        const int64_t left = p.M - (m0 + i * 32);
        return left > 32 ? 32 : (left < 0 ? 0 : (int)left);
    };
    if constexpr (COLS_FIRST && !SOLO) {
#pragma unroll
        for (int t = 0; t < TN; ++t) epi_cols<EPI>(p, n0 + (wave * TN + t) * 32, lane, FULL, ecols[t]);
    }
    e_v4i res[TM * TN];
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int i = 0; i < TM; ++i)
            epi_resid_load<EPI>(p, m0 + i * 32, rows_of(i), n0 + (wave * TN + t) * 32, lane, res[t * TM + i]);
    epi_join();
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int nt0 = n0 + (wave * TN + t) * 32;
        EpiCols<EPI> e;
        if constexpr (COLS_FIRST) e = ecols[t];
        else epi_cols<EPI>(p, nt0, lane, FULL, e);
#pragma unroll
        for (int i = 0; i < TM; ++i)
            epi_tile<EPI>(p, acc[i][t], SHIFT, e, m0 + i * 32, rows_of(i), nt0, lane, res[t * TM + i]);
    }
}

// Picks the rows per block: cost ~ (rounds of blocks over the compute units) x (TM + the per-K-step
// work that does not shrink with TM), two blocks sharing a unit counted as 0.85 of running one
// after the other.
inline int gemm_big_pick_tm(int64_t M, int64_t N, bool filter)
{
    const int64_t nblocks = (N + GB_BN - 1) / GB_BN;
    // A filter (implicit GEMM with a gather per tap) whose 128-row blocks would not even fill the compute units
    // once runs better as twice as many 64-row blocks, two per unit (3x3, 14x14x256 -> 256 at batch 128 inside
    // the ResNet-101 forward: 29.2 us against 31.0 us; 3x3 stride 2, 28x28x256 -> 256: 27.6 us against 34.8 us).
    // With at least three quarters of the compute units busy the 128-row blocks win after all, each with a unit to
    // itself (variant 6, chosen by the launcher: 24.8 us against 27.3 us for the first of these layers).
    if (filter && ((M + 127) / 128) * nblocks <= 256 && ((M + 127) / 128) * nblocks >= 190) return 4;
    if (filter && ((M + 127) / 128) * nblocks <= 256 && ((M + 63) / 64) * nblocks <= 512) return 2;
    int best = 4;
    double best_cost = 1e30;
    for (int tm = 2; tm <= 5; ++tm) {
        const int64_t blocks = ((M + 32 * tm - 1) / (32 * tm)) * nblocks;
        const double rounds = (double)((blocks + 255) / 256);
        const double cost = rounds * (tm + 1.5) * (tm <= 4 && blocks > 256 ? 0.85 : 1.0);
        if (cost < best_cost) { best_cost = cost; best = tm; }
    }
    return best;
}

template <int H, int L>
void launch_nested_gemm_big(bool full, const GemmParams &p, int tm_forced, int *tm_used, hipStream_t st,
                            void *ev_start, void *ev_stop)
{
    int nblocks = (p.N + GB_BN - 1) / GB_BN;
    const int mode = epi_mode(p);
    int tm = mode == EPI_ANY ? 4 : gemm_big_pick_tm(p.M, p.N, p.conv_big && p.KH * p.KW > 1);   // the element-wise epilogue is built for TM = 4 only
    // 128-row blocks that have a compute unit each anyway take its whole register file (variant 6)
    if (tm == 4 && mode != EPI_ANY && ((p.M + 127) / 128) * nblocks <= 256) tm = 6;
    // up to 128 output channels: 128-column blocks (variant 7)
    if (mode != EPI_ANY && p.N <= 128) tm = 7;
    if (mode != EPI_ANY && tm_forced >= 2 && tm_forced <= 7) tm = tm_forced;   // test / tuning aid
    if (tm == 7) nblocks = (p.N + 127) / 128;
    if (tm_used) *tm_used = tm;
#define NQ_GB_LAUNCH(FULLV, EPIV, TMV, CONVV)                                               \
    do {                                                                                    \
        auto k = k_nested_gemm_big<H, L, FULLV, EPIV, TMV, CONVV>;                          \
        constexpr int ROWS = 32 * (TMV >= 6 ? 4 : TMV);                                     \
        const size_t lds = 2 * (size_t)ROWS * GB_ROW + (CONVV ? 8 * ROWS : 0);              \
        const int64_t mblocks = (p.M + ROWS - 1) / ROWS;                                    \
        static bool granted = false;                                                        \
        if (!granted) {                                                                     \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k),                    \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            granted = true;                                                                 \
        }                                                                                   \
        launch_timed(k, dim3((unsigned)(mblocks * nblocks)), dim3(256), lds, st, ev_start, ev_stop, p); \
    } while (0)
#define NQ_GB_TM(FULLV, EPIV, CONVV)                             \
    do {                                                         \
        if (tm == 2) NQ_GB_LAUNCH(FULLV, EPIV, 2, CONVV);        \
        else if (tm == 3) NQ_GB_LAUNCH(FULLV, EPIV, 3, CONVV);   \
        else if (tm == 5) NQ_GB_LAUNCH(FULLV, EPIV, 5, CONVV);   \
        else if (tm == 6) NQ_GB_LAUNCH(FULLV, EPIV, 6, CONVV);   \
        else if (tm == 7) NQ_GB_LAUNCH(FULLV, EPIV, 7, CONVV);   \
        else NQ_GB_LAUNCH(FULLV, EPIV, 4, CONVV);                \
    } while (0)
#define NQ_GB_MODE(FULLV, CONVV)                                         \
    do {                                                                 \
        if (mode == EPI_ANY) NQ_GB_LAUNCH(FULLV, EPI_ANY, 4, CONVV);     \
        else if (mode == EPI_I8) NQ_GB_TM(FULLV, EPI_I8, CONVV);         \
        else NQ_GB_TM(FULLV, EPI_F32, CONVV);                            \
    } while (0)
    const int fmode = full ? (p.low_signed ? 2 : 1) : 0;
    if (p.conv_big) {
        if (fmode == 2) NQ_GB_MODE(2, true); else if (fmode == 1) NQ_GB_MODE(1, true); else NQ_GB_MODE(0, true);
    } else {
        if (fmode == 2) NQ_GB_MODE(2, false); else if (fmode == 1) NQ_GB_MODE(1, false); else NQ_GB_MODE(0, false);
    }
}

}  // namespace nq
