// Nested-integer GEMM for short reductions (K = 64, 128 or 256: the 1x1 convolutions of a CNN with that
// many input channels, at any stride), weights stationary in registers (paper Sec. 3.3: full-bit =
// w_high * 2^l + w_low recomposed on the fly, Eq. 4; part-bit = w_high with the scale s * 2^l, Eq. 8;
// 8-bit activations, Sec. 4.2).
//
// With K this short a layer is all input rows in, output rows out and epilogue arithmetic: a 128 x 256 output
// tile has 1 us of matrix-core work against 2 us of fp32 dequantisation, and a kernel that gives every tile its
// own block runs fetch, matrix cores, epilogue and stores one after the other.  Here a block is persistent.
// It loads and decodes the packed weights of its columns ONCE (wave tile 64 columns x K: 16 to 64 registers
// of decoded operand bytes per lane) and then walks over row tiles: the activation rows of the tiles ahead
// travel global -> LDS directly (buffer loads with the LDS bit, no registers, no store instructions) into a
// ring of two or three panels while the current tile is multiplied and the previous one is dequantised and
// stored, and the second block on the compute unit is in another phase of the same loop.  The tile loop has
// one barrier per tile and no decoding.  Every block gets the same number of consecutive rows.
//
// Rows are GEMM rows m = (image, oh, ow); for a strided 1x1 convolution row m starts at pixel
// (oh * stride, ow * stride) of its image, so only the pixels the layer needs are fetched.  Rows past M are
// requested out of the descriptor's range, which reads as zero.
//
// Panel layout: BM rows of K bytes, not padded (a wave-wide LDS-direct load writes 1024 contiguous bytes).
// The 16-byte pieces of row r are stored at position c ^ f(r), f chosen so that the sixteen rows a 16-byte
// LDS read serves together fall into sixteen different bank groups: f(r) = r & 15 for rows of 256 bytes or
// more, (r >> 1) & 7 for 128 bytes, (r >> 2) & 3 for 64 bytes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "nq_codec.h"
#include "nq_epilogue.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int s_v4i __attribute__((ext_vector_type(4)));
typedef int s_v16i __attribute__((ext_vector_type(16)));
typedef unsigned s_u4v __attribute__((__vector_size__(4 * sizeof(unsigned))));    // what the 16-byte buffer store takes

constexpr int ST_OOR = 0x7fff0000;            // beyond every descriptor range (the host keeps inputs smaller)

// KS: K steps of 64 (1, 2 or 4: exact, so that the decoded weights are a register array and the K loop is
// straight-line code).  WN: waves along N (4: 256 columns per block; 2: 128; 1: 64).
template <int H, int L, int FULL, int EPI, int KS, int WN>
__global__ void __launch_bounds__(256, EPI == EPI_ANY ? 1 : 2) k_nested_gemm_stat(const GemmParams p, const StatGeom g)
{
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;
    constexpr int WM = 4 / WN, TM = st_tm(WN), TN = 2;
    constexpr int BM = st_bm(WN);
    constexpr int ROWB = 64 * KS, P = ROWB / 16;             // bytes and 16-byte pieces per panel row
    constexpr int SW = P < 16 ? P : 16;                      // positions the exchange runs over
    constexpr int PANEL = BM * ROWB;
    constexpr int RD = st_ring(KS, WN);                      // panels in the ring
    constexpr int NWL = PANEL / 1024, LW = (NWL + 3) / 4;    // wave-wide loads per panel, per wave
    static_assert(PANEL % 1024 == 0 && P <= 64, "whole wave-wide loads");

    extern __shared__ __attribute__((aligned(16))) uint8_t ring[];
    uint8_t *dump = ring + RD * PANEL;
    float *cols_lds = reinterpret_cast<float *>(dump + 1024);
    uint8_t *resid_lds = dump + 1024 + 4 * 2 * 64 * sizeof(float);    // [wave][TN * TM tiles][64 lanes x 16 bytes]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    // Block id -> (row-tile slot, column group).  Consecutive ids go to different XCDs (id % 8), each with its
    // own L2; the blocks that stream the same rows for different column groups get ids 8 apart: same XCD,
    // dispatched back to back, so that all but the first find the rows in L2.
    const int bid = blockIdx.x, xcd = bid & 7, bj = bid >> 3;
    const int cg = bj % g.cgroups;
    const int slot = (bj / g.cgroups) * 8 + xcd;
    // Rows of a slot: either a run of g.rps consecutive rows, cut into tiles of BM rows from its first row on
    // (every slot then has the same number of rows, the last tile of a slot being a partial one), or, with
    // g.interleave, the tiles slot, slot + nslots, ... of the whole row range.
    if (slot >= g.nslots) return;                            // the whole block: no barrier is skipped
    const int64_t r_begin = g.interleave ? (int64_t)slot * BM : (int64_t)slot * g.rps;
    const int64_t r_step = g.interleave ? (int64_t)g.nslots * BM : BM;      // from one tile of the block to its next
    const int64_t r_end = g.interleave ? p.M : (r_begin + g.rps < p.M ? r_begin + g.rps : p.M);
    if (r_begin >= r_end) return;
    const int nt = (int)((r_end - r_begin + r_step - 1) / r_step);

    const int nb0 = (cg * WN + wn) * TN;
    // ---- lane constants of the requests, worked out before the first load is issued -------------------
    // (a 32-bit multiply-add is a 64-bit instruction whose unused upper halves the register allocator puts
    // anywhere, e.g. on a register that a load in flight is about to write, which costs a wait for that load)
    constexpr int NS = TM * TN;                              // residual loads = stores per wave and tile
    // wave-wide load j of this wave fills panel bytes [(wave * LW + j) * 1024, + 1024): lane l writes piece
    // slot q = (wave * LW + j) * 64 + l = (row, position), and therefore fetches piece c = position ^ f(row)
    int ld_row[LW], ld_c16[LW];
#pragma unroll
    for (int j = 0; j < LW; ++j) {
        const int q = (wave * LW + j) * 64 + lane;
        const int row = q / P, pos = q % P;
        ld_row[j] = row;
        ld_c16[j] = 16 * (pos ^ ((row / (16 / SW)) & (SW - 1)));
    }
    int pan_lane[LW];
#pragma unroll
    for (int j = 0; j < LW; ++j) pan_lane[j] = ld_row[j] * ROWB + ld_c16[j];
    // output / residual offsets: lane part of tile (t, i) = out0 + i * n32 + t * 32 (see NQ_ST_OUT_OFF below)
    const int brow0 = wm * 32 * TM + (lane & 31), ch0 = nb0 * 32 + 16 * (lane >> 5);
    const int out0 = brow0 * (int)p.N + ch0, n32 = 32 * (int)p.N;
    __builtin_amdgcn_sched_barrier(0);

    // ---- per-channel scale and bias (int8 epilogue) and weights: every K step of the wave's two column tiles ----
    // Scale and bias are requested here and turned into the epilogue's constants after everything else has been
    // requested: the counter of outstanding loads counts in order, so a load that is waited for after the panels
    // have been requested is a wait for the panels, the whole input of the block.
    EpiRaw16 craw[EPI == EPI_I8 ? TN : 1];
    uint32_t W8[TN][KS][H + LP::DW > 8 ? H + LP::DW : 8];    // packed dwords on arrival, decoded afterwards
    auto load_weights = [&]() {
        if constexpr (EPI == EPI_I8) {
#pragma unroll
            for (int t = 0; t < TN; ++t) epi_cols16_fetch(p, (nb0 + t) * 32 + 16 * (lane >> 5), craw[t]);
            __builtin_amdgcn_sched_barrier(0);
        }
        const int wslot = epi_weight_slot<EPI>(lane);        // channel order that suits the epilogue
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int nb = min(nb0 + t, p.NB - 1);           // a tile past N repeats the last one, never stored
            const uint32_t *ph = p.ph + (int64_t)nb * p.KB * (H * 64);
            const uint32_t *pl = FULL ? p.pl + (int64_t)nb * p.KB * (LP::DW * 64) : nullptr;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
#pragma unroll
                for (int i = 0; i < H; ++i) W8[t][s][i] = ph[(unsigned)(s * (H * 64) + wslot * H + i)];
                if constexpr (FULL != 0) {
#pragma unroll
                    for (int i = 0; i < LP::DW; ++i)
                        W8[t][s][H + i] = pl[(unsigned)(s * (LP::DW * 64) + wslot * LP::DW + i)];
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // A wave can have 63 memory instructions in flight; its 64 to 80 requests for weights and constants alone
    // exceed that, and whatever is issued after them waits for the first of them to come back from memory.  With
    // the int8 epilogue the panels and residual codes (24 requests, the ones that go all the way to memory) are
    // therefore requested first and the weights (mostly found in L2) behind them.
    if constexpr (EPI != EPI_I8) load_weights();

    // ---- activation panels ------------------------------------------------------------------------
    typedef __attribute__((address_space(3))) void *lds_ptr;
    const __amdgpu_buffer_rsrc_t xrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0, g.x_bytes, 0x00020000);
    // requests the rows of this block's i-th tile into panel i % RD; a tile that does not exist is requested
    // out of range into the dump area, so that every wave issues the same loads whatever happens (the waits
    // below count them).  The offset of a request is a scalar (the tile's first row) plus a lane part that never
    // changes, added on the vector ALU and not handed over in the instruction's scalar offset operand.  For the
    // 16-byte stores of the outputs that operand must stay an immediate: the compiler puts the wait state between
    // such a store and a vector instruction that overwrites its data registers only when the store has no register
    // there, and the hardware needs it in both cases (with a register, the first data dword of lanes 12-15 of every
    // sixteen was stored as the next instruction left it).  The loads of this kernel follow the same form.
    auto load_panel = [&](int i) {
        const bool real = i < nt;
        const int64_t m0 = r_begin + (int64_t)i * r_step;
        const int64_t left = r_end - m0;
        const int rl = real ? (left < BM ? (int)left : BM) : 0;          // rows of the tile that exist
        uint8_t *dst = ring + (i % RD) * PANEL;
        int b0 = 0, rem0 = 0, pbase = 0;
        if (g.strided) {
            b0 = (int)(m0 / g.howo);
            rem0 = (int)(m0 - (int64_t)b0 * g.howo);
        } else if (real) {
            pbase = (int)(m0 * ROWB);
        }
#pragma unroll
        for (int j = 0; j < LW; ++j) {
            const int k = wave * LW + j;
            const bool in = k < NWL && ld_row[j] < rl;
            int off;
            if (g.strided) {
                const unsigned n = (unsigned)(rem0 + ld_row[j]);
                // a magic of 0 stands for a divisor of 1, whose reciprocal does not fit 32 bits
                const unsigned qb = g.howo_magic ? __umulhi(n, g.howo_magic) : n, r = n - qb * (unsigned)g.howo;
                const unsigned oh = g.wo_magic ? __umulhi(r, g.wo_magic) : r, ow = r - oh * (unsigned)p.Wo;
                off = (b0 + (int)qb) * g.img_bytes + (int)oh * g.row_step + (int)ow * g.col_step + ld_c16[j];
            } else {
                off = pbase + pan_lane[j];
            }
            uint8_t *d = (real && k < NWL) ? dst + k * 1024 : dump;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (lds_ptr)d, 16, in ? off : ST_OOR, 0, 0, 0);
        }
    };

    // ---- int8 outputs: residual codes and output codes as buffer accesses ------------------------------
    // The tile loop of the int8 epilogue has no load into registers and a fixed number of vector-memory
    // instructions per tile, so that every wait in it is an exact count (loads and stores share one counter, and
    // a wait the compiler places for a register load with stores in flight is a wait for everything).  The
    // residual codes therefore travel global -> LDS directly like the panels (a lane's sixteen bytes land at
    // 16 * lane of the tile's KB: read back without bank conflicts), one tile ahead, and both they and the output
    // codes go through range-checked descriptors: what a lane has no row or channel for is requested out of
    // range (reads zero, writes nothing) instead of being branched around.
    const int64_t out_bytes = p.M * p.N;                     // the host keeps M * N below 2^31 - 2^16
    const __amdgpu_buffer_rsrc_t rrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(p.resid), 0, p.resid ? (int)out_bytes : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t yrsrc =
        __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<int8_t *>(p.y), 0, (int)out_bytes, 0x00020000);
    uint8_t *my_resid = resid_lds + wave * (NS * 1024);
    // Offset of the lane's sixteen channels of row (lane & 31) of tile (t, i) of the block's tile `it` in the output
    // (and the residual): a scalar, the tile's first row, plus a lane part that never changes, the sum replaced by
    // "out of range" for rows the tile does not have and channels past N.
#define NQ_ST_TILE(IT, RL, BASE)                                                            \
    const int64_t tm0_##RL = r_begin + (int64_t)(IT) * r_step, left_##RL = r_end - tm0_##RL; \
    const int RL = (IT) < nt ? (left_##RL < BM ? (int)left_##RL : BM) : 0;                   \
    const int BASE = (IT) < nt ? (int)(tm0_##RL * p.N) : 0
#define NQ_ST_OUT_OFF(RL, BASE, T, I) \
    ((brow0 + (I) * 32 < (RL) && ch0 + (T) * 32 < (int)p.N) ? (BASE) + out0 + (I) * n32 + (T) * 32 : (int)ST_OOR)
    // requests the residual codes of the block's tile IT into the wave's staging area.  (Macros and plain integers on
    // purpose: with a lambda called from a lambda here, and again with small per-tile index arrays in place of
    // brow0 / out0, the host pass silently dropped the kernel's stub, which shows only when the library is loaded;
    // the build loads it for that reason.)
#define NQ_ST_LOAD_RESID(IT, RL, BASE)                                                                            \
    do {                                                                                                          \
        NQ_ST_TILE(IT, RL, BASE);                                                                                 \
        _Pragma("unroll") for (int t_ = 0; t_ < TN; ++t_)                                                         \
            _Pragma("unroll") for (int i_ = 0; i_ < TM; ++i_)                                                     \
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rrsrc, (lds_ptr)(my_resid + (t_ * TM + i_) * 1024), 16,  \
                                                         NQ_ST_OUT_OFF(RL, BASE, t_, i_), 0, 0, 0);               \
    } while (0)

    __builtin_amdgcn_sched_barrier(0);                       // the waits below count on the order of the requests
    if constexpr (EPI == EPI_I8) {
        // the order of a tile of the loop below: residual codes, newest panel, stores (here: NS stores of nothing)
#pragma unroll
        for (int i = 0; i < RD - 1; ++i) {
            load_panel(i);
            __builtin_amdgcn_sched_barrier(0);
        }
        NQ_ST_LOAD_RESID(0, rl0, base0);
        __builtin_amdgcn_sched_barrier(0);
        load_panel(RD - 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NS; ++j)
            __builtin_amdgcn_raw_buffer_store_b128(s_u4v{(unsigned)j, 0u, 0u, 0u}, yrsrc, ST_OOR + 4096 * j + 16 * lane, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        load_weights();
    } else {
#pragma unroll
        for (int i = 0; i < RD; ++i) {
            load_panel(i);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- per-lane constants -------------------------------------------------------------------------
    // LDS offset of the lane's fragment of K step s, half hf, row tile 0: piece c = 4s + 2g + hf of its row
    int a_read[KS][2];
    {
        const int row = wm * 32 * TM + (lane & 31), gk = lane >> 5;
        const int fr = (row / (16 / SW)) & (SW - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) a_read[s][hf] = row * ROWB + 16 * ((4 * s + 2 * gk + hf) ^ fr);
    }
    const int rg = lane >> 5;
    // The per-channel constants of the wave's column tiles wait in LDS and are read back for every tile: held
    // in registers for the whole kernel they would push it into scratch.  A wave reads only what it wrote.
    float *my_cols = cols_lds + wave * (TN * 64);
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        EpiCols<EPI> ec;
        if constexpr (EPI == EPI_I8) epi_cols16_finish(p, FULL, craw[t], ec);
        else epi_cols<EPI>(p, (nb0 + t) * 32, lane, FULL, ec);
        if constexpr (EPI == EPI_F32) {
            my_cols[64 * t + (lane & 31)] = ec.c[0];
            my_cols[64 * t + 32 + (lane & 31)] = ec.bias[0];
        } else if ((lane & 31) == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                my_cols[64 * t + 32 * rg + r] = ec.c[r];
                my_cols[64 * t + 32 * rg + 16 + r] = ec.bias[r];
            }
        }
    }

    // ---- decode the weights in place into matrix-core fragments ---------------------------------------
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint32_t Pk[H], D[8];
#pragma unroll
            for (int i = 0; i < H; ++i) Pk[i] = W8[t][s][i];
            HighCodec<H>::decode(Pk, D);
            if constexpr (FULL != 0) {
                uint32_t Qk[LP::ARR];
#pragma unroll
                for (int i = 0; i < LP::DW; ++i) Qk[i] = W8[t][s][H + i];
                LP::apply(Qk, D);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) W8[t][s][i] = D[i];
        }

    // Loads complete in order, so "at most n loads outstanding" means that everything older than the newest n
    // has landed.  Stores share the counter and make the wait stricter, never weaker.
    auto wait_loads = [](auto n) {
        constexpr int N = decltype(n)::value;
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
    };
    // panel 0 (and the weights before it) are in: everything requested after it may still travel
    // (int8 epilogue: the weights were requested last, the decoding above has waited for them and with them for everything)
    wait_loads(std::integral_constant<int, EPI == EPI_I8 ? 0 : (RD - 1) * LW>{});
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);

    auto rows_of = [&](int64_t m0, int i) {
        const int64_t left = r_end - (m0 + i * 32);
        return left > 32 ? 32 : (left < 0 ? 0 : (int)left);
    };
    // residual codes of a tile (requested one tile ahead: they come from memory, not from a cache)
    auto load_resid = [&](int it, e_v4i (&res)[TM * TN]) {
        const int64_t m0 = r_begin + (int64_t)it * r_step + wm * 32 * TM;
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int i = 0; i < TM; ++i)
                epi_resid_load<EPI>(p, m0 + i * 32, it < nt ? rows_of(m0, i) : 0, (nb0 + t) * 32, lane, res[t * TM + i]);
    };
    if constexpr (EPI == EPI_I8) {
        for (int it = 0; it < nt; ++it) {
            const uint8_t *cur = ring + (it % RD) * PANEL;

            s_v16i acc[TM][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][t][r] = 0;
            constexpr int NF = 2 * KS * TM, PF = NF < 4 ? NF : 4;
            s_v4i af[PF];
#pragma unroll
            for (int f = 0; f < PF; ++f)
                af[f] = *reinterpret_cast<const s_v4i *>(cur + a_read[(f / TM) >> 1][(f / TM) & 1] + (f % TM) * 32 * ROWB);
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                const int i = f % TM, s = (f / TM) >> 1, hf = (f / TM) & 1;
                const s_v4i a = af[f % PF];
                __builtin_amdgcn_sched_barrier(0);
                if (f + PF < NF)
                    af[f % PF] = *reinterpret_cast<const s_v4i *>(
                        cur + a_read[((f + PF) / TM) >> 1][((f + PF) / TM) & 1] + ((f + PF) % TM) * 32 * ROWB);
#pragma unroll
                for (int t = 0; t < TN; ++t) {
                    const s_v4i bfrag = s_v4i{(int)W8[t][s][4 * hf], (int)W8[t][s][4 * hf + 1], (int)W8[t][s][4 * hf + 2],
                                              (int)W8[t][s][4 * hf + 3]};
                    acc[i][t] = epi_mfma<EPI>(bfrag, a, acc[i][t]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }

            // This tile's residual codes and the next tile's panel must have landed (this wave's share; the barrier
            // collects the others'), and every wave must be done with the current panel before it is requested
            // again.  Issue order per tile: residual codes of the next tile, the panel RD tiles ahead, this tile's
            // NS stores.  The newer of the two things waited for is the residual request of the previous tile (with
            // a ring of two: the panel requested after it); what was issued after it, one panel and NS stores (NS
            // stores), may stay in flight: no wait for the acknowledgements of the latest stores.
            wait_loads(std::integral_constant<int, (RD >= 3 ? LW : 0) + NS>{});
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            e_v4i res[NS];
#pragma unroll
            for (int j = 0; j < NS; ++j) res[j] = *reinterpret_cast<const e_v4i *>(my_resid + j * 1024 + 16 * lane);
            // the codes are in registers before their place in LDS is requested again
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(0xc07f);              // lgkmcnt(0) only
            __builtin_amdgcn_sched_barrier(0);
            NQ_ST_LOAD_RESID(it + 1, rl_n, base_n);
            __builtin_amdgcn_sched_barrier(0);
            load_panel(it + RD);                             // into the panel this tile has just been read from
            __builtin_amdgcn_sched_barrier(0);

            // ---- epilogue (Eq. 2 / Eq. 8) ------------------------------------------------------------
            NQ_ST_TILE(it, rl_out, base_out);
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                EpiCols<EPI_I8> e;
                const e_v4f *cl = reinterpret_cast<const e_v4f *>(my_cols + 64 * t + 32 * rg);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const e_v4f cc = cl[q], bb = cl[4 + q];
#pragma unroll
                    for (int i = 0; i < 4; ++i) { e.c[4 * q + i] = cc[i]; e.bias[4 * q + i] = bb[i]; }
                }
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const e_v4i q = epi_codes16(p, acc[i][t], SHIFT, e, res[t * TM + i]);
                    __builtin_amdgcn_raw_buffer_store_b128(s_u4v{(unsigned)q[0], (unsigned)q[1], (unsigned)q[2], (unsigned)q[3]},
                                                           yrsrc, NQ_ST_OUT_OFF(rl_out, base_out, t, i), 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        return;
    }
#undef NQ_ST_LOAD_RESID
#undef NQ_ST_OUT_OFF
#undef NQ_ST_TILE
    e_v4i res[TM * TN], res_next[TM * TN];
    load_resid(0, res);

    for (int it = 0; it < nt; ++it) {
        const uint8_t *cur = ring + (it % RD) * PANEL;
        const int64_t m0 = r_begin + (int64_t)it * r_step + wm * 32 * TM;

        s_v16i acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][t][r] = 0;
        // fragment f = (s, hf, i): LDS reads run PF fragments ahead of the MFMAs that use them
        constexpr int NF = 2 * KS * TM, PF = NF < 4 ? NF : 4;
        s_v4i af[PF];
#pragma unroll
        for (int f = 0; f < PF; ++f)
            af[f] = *reinterpret_cast<const s_v4i *>(cur + a_read[(f / TM) >> 1][(f / TM) & 1] + (f % TM) * 32 * ROWB);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            const int i = f % TM, s = (f / TM) >> 1, hf = (f / TM) & 1;
            const s_v4i a = af[f % PF];
            __builtin_amdgcn_sched_barrier(0);
            if (f + PF < NF)
                af[f % PF] = *reinterpret_cast<const s_v4i *>(
                    cur + a_read[((f + PF) / TM) >> 1][((f + PF) / TM) & 1] + ((f + PF) % TM) * 32 * ROWB);
#pragma unroll
            for (int t = 0; t < TN; ++t) {
                const s_v4i bfrag = s_v4i{(int)W8[t][s][4 * hf], (int)W8[t][s][4 * hf + 1], (int)W8[t][s][4 * hf + 2],
                                          (int)W8[t][s][4 * hf + 3]};
                acc[i][t] = epi_mfma<EPI>(bfrag, a, acc[i][t]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // The next tile's panel must have landed (this wave's share; the barrier collects the others') before
        // anyone reads it, and every wave must be done with the current panel before it is requested again.
        // Issue order per tile: residual loads of the next tile, this tile's stores, then the panel RD tiles
        // ahead.  So the loads newer than the next tile's panel are at least the RD - 2 panels after it, and the
        // newest of them came after this wave's latest stores: with a ring of four the wait lets the newest panel
        // and those stores stay in flight (no wait for store acknowledgements) and asks only for things issued
        // a whole tile ago.
        wait_loads(std::integral_constant<int, (RD - 2) * LW>{});
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        load_resid(it + 1, res_next);
        __builtin_amdgcn_sched_barrier(0);

        // ---- epilogue (Eq. 2 / Eq. 8) ----------------------------------------------------------------
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const int nt0 = (nb0 + t) * 32;
            EpiCols<EPI> e;
            if constexpr (EPI == EPI_F32) {
                e.c[0] = my_cols[64 * t + (lane & 31)];
                e.bias[0] = my_cols[64 * t + 32 + (lane & 31)];
            } else {
                const e_v4f *cl = reinterpret_cast<const e_v4f *>(my_cols + 64 * t + 32 * rg);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const e_v4f cc = cl[q], bb = cl[4 + q];
#pragma unroll
                    for (int i = 0; i < 4; ++i) { e.c[4 * q + i] = cc[i]; e.bias[4 * q + i] = bb[i]; }
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
                epi_tile<EPI>(p, acc[i][t], SHIFT, e, m0 + i * 32, rows_of(m0, i), nt0, lane, res[t * TM + i]);
        }
        __builtin_amdgcn_sched_barrier(0);
        load_panel(it + RD);                                 // into the panel this tile has just been read from
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < TM * TN; ++j) res[j] = res_next[j];
    }
}

template <int H, int L>
void launch_nested_gemm_stat(bool full, const GemmParams &p, const StatGeom &g, hipStream_t st, void *ev_start,
                             void *ev_stop)
{
    const dim3 grid((unsigned)(((g.nslots + 7) / 8) * 8 * g.cgroups)), block(256);
    const int mode = epi_mode(p);
#define NQ_ST_LAUNCH(FULLV, EPIV, KSV, WNV)                                                     \
    do {                                                                                        \
        auto k = k_nested_gemm_stat<H, L, FULLV, EPIV, KSV, WNV>;                               \
        const size_t lds = st_lds_bytes(KSV, WNV);                                              \
        static bool granted = false;                                                            \
        if (!granted) {                                                                         \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k),                        \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);    \
            granted = true;                                                                     \
        }                                                                                       \
        launch_timed(k, grid, block, lds, st, ev_start, ev_stop, p, g);                         \
    } while (0)
#define NQ_ST_WN(FULLV, EPIV, KSV)                               \
    do {                                                         \
        if (g.wn == 4) NQ_ST_LAUNCH(FULLV, EPIV, KSV, 4);        \
        else if (g.wn == 2) NQ_ST_LAUNCH(FULLV, EPIV, KSV, 2);   \
        else NQ_ST_LAUNCH(FULLV, EPIV, KSV, 1);                  \
    } while (0)
#define NQ_ST_KS(FULLV, EPIV)                                    \
    do {                                                         \
        if (g.ks == 4) NQ_ST_WN(FULLV, EPIV, 4);                 \
        else if (g.ks == 2) NQ_ST_WN(FULLV, EPIV, 2);            \
        else NQ_ST_WN(FULLV, EPIV, 1);                           \
    } while (0)
#define NQ_ST_MODES(FULLV)                                       \
    do {                                                         \
        if (mode == EPI_ANY) NQ_ST_KS(FULLV, EPI_ANY);           \
        else if (mode == EPI_I8) NQ_ST_KS(FULLV, EPI_I8);        \
        else NQ_ST_KS(FULLV, EPI_F32);                           \
    } while (0)
    if (full && p.low_signed) NQ_ST_MODES(2);
    else if (full) NQ_ST_MODES(1);
    else NQ_ST_MODES(0);
}

}  // namespace nq
