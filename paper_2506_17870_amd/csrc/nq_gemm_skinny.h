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
// blocks (they stay in L2); the block copies them chunk by chunk into LDS with whole-line loads and the
// waves read their fragments there (rows past M through the range check of buffer loads).  Packed
// weights are requested SK_PD K steps ahead in a rolling register pipeline.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_codec.h"
#include "nq_gemm_kernel.h"

namespace nq {

typedef int k_v4i __attribute__((ext_vector_type(4)));
typedef int k_v16i __attribute__((ext_vector_type(16)));


// Barrier of the block that orders LDS accesses only (a __syncthreads would also wait for every global load in
// flight, i.e. drain the weight pipeline).
__device__ __forceinline__ void sk_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Geometry of the activation chunks in LDS: a chunk is what CS consecutive K steps per wave read, i.e. a run
// of 64 * CS * NWS bytes of every row; rows are padded by 16 bytes so that they fall on different banks.
template <int TMS, int NWS>
struct SkinnyChunk {
    static constexpr int CS = (TMS == 1 && NWS == 4) ? 4 : 2;
    static constexpr int SPAN = 64 * CS * NWS;
    static constexpr int RS = SPAN + 16;
    static constexpr int ROWS = 32 * TMS;
    static constexpr int BUF = ROWS * RS + 16;                           // the last 16 bytes take pieces of no row
    static constexpr int PIECES = ROWS * (SPAN / 16);
    static constexpr int NPT = (PIECES + 64 * NWS - 1) / (64 * NWS);     // pieces a thread stages per chunk
};

template <int TMS, int NWS>
constexpr int sk_lds_bytes()
{
    constexpr int chunks = 2 * SkinnyChunk<TMS, NWS>::BUF, sums = (NWS - 1) * TMS * 16 * 64 * 4;
    return chunks > sums ? chunks : sums;
}

// TMS: 32-row tiles (1: M <= 32, 2: M <= 64).  NWS: waves per block (4 or 8).  STAGED: activations through
// LDS (long reductions), else straight from memory into the lanes' fragments (short ones, where the extra
// hop would only add to a latency-bound kernel).
// The work of one block: column tile nb of the problem p.  lds: the block's dynamic LDS.
template <int H, int L, int FULL, int EPI, int TMS, int NWS, bool STAGED>
__device__ __forceinline__ void skinny_block(const GemmParams &p, const int nb, uint8_t *lds)
{
    constexpr int S = 8 - H;
    constexpr int SHIFT = FULL ? (8 - H - L) : S;
    using LP = LowPage<L, S, FULL>;
    using CH = SkinnyChunk<TMS, NWS>;
    constexpr int SK_PD = 4;       // K steps of packed weights in flight per wave
    constexpr int CS = CH::CS, RS = CH::RS, NPT = CH::NPT;

    // lds: two activation chunks; the partial sums of the waves use the same memory at the end (sk_lds_bytes)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wslot = epi_weight_slot<EPI>(lane);

    // Activations go through LDS: fetched straight from memory, a step's fragments are one cache line per lane
    // and the look-ups, not the bytes, are what a compute unit runs out of (at 64 rows they cost more than the
    // weight stream).  The block copies a run of every row per chunk with whole-line loads instead; rows past
    // M and steps past K are out of the buffer's range and read as zero.
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(p.x), 0,
                                                                           (int)(p.M * p.K), 0x00020000);
    constexpr uint32_t NOWHERE = 0x7fff0000u;
    uint32_t st_x[NPT];     // byte offset of the piece in the activations for chunk 0
    int st_lds[NPT];        // where it goes in a buffer
    int st_k[NPT];          // its first k in chunk 0
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        const int q = tid + 64 * NWS * i;
        const int r = q / (CH::SPAN / 16), pc = q - r * (CH::SPAN / 16);
        const bool real = q < CH::PIECES && r < p.M;
        st_x[i] = real ? (uint32_t)(r * p.K + 16 * pc) : NOWHERE;
        st_lds[i] = q < CH::PIECES ? r * RS + 16 * pc : CH::ROWS * RS;
        st_k[i] = 16 * pc;
    }
    k_v4i stage[NPT];
    const int k_end = p.KB * 64;         // weights past K are zero fields up to here; nothing is read beyond
    auto stage_load = [&](int c) {
#pragma unroll
        for (int i = 0; i < NPT; ++i) {
            const int k = st_k[i] + c * CH::SPAN;
            const uint32_t at = (st_x[i] != NOWHERE && k < k_end) ? st_x[i] + (uint32_t)(c * CH::SPAN) : NOWHERE;
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, at, 0, 0);
            stage[i] = k_v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
        }
    };
    // the lane's fragments of local K step s of a chunk: row lane & 31 (+ 32 per tile), bytes
    // [64*(wave + NWS*s) + 32*g + 16*hf, +16) of the run
    const int a_lds = (lane & 31) * RS + 64 * wave + 32 * (lane >> 5);

    // not STAGED: row = lane & 31 (+ 32 per tile), bytes [64*kb + 32*g + 16*hf, +16) of the row, requested with
    // the weights of the step
    int a_row[TMS];
#pragma unroll
    for (int i = 0; i < TMS; ++i) a_row[i] = (32 * i + (lane & 31)) * p.K + 32 * (lane >> 5);
    k_v4i A[STAGED ? 1 : SK_PD][TMS][2];

    uint32_t P[SK_PD][H];
    uint32_t Q[SK_PD][LP::ARR];
    const int64_t tile0 = (int64_t)nb * p.KB;
    // K steps past the end are requested like the last real one; their activations are zero
    auto request = [&](int slot, int kb) {
        const int kbc = min(kb, p.KB - 1);
        const uint32_t *src = p.ph + (tile0 + kbc) * (H * 64);
#pragma unroll
        for (int i = 0; i < H; ++i) P[slot][i] = src[(unsigned)(wslot * H + i)];
        if constexpr (FULL != 0) {
            const uint32_t *srcl = p.pl + (tile0 + kbc) * (LP::DW * 64);
#pragma unroll
            for (int i = 0; i < LP::DW; ++i) Q[slot][i] = srcl[(unsigned)(wslot * LP::DW + i)];
        }
        if constexpr (!STAGED) {
            const int koff = kb < p.KB ? 64 * kb : 0x7fff0000;
#pragma unroll
            for (int i = 0; i < TMS; ++i)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const auto v = __builtin_amdgcn_raw_buffer_load_b128(xrsrc, a_row[i] + koff + 16 * hf, 0, 0);
                    A[slot][i][hf] = k_v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
                }
        }
    };

    k_v16i acc[TMS];
#pragma unroll
    for (int i = 0; i < TMS; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;

    if constexpr (STAGED) stage_load(0);
#pragma unroll
    for (int d = 0; d < SK_PD; ++d) request(d, wave + NWS * d);

    // wave w: K steps w + NWS*j; all waves run the same number of rounds (the extra ones add zeros) and meet
    // at one barrier per chunk
    const int rounds = (p.KB + NWS - 1) / NWS;
    for (int j0 = 0; j0 < rounds; j0 += SK_PD) {
#pragma unroll
        for (int d = 0; d < SK_PD; ++d) {
            const int c = (j0 + d) / CS;           // chunk of this step
            if (STAGED && d % CS == 0) {
                // The buffer was last read two chunks ago, and every wave has passed the barrier of the chunk
                // in between since.
                uint8_t *buf = lds + (c & 1) * CH::BUF;
#pragma unroll
                for (int i = 0; i < NPT; ++i) *reinterpret_cast<k_v4i *>(buf + st_lds[i]) = stage[i];
                stage_load(c + 1);                  // travels while this chunk is computed
                sk_lds_barrier();
            }
            const uint8_t *frag = lds + (c & 1) * CH::BUF + a_lds + 64 * NWS * (d % CS);
            uint32_t D[8];
            HighCodec<H>::decode(P[d], D);
            LP::apply(Q[d], D);
            k_v4i a[TMS][2];
#pragma unroll
            for (int i = 0; i < TMS; ++i)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    if constexpr (STAGED) a[i][hf] = *reinterpret_cast<const k_v4i *>(frag + 32 * i * RS + 16 * hf);
                    else a[i][hf] = A[d][i][hf];
                }
            request(d, wave + NWS * (j0 + d + SK_PD));
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const k_v4i b = k_v4i{(int)D[4 * hf], (int)D[4 * hf + 1], (int)D[4 * hf + 2], (int)D[4 * hf + 3]};
#pragma unroll
                for (int i = 0; i < TMS; ++i) acc[i] = epi_mfma<EPI>(b, a[i][hf], acc[i]);
            }
        }
    }
    if constexpr (STAGED) sk_lds_barrier();       // the chunk buffers are free for the partial sums

    // ---- add the partial sums of the waves -----------------------------------------------------------
    int *red = reinterpret_cast<int *>(lds);          // [NWS - 1][TMS][16][64]
    if (wave > 0) {
        int *mine = red + (wave - 1) * (TMS * 16 * 64) + lane;       // constant offsets from one address
#pragma unroll
        for (int i = 0; i < TMS; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[(i * 16 + r) * 64] = acc[i][r];
    }
    __syncthreads();
    if (wave > 0) return;
    const int *all = red + lane;
#pragma unroll
    for (int w = 0; w < NWS - 1; ++w)
#pragma unroll
        for (int i = 0; i < TMS; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] += all[((w * TMS + i) * 16 + r) * 64];

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

template <int H, int L, int FULL, int EPI, int TMS, int NWS, bool STAGED>
__global__ void __launch_bounds__(64 * NWS, NWS == 4 ? 2 : 1) k_nested_gemm_skinny(const GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    skinny_block<H, L, FULL, EPI, TMS, NWS, STAGED>(p, blockIdx.x, lds);
}

// Many small layers in one launch (the weights of a stack of layers are the traffic, and a launch per layer
// of a few blocks each is launch bound): the problems wait as a table in device memory, `first` holds the
// running count of their blocks, and a block finds its problem by binary search (everything uniform, so the
// search and the copy of the problem's parameters run on the scalar unit).
template <int H, int L, int FULL, int EPI, int TMS, bool STAGED>
__global__ void __launch_bounds__(256, 2) k_nested_gemm_skinny_batch(const GemmParams *__restrict__ jobs,
                                                                      const int *__restrict__ first, const int count)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int b = blockIdx.x;
    int lo = 0, hi = count - 1;                  // the last job with first[job] <= b
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (first[mid] <= b) lo = mid; else hi = mid - 1;
    }
    const GemmParams p = jobs[lo];
    skinny_block<H, L, FULL, EPI, TMS, 4, STAGED>(p, b - first[lo], lds);
}

// Launches the batch kernel: one instantiation for the whole table (mode: epilogue layout shared by all
// problems; two_tiles: some problem has more than 32 rows; staged: some reduction is 2048 or longer).
template <int H, int L>
void launch_nested_gemm_skinny_batch(int fmode, int mode, bool two_tiles, bool staged, const GemmParams *d_jobs,
                                     const int *d_first, int count, int blocks, hipStream_t st, void *ev_start,
                                     void *ev_stop)
{
#define NQ_SKB_ONE(FULLV, EPIV, TMSV, STAGEDV)                                                          \
    do {                                                                                                \
        auto k = k_nested_gemm_skinny_batch<H, L, FULLV, EPIV, TMSV, STAGEDV>;                           \
        constexpr int lds = STAGEDV ? sk_lds_bytes<TMSV, 4>() : 3 * TMSV * 4096;                         \
        static bool granted = false;                                                                    \
        if (!granted) {                                                                                 \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k),                                \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds);                 \
            granted = true;                                                                             \
        }                                                                                               \
        launch_timed(k, dim3((unsigned)blocks), dim3(256), lds, st, ev_start, ev_stop, d_jobs, d_first, count); \
    } while (0)
#define NQ_SKB_SHAPE(FULLV, EPIV)                                        \
    do {                                                                 \
        if (two_tiles && staged) NQ_SKB_ONE(FULLV, EPIV, 2, true);       \
        else if (two_tiles) NQ_SKB_ONE(FULLV, EPIV, 2, false);           \
        else if (staged) NQ_SKB_ONE(FULLV, EPIV, 1, true);               \
        else NQ_SKB_ONE(FULLV, EPIV, 1, false);                          \
    } while (0)
#define NQ_SKB_MODES(FULLV)                                      \
    do {                                                         \
        if (mode == EPI_I8) NQ_SKB_SHAPE(FULLV, EPI_I8);         \
        else NQ_SKB_SHAPE(FULLV, EPI_F32);                       \
    } while (0)
    if (fmode == 2) NQ_SKB_MODES(2); else if (fmode == 1) NQ_SKB_MODES(1); else NQ_SKB_MODES(0);
}

template <int H, int L>
void launch_nested_gemm_skinny(bool full, const GemmParams &p, hipStream_t st, void *ev_start, void *ev_stop)
{
    const dim3 grid((unsigned)p.NB);
    const int mode = epi_mode(p);
    // eight waves where every compute unit gets at most one block, the reduction is long enough to share and
    // there is one row tile (with two, measured slower: 25.8 us against 23.1 us at 64 x 8192 -> 8192)
    const bool wide = p.NB <= 256 && p.KB >= 32 && p.M <= 32;
    // activations through LDS from 2048 columns on (a 64 x 512 x 512 layer: 4.4 us straight, 4.8 us staged)
    const bool staged = p.KB >= 32;
#define NQ_SK_ONE(FULLV, EPIV, TMSV, NWSV, STAGEDV)                                                     \
    do {                                                                                                \
        auto k = k_nested_gemm_skinny<H, L, FULLV, EPIV, TMSV, NWSV, STAGEDV>;                           \
        constexpr int lds = STAGEDV ? sk_lds_bytes<TMSV, NWSV>() : (NWSV - 1) * TMSV * 4096;             \
        static bool granted = false;   /* one per kernel instantiation */                               \
        if (!granted) {                                                                                 \
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k),                                \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds);                 \
            granted = true;                                                                             \
        }                                                                                               \
        launch_timed(k, grid, dim3(64 * NWSV), lds, st, ev_start, ev_stop, p);                          \
    } while (0)
#define NQ_SK_LAUNCH(FULLV, EPIV)                                       \
    do {                                                                \
        if (wide) NQ_SK_ONE(FULLV, EPIV, 1, 8, true);                   \
        else if (p.M <= 32 && staged) NQ_SK_ONE(FULLV, EPIV, 1, 4, true); \
        else if (p.M <= 32) NQ_SK_ONE(FULLV, EPIV, 1, 4, false);        \
        else if (staged) NQ_SK_ONE(FULLV, EPIV, 2, 4, true);            \
        else NQ_SK_ONE(FULLV, EPIV, 2, 4, false);                       \
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
