// Kernel arguments of the nested GEMM / convolution and the launcher that every
// (h, l) translation unit instantiates.  Internal to libnq.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nq {

struct GemmParams {
    const int8_t *x;
    const uint32_t *ph;
    const uint32_t *pl;
    const float *scale;
    void *y;
    const float *bias;
    const int8_t *resid;
    int32_t *acc_dump;
    int64_t M;
    int N, K, KB, NB;
    // geometry of the implicit GEMM; a plain GEMM is H = W = Ho = Wo = KH = KW = 1, Cin = K
    int H, W, Cin, Ho, Wo, KH, KW, stride, pad;
    float act_scale, resid_scale, inv_out_scale, part_mul;
    int relu, out_int8, fast_a;
    int low_signed;   // lower-bit page holds signed fields of l + 1 bits (compensated format)
    int general;   // 1: the element-wise epilogue is needed (set by the host from the arguments)
    // implicit GEMM of the large-GEMM kernel: Cin = 2^cin_shift, tap / KW = (tap * kw_magic) >> 16
    int conv_big, cin_shift, kw_magic;
};

// Geometry of the LDS-resident input window of the windowed convolution kernel.
struct WindowGeom {
    int R;          // output rows per block
    int RB;         // row blocks per image = ceil(Ho / R)
    int IR;         // input rows in the window = (R-1)*stride + KH
    int WC;         // window columns = W + 2*pad
    int CK;         // input channels per chunk (64, 128 or 256)
    int NCH;        // chunks = Cin / CK
    int c16_shift;  // log2(CK / 16)
};

// Geometry of the register-stationary-weights convolution kernel (work unit = R output rows).
// Everything that does not depend on the data is worked out on the host.
struct StreamGeom {
    int R;            // output rows per unit (R * Wo <= 128)
    int RB;           // units per image = ceil(Ho / R)
    int WC;           // window columns = W + 2*pad
    int units;        // B * RB
    int ksteps;       // KH*KW*Cin / 64: 1, 2, 4, 8 or 9
    int items;        // 16-byte pieces of one window = IR * WC * Cin / 16
    int win_bytes;    // bytes of one LDS window = IR * WC * (Cin + 16)
    int win_stride;   // win_bytes + 16: one spare slot for pieces past the window
    int c16_shift;    // log2(Cin / 16)
    unsigned wc_magic;  // ceil(2^32 / WC): n / WC == umulhi(n, wc_magic) for n < 2^16
    unsigned wo_magic;  // ceil(2^32 / Wo)
    int grid_x, nblk;     // unit slots (a block takes units slot, slot + grid_x, ...) and channel-tile groups
    int step_b, step_rb;  // grid_x = step_b * RB + step_rb: how (image, row block) advance per unit
    int img_bytes;    // H * W * Cin
    int row_bytes;    // W * Cin
    int tap_off[9];   // LDS byte offset of K step s: (kh*WC + kw)*(Cin+16) + 64*cb
};

// 32-channel tiles per block of the register-stationary kernel, by K steps of the layer.
inline int rs_channel_tiles(int ksteps) { return ksteps <= 2 ? 4 : (ksteps == 4 ? 2 : 1); }

// Geometry of the few-input-channels convolution kernel (work unit = R output rows of one image).
struct SmallCinGeom {
    int R;            // output rows per unit
    int RB;           // units per image = ceil(Ho / R)
    int units;        // B * RB
    int IR;           // input rows of a unit = (R-1)*stride + KH
    int seg;          // KW * Cin: bytes of one filter row (<= 32)
    int d0;           // byte offset of input column 0 inside an LDS row (zero halo before it), multiple of 4
    int row_stride;   // LDS bytes per input row, multiple of 4
    int row_dwords;   // W * Cin / 4
    int row_bytes;    // W * Cin
    int img_bytes;    // H * W * Cin
    int win_bytes;    // LDS bytes of one window incl. slack, multiple of 16
    int grid_x;       // persistent blocks per channel group
};

// Geometry of the depthwise / grouped convolution kernel (work unit = patch of R x CW output pixels of
// one image).
struct GroupGeom {
    int gs;           // channels per group (1, 2 or 4), inputs and outputs alike
    int taps;         // KH * KW (<= 28)
    int CT;           // 64-channel tiles = ceil(C / 64)
    int R, CW;        // output rows and columns of a patch
    int RB, CB;       // patches per image: ceil(Ho / R) x ceil(Wo / CW)
    int IRp, ICp;     // input rows and columns of a patch: (R-1)*stride + KH, (CW-1)*stride + KW
    int units;        // B * RB * CB
    int ptiles;       // 16-pixel tiles of a patch = ceil(R * CW / 16)
    int np;           // 16-byte pieces a thread stages per window = ceil(IRp * ICp * 4 / 256) (<= 10)
    int cw_magic;     // 2^20 / CW + 1: n / CW == (n * cw_magic) >> 20 for n < 4096
    int icp_magic;    // 2^20 / ICp + 1, likewise for window pixels
    int step_b, step_rb, step_cb;   // grid_x = (step_b * RB + step_rb) * CB + step_cb: how a unit advances
    int zero_off;     // LDS offset of 64 zero bytes (behind the window of IRp * ICp pixels of 80 bytes)
    int lds_bytes;    // dynamic LDS of the kernel
    int grid_x;       // persistent blocks per channel tile
    int64_t x_bytes;  // B * H * W * C (< 2^31)
};

// Geometry of the stationary-weights GEMM (1x1 convolutions with 64, 128 or 256 input channels at any stride,
// GEMMs with that K): persistent blocks, each a column group of 64 * wn columns and a slot of row tiles.
struct StatGeom {
    int ks;            // K steps of 64: 1, 2 or 4
    int wn;            // waves along N: 4, 2 or 1 (256, 128 or 64 columns per block)
    int rps;           // rows per slot: a block takes the rows [slot * rps, (slot + 1) * rps), tile by tile
    int nslots;        // slots = ceil(M / rps)
    int cgroups;       // column groups = ceil(N / (64 * wn))
    int interleave;    // 1: a block takes the tiles slot, slot + nslots, ... instead of a run of rps rows
    int strided;       // 1: row m is pixel (oh * stride, ow * stride) of its image (strided 1x1 convolution)
    int howo;          // Ho * Wo
    unsigned howo_magic, wo_magic;   // ceil(2^32 / d): n / d == umulhi(n, magic) as long as n * d < 2^32; 0 for d = 1
    int img_bytes;     // H * W * Cin
    int row_step;      // stride * W * Cin: input bytes from one output row to the next
    int col_step;      // stride * Cin
    int x_bytes;       // bytes of the whole input (< 2^31 - 2^16)
};

// Block tile of the stationary-weights GEMM: waves side by side along N (wn of them, 64 columns each), the
// rest stacked along M with one or two 32-row tiles each; panels of the ring (as many as fit, up to four); dynamic
// LDS of the kernel.
constexpr int st_tm(int wn) { return wn == 4 ? 2 : 1; }
constexpr int st_bm(int wn) { return (4 / wn) * 32 * st_tm(wn); }
constexpr int st_ring(int ks, int wn)
{
    const int panel = st_bm(wn) * 64 * ks;
    return 4 * panel <= 56 * 1024 ? 4 : (3 * panel <= 56 * 1024 ? 3 : 2);
}
// bytes of the residual staging area: one KB per 32 x 32 tile of every wave
constexpr int st_resid_bytes(int wn) { return 4 * st_tm(wn) * 2 * 1024; }
constexpr size_t st_lds_bytes(int ks, int wn)
{
    return (size_t)st_ring(ks, wn) * st_bm(wn) * 64 * ks + 1024 /* dump */ + 4 * 2 * 64 * sizeof(float) /* constants */ +
           st_resid_bytes(wn);
}

// Tile shapes: 0 = 256x64 (narrow outputs), 1 = 128x256 (large), 2 = 64x256 (few rows).
constexpr int NQ_TILE_BM[3] = {256, 128, 64};
constexpr int NQ_TILE_BN[3] = {64, 256, 256};

// Defined in nq_gemm_kernel.h, instantiated once per (h, l) by nq_gemm_inst.hip.
// ev_start / ev_stop, if not null, are hipEvent_t that receive the begin and end time stamps
// of the kernel itself.
template <int H, int L>
void launch_nested_gemm(bool full, int tile, const GemmParams &p, hipStream_t st, void *ev_start, void *ev_stop);

// Windowed convolution, shape 0: 2x2 waves, 8 row tiles x 64 channels per block.
template <int H, int L>
void launch_nested_conv_window(bool full, int shape, const GemmParams &p, const WindowGeom &g, size_t lds_bytes,
                               hipStream_t st, void *ev_start, void *ev_stop);

// Register-stationary weights, persistent blocks over row units; 64 output channels per block.
template <int H, int L>
void launch_nested_conv_rowstream(bool full, const GemmParams &p, const StreamGeom &g, int grid_x, hipStream_t st,
                                  void *ev_start, void *ev_stop);

// Few input channels (KW * Cin <= 32): one matrix-core step per filter row.
template <int H, int L>
void launch_nested_conv_smallcin(bool full, const GemmParams &p, const SmallCinGeom &g, hipStream_t st, void *ev_start,
                                 void *ev_stop);

// Depthwise / grouped convolution with 1, 2 or 4 channels per group.
template <int H, int L>
void launch_nested_conv_grouped(bool full, const GemmParams &p, const GroupGeom &g, hipStream_t st, void *ev_start,
                                void *ev_stop);

// Grouped convolution with groups of any width and unequal channel counts (direct, on the vector ALU).
template <int H, int L>
void launch_nested_conv_grouped_any(bool full, const GemmParams &p, int gs_in, int gs_out, int quads, hipStream_t st,
                                    void *ev_start, void *ev_stop);

// Few rows (M <= 64): one block per 32-column tile, the waves split K.
template <int H, int L>
void launch_nested_gemm_skinny(bool full, const GemmParams &p, hipStream_t st, void *ev_start, void *ev_stop);

// Many few-row problems in one launch: d_jobs / d_first are the table in device memory (count problems, the
// running count of their blocks), fmode 0 part-bit, 1 full-bit, 2 full-bit compensated; mode EPI_F32 or EPI_I8.
template <int H, int L>
void launch_nested_gemm_skinny_batch(int fmode, int mode, bool two_tiles, bool staged, const GemmParams *d_jobs,
                                     const int *d_first, int count, int blocks, hipStream_t st, void *ev_start,
                                     void *ev_stop);

// Large GEMM / 1x1 stride-1 convolution: 128 x 256 tiles, K advanced 256 per barrier.
// tm_forced: 2..5 forces the rows per block (32 * tm), anything else leaves the choice to the launcher;
// tm_used, if not null, receives the height that was launched.
template <int H, int L>
void launch_nested_gemm_big(bool full, const GemmParams &p, int tm_forced, int *tm_used, hipStream_t st,
                            void *ev_start, void *ev_stop);

// Short reductions (K = 64, 128, 256): weights stationary in registers, persistent blocks over row tiles.
template <int H, int L>
void launch_nested_gemm_stat(bool full, const GemmParams &p, const StatGeom &g, hipStream_t st, void *ev_start,
                             void *ev_stop);

// GEMM over the paper's word pages (64 / k fields per 64-bit word); WH, WL: words per row of the two pages.
// Not a template: nq_gemm_words.hip holds every nesting.
void launch_nested_gemm_words(bool full, int h, int l, const GemmParams &p, int WH, int WL, hipStream_t st,
                              void *ev_start, void *ev_stop);

}  // namespace nq
