// Host side of the inference entry points: argument checks, residency of the lower-bit
// page (paper Sec. 3.2.3 / 3.3: the caller picks full-bit or part-bit; a paged-out page is
// an error, never a silent downgrade), tile choice and launch.
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "nq_common.h"
#include "nq_gemm_params.h"

using namespace nq;

namespace {

struct Geometry {
    int64_t M;
    int H, W, Cin, Ho, Wo, KH, KW, stride, pad;
};

// One-shot profiling hook: events handed over by nq_profile_next_launch, consumed by the next launch.
thread_local void *g_ev_start = nullptr;
thread_local void *g_ev_stop = nullptr;

// Test and tuning overrides set through nq_set_tuning; 0 = the library's own choice.
std::atomic<int> g_tune[NQ_TUNE_COUNT];

// What the last launch of this thread ran (nq_profile_last_kernel): kernel family as in NQ_TUNE_KERNEL
// (7 = depthwise / grouped, 8 = word pages, 9 = stationary-weights GEMM) and, for the large-GEMM kernel, its tile height.
thread_local int g_last_family = 0;
thread_local int g_last_variant = 0;

// Decides whether the windowed convolution kernel applies and fills its geometry.
bool plan_window(const Geometry &g, const int8_t *d_x, WindowGeom *wg, size_t *lds)
{
    if (g.KH * g.KW <= 1) return false;
    if (g.Cin % 64 != 0 || !aligned16(d_x)) return false;
    if (g.Wo > 256 || g.Wo < 1) return false;
    const int WC = g.W + 2 * g.pad;
    for (int CK : {256, 128, 64}) {
        if (g.Cin % CK != 0) continue;
        int R = 256 / g.Wo;                       // at most eight 32-row tiles per block
        if (R > g.Ho) R = g.Ho;
        for (; R >= 1; --R) {
            const int IR = (R - 1) * g.stride + g.KH;
            const size_t bytes = (size_t)IR * WC * (CK + 16);
            if (bytes <= 72 * 1024) {
                // do not shrink the block below half of its row budget just to widen the chunk
                if (R * g.Wo < 128 && CK > 64 && 256 / g.Wo > R) break;
                wg->R = R; wg->RB = (g.Ho + R - 1) / R; wg->IR = IR; wg->WC = WC; wg->CK = CK;
                wg->NCH = g.Cin / CK;
                wg->c16_shift = CK == 256 ? 4 : (CK == 128 ? 3 : 2);
                *lds = bytes;
                return true;
            }
        }
    }
    return false;
}

// Decides whether the register-stationary-weights kernel applies (short K, power-of-two Cin)
// and works out its geometry.
bool plan_rowstream(const Geometry &g, const int8_t *d_x, int64_t n_out, StreamGeom *sg, int *grid_x)
{
    const int Cin = g.Cin;
    if (Cin < 64 || (Cin & (Cin - 1)) != 0 || !aligned16(d_x)) return false;
    const int ksteps = g.KH * g.KW * (Cin / 64);
    if (ksteps != 9 && ksteps != 1 && ksteps != 2 && ksteps != 4 && ksteps != 8) return false;
    if (g.Wo > 128 || g.Wo < 1) return false;
    const int64_t img_bytes = (int64_t)g.H * g.W * Cin;
    if (img_bytes > (int64_t(1) << 29)) return false;
    const int WC = g.W + 2 * g.pad;
    const int ld_max = (ksteps == 9 || ksteps == 1) ? 4 : 8;   // window pieces per thread of that instantiation
    int R = 128 / g.Wo;
    if (R > g.Ho) R = g.Ho;
    for (; R >= 1; --R) {
        const int IR = (R - 1) * g.stride + g.KH;
        const int64_t items = (int64_t)IR * WC * (Cin / 16);
        const int64_t bytes = (int64_t)IR * WC * (Cin + 16);
        if (items > ld_max * 256 || 4 * (bytes + 16) > 75 * 1024) continue;
        if (R * g.Wo < 64 && 128 / g.Wo > R) return false;   // the window limit left too little work per unit
        const int64_t images = g.M / ((int64_t)g.Ho * g.Wo);
        const int RB = (g.Ho + R - 1) / R;
        if (images * RB > 0x3fffffffLL) return false;
        sg->R = R; sg->RB = RB; sg->WC = WC; sg->units = (int)(images * RB);
        sg->ksteps = ksteps; sg->items = (int)items; sg->win_bytes = (int)bytes; sg->win_stride = (int)bytes + 16;
        int sh = 0;
        while ((16 << sh) < Cin) ++sh;
        sg->c16_shift = sh;
        sg->wc_magic = (unsigned)(((uint64_t(1) << 32) + WC - 1) / WC);
        sg->wo_magic = (unsigned)(((uint64_t(1) << 32) + g.Wo - 1) / g.Wo);
        if (WC == 1) sg->wc_magic = 0xFFFFFFFFu;   // not reached: WC >= KW >= 1 and a 1-wide window has Cin pieces only
        sg->img_bytes = (int)img_bytes; sg->row_bytes = g.W * Cin;
        const int cin64 = Cin / 64;
        for (int s = 0; s < 9; ++s) {
            const int tap = s / cin64, cb = s % cin64;
            const int kh = tap / g.KW, kw = tap % g.KW;
            sg->tap_off[s] = s < ksteps ? (kh * WC + kw) * (Cin + 16) + cb * 64 : 0;
        }
        // persistent blocks, two per compute unit (LDS windows), each with the same number of units
        // channel-tile groups: a block keeps the weights of rs_channel_tiles() tiles
        const int nblk = (int)ceil_div(ceil_div(n_out, 32), rs_channel_tiles(ksteps));
        int slots = 512 / nblk;
        if (slots < 1) slots = 1;
        // every slot is used: with 3.5 units per slot the first half of the blocks (dispatched first, one
        // per compute unit) gets four units and the second half three, instead of fewer blocks of four
        *grid_x = sg->units < slots ? sg->units : slots;
        sg->step_b = *grid_x / RB; sg->step_rb = *grid_x % RB;
        sg->grid_x = *grid_x; sg->nblk = nblk;
        return true;
    }
    return false;
}

// Decides whether the few-input-channels kernel applies (a filter row is at most 32 bytes of the
// NHWC input) and works out its geometry.
bool plan_smallcin(const Geometry &g, const int8_t *d_x, int64_t n_out, SmallCinGeom *sg)
{
    const int seg = g.KW * g.Cin;
    if (seg > 32 || g.Cin >= 16 || (g.KH != 7 && g.KH != 3)) return false;
    const int row_bytes = g.W * g.Cin;
    if (row_bytes % 4 != 0 || ((uintptr_t)d_x & 3) != 0) return false;
    const int64_t img_bytes = (int64_t)g.H * row_bytes;
    if (img_bytes > (int64_t(1) << 29)) return false;
    const int64_t images = g.M / ((int64_t)g.Ho * g.Wo);
    // pixels to the right of the image that the last output column still reaches
    const int over = (g.Wo - 1) * g.stride - g.pad + g.KW - 1 - (g.W - 1);
    const int halo = g.pad > over ? g.pad : over;
    const int d0 = (halo * g.Cin + 3) / 4 * 4;
    const int row_stride = (d0 + row_bytes + 3) / 4 * 4;
    const int row_dwords = row_bytes / 4;
    const int64_t kb = ceil_div((int64_t)g.KH * seg, 64);
    for (int R = g.Ho; R >= 1; --R) {
        const int IR = (R - 1) * g.stride + g.KH;
        if ((int64_t)IR * row_dwords > 256 * 8) continue;          // dwords a block stages per window
        const int64_t win = ((int64_t)IR * row_stride + 128 + 15) / 16 * 16;   // slack: fragments of the last row read past it
        if (2 * win + 2 * 32 * kb * 64 + 512 > 72 * 1024) continue;   // two blocks per compute unit
        if (images * ceil_div(g.Ho, R) > 0x3fffffffLL) return false;
        sg->R = R; sg->RB = (int)ceil_div(g.Ho, R); sg->units = (int)(images * sg->RB);
        sg->IR = IR; sg->seg = seg; sg->d0 = d0; sg->row_stride = row_stride; sg->row_dwords = row_dwords;
        sg->row_bytes = row_bytes; sg->img_bytes = (int)img_bytes; sg->win_bytes = (int)win;
        const int64_t groups = ceil_div(ceil_div(n_out, 32), 2);
        if (groups > 65535) return false;
        int64_t gx = 512 / groups;
        if (gx < 1) gx = 1;
        sg->grid_x = (int)(gx < sg->units ? gx : sg->units);
        return sg->units > 0;
    }
    return false;
}

// Patch shape of the depthwise / grouped kernel: the window of a patch must fit the registers that stage
// it (640 pixels of 64 bytes); among the shapes that do, the one that fetches the fewest halo pixels per
// output, fills its 16-pixel tiles and still leaves enough units for the whole GPU.
bool plan_grouped(const Geometry &g, int gs, int64_t C, GroupGeom *gg)
{
    const int64_t images = g.M / ((int64_t)g.Ho * g.Wo);
    const int CT = (int)ceil_div(C, 64);
    double best = -1.0;
    int bR = 0, bCW = 0;
    const int tuned_units = g_tune[NQ_TUNE_GC_UNITS].load(std::memory_order_relaxed);
    const double units_target = tuned_units > 0 ? (double)tuned_units : 512.0;
    const int cands[5] = {g.Wo, (g.Wo + 1) / 2, (g.Wo + 2) / 3, (g.Wo + 3) / 4, 16};
    for (int CW : cands) {
        if (CW > g.Wo) CW = g.Wo;
        if (CW < 1 || CW > 255) continue;
        const int ICp = (CW - 1) * g.stride + g.KW;
        for (int R = g.Ho; R >= 1; --R) {
            const int IRp = (R - 1) * g.stride + g.KH;
            if ((int64_t)IRp * ICp > 640 || R * CW > 4000) continue;
            const double halo = (double)R * CW * g.stride * g.stride / ((double)IRp * ICp);
            const double fill = (double)R * CW / (16.0 * (double)ceil_div(R * CW, 16));
            const double units = (double)images * (double)ceil_div(g.Ho, R) * (double)ceil_div(g.Wo, CW) * CT;
            const int64_t pt = ceil_div(R * CW, 16);
            const double balance = (double)pt / (4.0 * (double)ceil_div(pt, 4));   // tiles are dealt to four waves
            // how many (unit, channel tile) pairs a launch should at least have: measured best at one per
            // resident block, larger patches beating more of them (NQ_TUNE_GC_UNITS overrides)
            const double target = units_target;
            const double score = halo * fill * balance * (units >= target ? 1.0 : units / target);
            if (score > best) { best = score; bR = R; bCW = CW; }
        }
    }
    if (best < 0.0) return false;
    gg->gs = gs;
    gg->taps = g.KH * g.KW;
    gg->CT = CT;
    gg->R = bR; gg->CW = bCW;
    gg->RB = (int)ceil_div(g.Ho, bR); gg->CB = (int)ceil_div(g.Wo, bCW);
    gg->IRp = (bR - 1) * g.stride + g.KH; gg->ICp = (bCW - 1) * g.stride + g.KW;
    const int64_t units = images * gg->RB * gg->CB;
    if (units > 0x3fffffffLL) return false;
    gg->units = (int)units;
    gg->ptiles = (int)ceil_div(bR * bCW, 16);
    gg->np = (int)ceil_div((int64_t)gg->IRp * gg->ICp * 4, 256);
    gg->cw_magic = (1 << 20) / bCW + 1;
    gg->icp_magic = (1 << 20) / gg->ICp + 1;
    gg->zero_off = gg->IRp * gg->ICp * 80;
    // the decoded weights (8 KiB) and the fragment table (up to 28 KiB) pass through the same memory first
    const int setup_bytes = 8192 + (gg->taps <= 12 ? 3 : 7) * 4096;
    gg->lds_bytes = gg->zero_off + 64 < setup_bytes ? setup_bytes : gg->zero_off + 64;
    gg->x_bytes = images * g.H * g.W * C;
    // two resident blocks per compute unit, never more blocks than there are units
    int64_t gx = ceil_div(512, CT);
    if (gx > units) gx = units;
    gg->grid_x = (int)(gx < 1 ? 1 : gx);
    gg->step_cb = gg->grid_x % gg->CB;
    gg->step_rb = (gg->grid_x / gg->CB) % gg->RB;
    gg->step_b = gg->grid_x / (gg->CB * gg->RB);
    return true;
}

// Decides whether the stationary-weights GEMM applies (1x1 filter without padding, K = 64, 128 or 256) and
// works out its geometry.
bool plan_stat(const Geometry &g, const int8_t *d_x, int64_t N, int64_t K, StatGeom *sg)
{
    if (g.KH != 1 || g.KW != 1 || g.pad != 0 || g.Cin != K) return false;
    if (K != 64 && K != 128 && K != 256) return false;
    if (!aligned16(d_x) || N < 1) return false;
    const int64_t howo = (int64_t)g.Ho * g.Wo;
    const int64_t images = g.M / howo;
    const int64_t x_bytes = images * g.H * g.W * g.Cin;
    if (x_bytes >= 0x7fff0000LL - 65536 || g.M >= (int64_t(1) << 31) - 512) return false;
    if (g.M * N >= 0x7fff0000LL - 65536) return false;      // int8 outputs and residual codes: 32-bit byte offsets
    const bool strided = g.stride > 1;
    // the divisions by Ho * Wo and by Wo are multiplications by a rounded-up reciprocal: exact while
    // dividend * divisor < 2^32 (dividends: a row index inside an image plus one tile; a pixel index)
    if (strided && ((howo + 256) * howo >= (int64_t(1) << 32) || howo * g.Wo >= (int64_t(1) << 32))) return false;
    sg->ks = (int)(K / 64);
    sg->wn = N <= 64 ? 1 : (N <= 128 ? 2 : 4);
    sg->cgroups = (int)ceil_div(N, 64 * sg->wn);
    if (sg->cgroups > 0x3fffff) return false;
    // persistent blocks, two per compute unit; whole groups of eight slots (one per XCD) where there are that
    // many; every slot the same number of rows, at least one 32-row tile
    int64_t nslots = 512 / sg->cgroups;
    if (nslots < 1) nslots = 1;
    if (nslots >= 8) nslots -= nslots % 8;
    if (nslots > ceil_div(g.M, 32)) nslots = ceil_div(g.M, 32);
    // Row tiles are dealt to the blocks in turn (tile t to slot t % nslots): the blocks then stream one region of
    // the tensors together, which measured 7-10 % faster than giving every block one run of consecutive rows
    // (NQ_TUNE_STAT_ROWS = 1), although the runs are the more even split.
    sg->interleave = g_tune[NQ_TUNE_STAT_ROWS].load(std::memory_order_relaxed) != 1;
    if (sg->interleave) {
        if (nslots > ceil_div(g.M, st_bm(sg->wn))) nslots = ceil_div(g.M, st_bm(sg->wn));
        sg->rps = 0;
        sg->nslots = (int)nslots;
    } else {
        sg->rps = (int)ceil_div(g.M, nslots);
        sg->nslots = (int)ceil_div(g.M, sg->rps);
    }
    sg->strided = strided;
    sg->howo = (int)howo;
    sg->howo_magic = (unsigned)(((uint64_t(1) << 32) + howo - 1) / howo);
    sg->wo_magic = (unsigned)(((uint64_t(1) << 32) + g.Wo - 1) / g.Wo);
    if (howo == 1) sg->howo_magic = 0;              // divisor 1: the kernel takes the dividend as it is
    if (g.Wo == 1) sg->wo_magic = 0;
    sg->img_bytes = g.H * g.W * g.Cin;
    sg->row_step = g.stride * g.W * g.Cin;
    sg->col_step = g.stride * g.Cin;
    sg->x_bytes = (int)x_bytes;
    return true;
}

int pick_tile(int64_t M, int64_t N)
{
    if (N <= 64) return 0;
    if (M <= 64) return 2;
    return 1;
}

// gs: 0 for a GEMM or a dense convolution, else the channels per group of a grouped convolution
// (the caller has checked that the shape is one the grouped kernel takes).
// The checks every inference call makes on its descriptor and pointers.  *empty: nothing to compute.
nq_status check_problem(bool full, const int8_t *d_x, int64_t M, const nq_weight *w, const nq_epilogue *epi,
                        const void *d_y, bool *empty)
{
    *empty = false;
    if (!w || !epi) return NQ_ERR_INVALID_ARG;
    nq_status st = check_cfg(&w->cfg);
    if (st != NQ_OK) return st;
    if ((st = check_shape(w->N, w->K)) != NQ_OK) return st;
    if (M < 0) return NQ_ERR_INVALID_ARG;
    const int h = w->cfg.n_bits - w->cfg.l_bits;
    if (full && !w->low_resident) return NQ_ERR_NOT_RESIDENT;
    if (M == 0 || w->N == 0) {
        *empty = true;
        return NQ_OK;
    }
    if (w->K == 0) return NQ_ERR_SHAPE;
    if (!d_x || !d_y || !w->d_high || !w->d_scale || (full && !w->d_low)) return NQ_ERR_INVALID_ARG;
    if (!aligned16(w->d_high) || (full && !aligned16(w->d_low))) return NQ_ERR_ALIGN;
    if (w->high_bytes < nq_packed_bytes(w->N, w->K, h, w->cfg.layout)) return NQ_ERR_RANGE;
    if (full && w->low_bytes < nq_packed_bytes(w->N, w->K, low_field_bits(&w->cfg), w->cfg.layout)) return NQ_ERR_RANGE;
    if (w->N > (1 << 24) || M > (int64_t(1) << 40) / (w->N > 0 ? w->N : 1)) return NQ_ERR_SHAPE;
    return NQ_OK;
}

// Kernel arguments of a checked problem.
void fill_params(bool full, const int8_t *d_x, const Geometry &g, const nq_weight *w, const nq_epilogue *epi,
                 void *d_y, GemmParams *out)
{
    GemmParams &p = *out;
    const int l = w->cfg.l_bits;
    p.x = d_x;
    p.ph = (const uint32_t *)w->d_high;
    p.pl = full ? (const uint32_t *)w->d_low : nullptr;
    p.scale = w->d_scale;
    p.y = d_y;
    p.bias = epi->d_bias;
    p.resid = epi->d_residual;
    p.acc_dump = epi->d_acc_dump;
    p.M = g.M;
    p.N = (int)w->N;
    p.K = (int)w->K;
    p.KB = (int)ceil_div(w->K, 64);
    p.NB = (int)ceil_div(w->N, 32);
    p.H = g.H; p.W = g.W; p.Cin = g.Cin; p.Ho = g.Ho; p.Wo = g.Wo;
    p.KH = g.KH; p.KW = g.KW; p.stride = g.stride; p.pad = g.pad;
    p.act_scale = epi->act_scale;
    p.resid_scale = epi->residual_scale;
    p.inv_out_scale = epi->inv_out_scale;
    p.part_mul = (float)(1 << l);
    p.relu = epi->relu != 0;
    p.out_int8 = epi->out_int8 != 0;
    // 16-byte activation loads need every chunk of 16 consecutive k inside one pixel
    p.fast_a = (g.Cin % 16 == 0) && aligned16(d_x);
    p.low_signed = w->cfg.low_format == NQ_LOW_SIGNED_L1;
    // the vector epilogue of int8 outputs moves 16 channels at a time; fp32 outputs with a residual
    // (a calibration pass) and the accumulator dump take the element-wise one as well
    if (p.out_int8)
        p.general = p.acc_dump != nullptr || p.N % 16 != 0 || !aligned16(d_y) || !aligned16(p.resid) ||
                    !aligned16(p.scale) || !aligned16(p.bias);
    else
        p.general = p.acc_dump != nullptr || p.resid != nullptr;
    p.conv_big = 0;
    p.cin_shift = 0;
    p.kw_magic = 0;
}

// Makes `s` wait for a lower-bit page that may still be in flight on its copy stream.
bool wait_for_page(const nq_weight *w, hipStream_t s)
{
    if (!(w->low_event_armed && w->low_event)) return true;
    // Once the copy has completed no later launch needs to wait for it: the flag (an internal field of
    // the caller's descriptor) is dropped, so that only the launches issued while the page travels pay
    // for a wait.  Not while the stream is being captured: an event recorded inside a capture cannot
    // be queried, and a replay needs the dependency every time.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    const bool capturing = hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone;
    if (!capturing && hipEventQuery((hipEvent_t)w->low_event) == hipSuccess) {
        const_cast<nq_weight *>(w)->low_event_armed = 0;
        return true;
    }
    (void)hipGetLastError();   // hipErrorNotReady from the query is not an error
    if (hipStreamWaitEvent(s, (hipEvent_t)w->low_event, 0) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return true;
}

// gs: 0 for a GEMM or a dense convolution, else the channels per group of a grouped convolution
// (the caller has checked that the shape is one the grouped kernel takes).
// gs_out: 0, or the output channels per group of a grouped convolution that the kernel for 1, 2 or 4 channels per
// group does not take (then gs is the input channels per group, and the direct kernel runs).
nq_status run(bool full, const int8_t *d_x, const Geometry &g, const nq_weight *w, const nq_epilogue *epi,
              void *d_y, void *stream, int gs = 0, int gs_out = 0)
{
    if (!w || !epi) return NQ_ERR_INVALID_ARG;
    nq_status st = check_cfg(&w->cfg);
    if (st != NQ_OK) return st;
    // the paper's word pages (Sec. 3.3.4) are read by the GEMM and the dense convolution, not by the grouped one
    const bool words = w->cfg.layout == NQ_LAYOUT_PAPER_U64;
    if (words && gs > 0) return NQ_ERR_UNSUPPORTED;
    bool empty = false;
    if ((st = check_problem(full, d_x, g.M, w, epi, d_y, &empty)) != NQ_OK || empty) return st;
    const int h = w->cfg.n_bits - w->cfg.l_bits, l = w->cfg.l_bits;

    hipStream_t s = (hipStream_t)stream;

    GemmParams p;
    fill_params(full, d_x, g, w, epi, d_y, &p);

    // Everything that can fail is checked before anything is enqueued: `commit` is called once the kernel
    // and its geometry are fixed, right before the launch.  It makes the stream wait for a page that may
    // still be in flight on the copy stream and takes the one-shot profiling events.
    void *ev0 = nullptr, *ev1 = nullptr;
    auto commit = [&]() -> bool {
        if (full && !wait_for_page(w, s)) return false;
        ev0 = g_ev_start;
        ev1 = g_ev_stop;
        g_ev_start = g_ev_stop = nullptr;
        return true;
    };
    if (words) {
        // 32-bit byte offsets into the activations (a filter other than 1x1 stride 1 gathers its rows from the whole
        // input tensor, pixel coordinates in 16 bits), dword loads relative to their first byte
        const bool gather = g.KH != 1 || g.KW != 1 || g.stride != 1 || g.pad != 0;
        const int64_t x_bytes = gather ? (g.M / ((int64_t)g.Ho * g.Wo)) * g.H * g.W * g.Cin : g.M * w->K;
        if (x_bytes >= 0x7fff0000LL || ceil_div(g.M, 32) > 65535) return NQ_ERR_SHAPE;
        if (gather && (g.H > 16000 || g.W > 16000 || g.pad > 255 || g.KH > 255 || g.KW > 255)) return NQ_ERR_SHAPE;
        if ((reinterpret_cast<uintptr_t>(d_x) & 3u) != 0) return NQ_ERR_ALIGN;
        p.conv_big = 0;
        p.cin_shift = 0;
        p.kw_magic = 0;
        const int WH = (int)ceil_div(w->K, 64 / h);
        const int lf = low_field_bits(&w->cfg);
        const int WL = (int)ceil_div(w->K, 64 / lf);
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 8; g_last_variant = 0;
        launch_nested_gemm_words(full, h, l, p, WH, WL, s, ev0, ev1);
        return launch_status();
    }
    if (gs > 0 && gs_out > 0) {
        p.conv_big = 0;
        p.cin_shift = 0;
        p.kw_magic = 0;
        p.general = 1;
        // four consecutive k are one aligned dword of the input when the group width, the channel count and the
        // pointer are multiples of four
        const int quads = gs % 4 == 0 && g.Cin % 4 == 0 && (reinterpret_cast<uintptr_t>(d_x) & 3u) == 0;
        if (ceil_div(g.M, 32) > 0x7fffffffLL || ceil_div(w->N, 64) > 65535) return NQ_ERR_SHAPE;
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 10; g_last_variant = quads;
        NQ_DISPATCH_HL(h, l, launch_nested_conv_grouped_any, full, p, gs, gs_out, quads, s, ev0, ev1);
        return launch_status();
    }
    if (gs > 0) {
        GroupGeom gg;
        if (!plan_grouped(g, gs, w->N, &gg)) return NQ_ERR_UNSUPPORTED;
        p.conv_big = 0;
        p.cin_shift = 0;
        p.kw_magic = 65536 / g.KW + 1;      // tap / KW == (tap * kw_magic) >> 16 for the few taps of a filter
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 7; g_last_variant = 0;
        NQ_DISPATCH_HL(h, l, launch_nested_conv_grouped, full, p, gg, s, ev0, ev1);
        return launch_status();
    }
    // NQ_TUNE_KERNEL (test and tuning aid): 1 generic, 2 windowed, 3 register-stationary, 4 large GEMM,
    // 5 few input channels, 6 few rows, 9 stationary-weights GEMM;
    // a kernel that does not apply to the shape is never forced, the choice falls through.
    const int force = g_tune[NQ_TUNE_KERNEL].load(std::memory_order_relaxed);
    const bool plain_gemm = g.KH == 1 && g.KW == 1 && g.stride == 1 && g.pad == 0 && w->K % 256 == 0 && aligned16(d_x);
    // implicit GEMM on the same kernel: any filter over a power-of-two number (>= 16) of input channels
    const int64_t x_bytes = (g.M / ((int64_t)g.Ho * g.Wo)) * g.H * g.W * g.Cin;
    const bool conv_gemm = !plain_gemm && g.Cin >= 16 && (g.Cin & (g.Cin - 1)) == 0 && aligned16(d_x) &&
                           x_bytes < 0x7fff0000LL && g.M < (int64_t(1) << 31) && g.H <= 8192 && g.W <= 8192 &&
                           g.KH * g.KW * g.KW < 65536 && g.KH <= 15 && g.KW <= 16;
    p.conv_big = conv_gemm;
    p.cin_shift = 0;
    while ((1 << p.cin_shift) < g.Cin) ++p.cin_shift;
    p.kw_magic = 65536 / g.KW + 1;
    const bool big_ok = plain_gemm || conv_gemm;
    bool big_wanted = g.M > 64 && w->N > 64 && w->K >= 256;
    // short reductions stay with the register-stationary kernel, which fetches the input once per 32 to 128
    // output channels; with 512 channels or more out of 512 in, the large kernel's 256-column tiles win
    // (strided 1x1, 28x28x512 -> 1024 at batch 128: 30 us against 48 us)
    if (conv_gemm && w->K <= 576 && !(w->K >= 512 && w->N >= 512)) big_wanted = false;
    // Filters over up to 64 output channels at stride 1 go to the windowed kernel (64 channels per block): the
    // large-GEMM kernel's tiles, 128 columns at the least, would be half empty.  (Up to 128 channels they went there
    // too while the large kernel had 256-column tiles only; with its 128 x 128 variant, 3x3, 28x28x128 -> 128 at
    // batch 128 takes 29 us against 42 us, and at stride 2 31 us against 59 us.)
    {
        WindowGeom wg0;
        size_t lds0 = 0;
        if (conv_gemm && w->N <= 64 && g.stride == 1 && g.KH * g.KW > 1 && plan_window(g, d_x, &wg0, &lds0))
            big_wanted = false;
    }
    // short reductions without a filter window: weights stationary in registers, rows streamed
    StatGeom tg;
    if ((force == 9 || (force == 0 && g.M > 64)) && plan_stat(g, d_x, w->N, w->K, &tg)) {
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 9; g_last_variant = tg.wn;
        NQ_DISPATCH_HL(h, l, launch_nested_gemm_stat, full, p, tg, s, ev0, ev1);
        return launch_status();
    }
    if (big_ok && (force == 4 || (force == 0 && big_wanted))) {
        const int64_t blocks = ceil_div(g.M, 64) * ceil_div(w->N, 256);
        if (blocks > 0x7fffffffLL) return NQ_ERR_SHAPE;
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 4;
        NQ_DISPATCH_HL(h, l, launch_nested_gemm_big, full, p, g_tune[NQ_TUNE_BIG_TM].load(std::memory_order_relaxed),
                       &g_last_variant, s, ev0, ev1);
        return launch_status();
    }
    // few rows: the packed weights are the traffic; one block per 32 columns, K split over the waves
    const bool skinny_ok = g.KH == 1 && g.KW == 1 && g.stride == 1 && g.pad == 0 && g.M <= 64 && w->K % 16 == 0 &&
                           aligned16(d_x) && ceil_div(w->N, 32) <= 0x7fffffffLL;
    if (skinny_ok && (force == 6 || (force == 0 && w->K >= 256))) {
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 6; g_last_variant = 0;
        NQ_DISPATCH_HL(h, l, launch_nested_gemm_skinny, full, p, s, ev0, ev1);
        return launch_status();
    }
    SmallCinGeom cg;
    if ((force == 0 || force == 5) && plan_smallcin(g, d_x, w->N, &cg)) {
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 5; g_last_variant = 0;
        NQ_DISPATCH_HL(h, l, launch_nested_conv_smallcin, full, p, cg, s, ev0, ev1);
        return launch_status();
    }
    StreamGeom sg;
    int grid_x = 0;
    if ((force == 0 || force == 3) && plan_rowstream(g, d_x, w->N, &sg, &grid_x)) {
        if ((int64_t)(grid_x + 7) * ceil_div(w->N, 32) > 0x7fffffffLL) return NQ_ERR_SHAPE;
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 3; g_last_variant = 0;
        NQ_DISPATCH_HL(h, l, launch_nested_conv_rowstream, full, p, sg, grid_x, s, ev0, ev1);
        return launch_status();
    }
    WindowGeom wg;
    size_t lds = 0;
    if ((force == 0 || force == 2) && plan_window(g, d_x, &wg, &lds)) {
        const int64_t blocks_x = (g.M / ((int64_t)g.Ho * g.Wo)) * wg.RB;
        if (blocks_x > 0x7fffffffLL || ceil_div(w->N, 64) > 65535) return NQ_ERR_SHAPE;
        if (!commit()) return NQ_ERR_HIP;
        g_last_family = 2; g_last_variant = 0;
        NQ_DISPATCH_HL(h, l, launch_nested_conv_window, full, 0, p, wg, lds, s, ev0, ev1);
        return launch_status();
    }
    const int tile = pick_tile(g.M, w->N);
    if (ceil_div(g.M, NQ_TILE_BM[tile]) > 0x7fffffffLL || ceil_div(w->N, NQ_TILE_BN[tile]) > 65535)
        return NQ_ERR_SHAPE;
    if (!commit()) return NQ_ERR_HIP;
    g_last_family = 1; g_last_variant = tile;
    NQ_DISPATCH_HL(h, l, launch_nested_gemm, full, tile, p, s, ev0, ev1);
    return launch_status();
}

nq_status gemm(bool full, const int8_t *d_x, int64_t M, const nq_weight *w, const nq_epilogue *epi, void *d_y,
               void *stream)
{
    if (!w) return NQ_ERR_INVALID_ARG;
    Geometry g;
    g.M = M;
    g.H = g.W = g.Ho = g.Wo = g.KH = g.KW = g.stride = 1;
    g.pad = 0;
    g.Cin = (int)w->K;
    return run(full, d_x, g, w, epi, d_y, stream);
}

// ---- many few-row GEMMs in one launch ------------------------------------------------------------------------
// Layout of the table the batch kernel reads: `count` problems, then the running count of their blocks.
size_t batch_table_bytes(int64_t count)
{
    return (size_t)count * sizeof(GemmParams) + (size_t)(count + 1) * sizeof(int);
}

// Scratch of nq_gemm_batch_static: the same table in a device array of the library itself, for callers that
// cannot allocate.  Every GPU the library runs on holds its own copy; host code reaches it through the address
// hipGetSymbolAddress returns for the current device, never through the array's name.
constexpr int64_t BATCH_STATIC_MAX = NQ_GEMM_BATCH_STATIC_MAX;
static __device__ __align__(256) unsigned char g_batch_scratch[BATCH_STATIC_MAX * sizeof(GemmParams) +
                                                               (BATCH_STATIC_MAX + 1) * sizeof(int)];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES];        // per device, filled on the first call made with that device current

nq_status static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(g_batch_scratch)) != hipSuccess || !q) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
        g_scratch_ptr[dev] = q;
    }
    *ptr = g_scratch_ptr[dev];
    return NQ_OK;
}

nq_status gemm_batch(const nq_gemm_job *jobs, int64_t count, int full_bit, void *d_table, size_t table_bytes,
                     void *stream)
{
    if (count < 0 || (count > 0 && !jobs)) return NQ_ERR_INVALID_ARG;
    if (count == 0) return NQ_OK;
    if (count > (int64_t(1) << 20)) return NQ_ERR_SHAPE;
    if (!d_table || ((uintptr_t)d_table & 15u) != 0) return d_table ? NQ_ERR_ALIGN : NQ_ERR_INVALID_ARG;
    if (table_bytes < batch_table_bytes(count)) return NQ_ERR_RANGE;
    const bool full = full_bit != 0;
    // The table is staged in host memory that stays valid until this thread's next call; the copy below is
    // ordered on the stream like the launch that reads it.
    thread_local std::vector<unsigned char> staging;
    staging.resize(batch_table_bytes(count));
    GemmParams *hp = reinterpret_cast<GemmParams *>(staging.data());
    int *hfirst = reinterpret_cast<int *>(staging.data() + (size_t)count * sizeof(GemmParams));
    const nq_cfg cfg0 = jobs[0].w ? jobs[0].w->cfg : nq_cfg{0, 0, 0, 0};
    int mode0 = -1;
    bool two_tiles = false, staged = false;
    int64_t blocks = 0, live = 0;
    for (int64_t i = 0; i < count; ++i) {
        const nq_gemm_job &j = jobs[i];
        bool empty = false;
        nq_status st = check_problem(full, j.d_x, j.M, j.w, &j.epi, j.d_y, &empty);
        if (st != NQ_OK) return st;
        // one kernel instantiation serves the whole table: same nesting and format, dense pages, few rows,
        // the 16-byte activation path, one epilogue layout
        if (j.w->cfg.n_bits != cfg0.n_bits || j.w->cfg.l_bits != cfg0.l_bits || j.w->cfg.low_format != cfg0.low_format ||
            j.w->cfg.layout != NQ_LAYOUT_DENSE)
            return NQ_ERR_UNSUPPORTED;
        if (empty) continue;
        if (j.M > 64 || j.w->K % 16 != 0) return NQ_ERR_UNSUPPORTED;
        if (!aligned16(j.d_x)) return NQ_ERR_ALIGN;
        if (j.M * j.w->K >= 0x7fff0000LL) return NQ_ERR_SHAPE;
        Geometry g;
        g.M = j.M;
        g.H = g.W = g.Ho = g.Wo = g.KH = g.KW = g.stride = 1;
        g.pad = 0;
        g.Cin = (int)j.w->K;
        fill_params(full, j.d_x, g, j.w, &j.epi, j.d_y, &hp[live]);
        const int mode = hp[live].general ? 2 : (hp[live].out_int8 ? 1 : 0);
        if (mode == 2) return NQ_ERR_UNSUPPORTED;           // accumulator dump, ragged N, fp32 output with residual
        if (mode0 < 0) mode0 = mode;
        if (mode != mode0) return NQ_ERR_UNSUPPORTED;
        two_tiles = two_tiles || j.M > 32;
        staged = staged || hp[live].KB >= 32;
        hfirst[live] = (int)blocks;
        blocks += hp[live].NB;
        if (blocks > 0x7fffffffLL) return NQ_ERR_SHAPE;
        ++live;
    }
    if (live == 0) return NQ_OK;
    hfirst[live] = (int)blocks;
    // compact layout on the device: `live` problems, then live + 1 running counts
    std::memmove(staging.data() + (size_t)live * sizeof(GemmParams), hfirst, (size_t)(live + 1) * sizeof(int));
    hipStream_t s = (hipStream_t)stream;
    if (full) {
        const void *last = nullptr;
        for (int64_t i = 0; i < count; ++i) {            // one wait per distinct event (a group shares one)
            const nq_weight *w = jobs[i].w;
            if (jobs[i].M == 0 || w->N == 0 || w->low_event == last) continue;
            last = w->low_event;
            if (!wait_for_page(w, s)) return NQ_ERR_HIP;
        }
    }
    const size_t bytes = (size_t)live * sizeof(GemmParams) + (size_t)(live + 1) * sizeof(int);
    if (hipMemcpyAsync(d_table, staging.data(), bytes, hipMemcpyHostToDevice, s) != hipSuccess) {
        (void)hipGetLastError();
        return NQ_ERR_HIP;
    }
    const GemmParams *d_jobs = reinterpret_cast<const GemmParams *>(d_table);
    const int *d_first = reinterpret_cast<const int *>((const unsigned char *)d_table + (size_t)live * sizeof(GemmParams));
    const int h = cfg0.n_bits - cfg0.l_bits, l = cfg0.l_bits;
    const int fmode = full ? (cfg0.low_format == NQ_LOW_SIGNED_L1 ? 2 : 1) : 0;
    g_last_family = 6; g_last_variant = 1;
    void *ev0 = g_ev_start, *ev1 = g_ev_stop;            // one-shot profiling events, as for a single launch
    g_ev_start = g_ev_stop = nullptr;
    NQ_DISPATCH_HL(h, l, launch_nested_gemm_skinny_batch, fmode, mode0, two_tiles, staged, d_jobs, d_first, (int)live,
                   (int)blocks, s, ev0, ev1);
    return launch_status();
}

nq_status conv(bool full, const int8_t *d_x, const nq_conv_shape *sh, const nq_weight *w, const nq_epilogue *epi,
               void *d_y, void *stream)
{
    if (!sh || !w) return NQ_ERR_INVALID_ARG;
    if (sh->B < 0 || sh->H < 1 || sh->W < 1 || sh->Cin < 1 || sh->Cout < 0 || sh->KH < 1 || sh->KW < 1 ||
        sh->stride < 1 || sh->pad < 0)
        return NQ_ERR_INVALID_ARG;
    if (sh->H > 32768 || sh->W > 32768 || sh->Cin > NQ_MAX_K || sh->KH > 64 || sh->KW > 64 || sh->pad > 64 ||
        sh->stride > 64)
        return NQ_ERR_SHAPE;
    if (w->N != sh->Cout || w->K != (int64_t)sh->KH * sh->KW * sh->Cin) return NQ_ERR_SHAPE;
    const int64_t Ho = (sh->H + 2 * sh->pad - sh->KH) / sh->stride + 1;
    const int64_t Wo = (sh->W + 2 * sh->pad - sh->KW) / sh->stride + 1;
    if (sh->H + 2 * sh->pad < sh->KH || sh->W + 2 * sh->pad < sh->KW) return NQ_ERR_SHAPE;
    Geometry g;
    g.M = sh->B * Ho * Wo;
    g.H = (int)sh->H; g.W = (int)sh->W; g.Cin = (int)sh->Cin; g.Ho = (int)Ho; g.Wo = (int)Wo;
    g.KH = sh->KH; g.KW = sh->KW; g.stride = sh->stride; g.pad = sh->pad;
    return run(full, d_x, g, w, epi, d_y, stream);
}

// Depthwise / grouped convolution: as many output as input channels, groups of 1, 2 or 4 channels.
nq_status gconv(bool full, const int8_t *d_x, const nq_conv_shape *sh, int groups, const nq_weight *w,
                const nq_epilogue *epi, void *d_y, void *stream)
{
    if (!sh || !w) return NQ_ERR_INVALID_ARG;
    if (sh->B < 0 || sh->H < 1 || sh->W < 1 || sh->Cin < 1 || sh->Cout < 0 || sh->KH < 1 || sh->KW < 1 ||
        sh->stride < 1 || sh->pad < 0 || groups < 1)
        return NQ_ERR_INVALID_ARG;
    if (sh->H > 32768 || sh->W > 32768 || sh->Cin > NQ_MAX_K || sh->KH > 64 || sh->KW > 64 || sh->pad > 64 ||
        sh->stride > 64)
        return NQ_ERR_SHAPE;
    if (sh->Cin % groups != 0 || sh->Cout % groups != 0 || sh->Cout < 1) return NQ_ERR_SHAPE;
    const int64_t gs = sh->Cin / groups, gs_out = sh->Cout / groups;
    if (w->N != sh->Cout || w->K != (int64_t)sh->KH * sh->KW * gs) return NQ_ERR_SHAPE;
    if (sh->H + 2 * sh->pad < sh->KH || sh->W + 2 * sh->pad < sh->KW) return NQ_ERR_SHAPE;
    // what the matrix-core kernel is built for: as many output as input channels, groups inside a run of 4
    // channels, 16-byte pieces of a pixel, up to 28 taps, 16-byte aligned input; everything else (wider groups,
    // unequal channel counts, odd channel counts, any alignment) goes to the direct kernel
    const bool narrow = sh->Cin == sh->Cout && (gs == 1 || gs == 2 || gs == 4) && sh->Cin % 16 == 0 &&
                        sh->KH * sh->KW <= 28 && aligned16(d_x);
    const int64_t Ho = (sh->H + 2 * sh->pad - sh->KH) / sh->stride + 1;
    const int64_t Wo = (sh->W + 2 * sh->pad - sh->KW) / sh->stride + 1;
    if (sh->B * sh->H * sh->W * sh->Cin >= 0x7fff0000LL || sh->B * Ho * Wo >= (int64_t(1) << 31) - 64)
        return NQ_ERR_SHAPE;
    Geometry g;
    g.M = sh->B * Ho * Wo;
    g.H = (int)sh->H; g.W = (int)sh->W; g.Cin = (int)sh->Cin; g.Ho = (int)Ho; g.Wo = (int)Wo;
    g.KH = sh->KH; g.KW = sh->KW; g.stride = sh->stride; g.pad = sh->pad;
    return run(full, d_x, g, w, epi, d_y, stream, (int)gs, narrow ? 0 : (int)gs_out);
}

}  // namespace

extern "C" nq_status nq_gconv_full(const int8_t *d_x, const nq_conv_shape *shape, int groups, const nq_weight *w,
                                   const nq_epilogue *epi, void *d_y, void *stream)
{
    return gconv(true, d_x, shape, groups, w, epi, d_y, stream);
}

extern "C" nq_status nq_gconv_part(const int8_t *d_x, const nq_conv_shape *shape, int groups, const nq_weight *w,
                                   const nq_epilogue *epi, void *d_y, void *stream)
{
    return gconv(false, d_x, shape, groups, w, epi, d_y, stream);
}

extern "C" size_t nq_gemm_batch_workspace_bytes(int64_t count)
{
    return count > 0 ? batch_table_bytes(count) : 0;
}

extern "C" nq_status nq_gemm_batch(const nq_gemm_job *jobs, int64_t count, int full_bit, void *d_workspace,
                                   size_t workspace_bytes, void *stream)
{
    return gemm_batch(jobs, count, full_bit, d_workspace, workspace_bytes, stream);
}

extern "C" nq_status nq_gemm_batch_static(const nq_gemm_job *jobs, int64_t count, int full_bit, void *stream)
{
    if (count > BATCH_STATIC_MAX) return NQ_ERR_SHAPE;      // beyond the library's own table
    if (count <= 0) return count < 0 ? NQ_ERR_INVALID_ARG : NQ_OK;
    void *scratch = nullptr;
    nq_status st = static_scratch(&scratch);
    if (st != NQ_OK) return st;
    return gemm_batch(jobs, count, full_bit, scratch, sizeof(g_batch_scratch), stream);
}

extern "C" nq_status nq_set_tuning(int key, int value)
{
    if (key < 0 || key >= NQ_TUNE_COUNT || value < 0) return NQ_ERR_INVALID_ARG;
    g_tune[key].store(value, std::memory_order_relaxed);
    return NQ_OK;
}

extern "C" nq_status nq_profile_last_kernel(int *family, int *variant)
{
    if (family) *family = g_last_family;
    if (variant) *variant = g_last_variant;
    return NQ_OK;
}

extern "C" nq_status nq_profile_next_launch(void *start_event, void *stop_event)
{
    g_ev_start = start_event;
    g_ev_stop = stop_event;
    return NQ_OK;
}

extern "C" nq_status nq_gemm_full(const int8_t *d_x, int64_t M, const nq_weight *w, const nq_epilogue *epi,
                                  void *d_y, void *stream)
{
    return gemm(true, d_x, M, w, epi, d_y, stream);
}

extern "C" nq_status nq_gemm_part(const int8_t *d_x, int64_t M, const nq_weight *w, const nq_epilogue *epi,
                                  void *d_y, void *stream)
{
    return gemm(false, d_x, M, w, epi, d_y, stream);
}

extern "C" nq_status nq_conv_full(const int8_t *d_x, const nq_conv_shape *shape, const nq_weight *w,
                                  const nq_epilogue *epi, void *d_y, void *stream)
{
    return conv(true, d_x, shape, w, epi, d_y, stream);
}

extern "C" nq_status nq_conv_part(const int8_t *d_x, const nq_conv_shape *shape, const nq_weight *w,
                                  const nq_epilogue *epi, void *d_y, void *stream)
{
    return conv(false, d_x, shape, w, epi, d_y, stream);
}
