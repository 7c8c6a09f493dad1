// Instantiations and launcher of the GEMM over the paper's word pages (nq_gemm_words.h): one kernel per
// field width of the higher-bit page in part-bit mode, one per nesting and lower-bit format in full-bit mode.
#include "nq_gemm_words.h"

namespace nq {

template <int HB, int LB, int MODE>
static void launch_words(const GemmParams &p, int WH, int WL, hipStream_t st, void *ev_start, void *ev_stop)
{
    // Four waves per block.  (Sixteen, to have more of the pages in flight when a layer has few blocks, measured
    // slower: the activation fetches of a step, one cache line per lane, are what a compute unit runs out of.)
    const dim3 grid((unsigned)p.NB, (unsigned)((p.M + 31) / 32));
    const int waves = 4;
    launch_timed(k_nested_gemm_words<HB, LB, MODE>, grid, dim3(64 * waves), (size_t)(waves - 1) * 4096, st, ev_start,
                 ev_stop, p, WH, WL);
}

template <int H, int L>
static void launch_words_hl(bool full, const GemmParams &p, int WH, int WL, hipStream_t st, void *ev_start,
                            void *ev_stop)
{
    if (!full) launch_words<H, 0, 0>(p, WH, WL, st, ev_start, ev_stop);
    else if (p.low_signed) launch_words<H, L + 1, 2>(p, WH, WL, st, ev_start, ev_stop);
    else launch_words<H, L, 1>(p, WH, WL, st, ev_start, ev_stop);
}

void launch_nested_gemm_words(bool full, int h, int l, const GemmParams &p, int WH, int WL, hipStream_t st,
                              void *ev_start, void *ev_stop)
{
    switch (h * 8 + l) {
    case 7 * 8 + 1: launch_words_hl<7, 1>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 6 * 8 + 2: launch_words_hl<6, 2>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 5 * 8 + 3: launch_words_hl<5, 3>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 4 * 8 + 4: launch_words_hl<4, 4>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 3 * 8 + 5: launch_words_hl<3, 5>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 2 * 8 + 6: launch_words_hl<2, 6>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 5 * 8 + 1: launch_words_hl<5, 1>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 4 * 8 + 2: launch_words_hl<4, 2>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 3 * 8 + 3: launch_words_hl<3, 3>(full, p, WH, WL, st, ev_start, ev_stop); break;
    case 2 * 8 + 4: launch_words_hl<2, 4>(full, p, WH, WL, st, ev_start, ev_stop); break;
    default: break;
    }
}

}  // namespace nq
