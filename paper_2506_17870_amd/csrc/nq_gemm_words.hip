// Instantiations and launcher of the GEMM over the paper's word pages (nq_gemm_words.h): one kernel per
// field width of the higher-bit page in part-bit mode, one per nesting and lower-bit format in full-bit mode.
#include "nq_gemm_words.h"

namespace nq {

template <typename K>
static void words_grant_lds(K kernel, size_t lds)
{
    static bool granted = false;   // one per kernel instantiation
    if (!granted && lds > 64 * 1024) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
        granted = true;
    }
}

template <int HB, int LB, int MODE>
static void launch_words(const GemmParams &p, int WH, int WL, hipStream_t st, void *ev_start, void *ev_stop)
{
    // Four waves per block, two or more blocks per compute unit; where a layer with long rows has fewer blocks
    // than that, eight waves per block share a page's steps.
    const dim3 grid((unsigned)p.NB, (unsigned)((p.M + 31) / 32));
    const bool wide = (int64_t)grid.x * grid.y < 512 && WH >= 128;
    // a filter other than 1x1 stride 1 gathers its rows from the NHWC input (four waves only)
    const bool gather = p.KH != 1 || p.KW != 1 || p.stride != 1 || p.pad != 0;
    if (gather) {
        auto k = k_nested_gemm_words<HB, LB, MODE, 4, true>;
        constexpr size_t lds = words_lds_bytes<HB, LB, 4>();
        words_grant_lds(k, lds);
        launch_timed(k, grid, dim3(256), lds, st, ev_start, ev_stop, p, WH, WL);
    } else if (wide) {
        auto k = k_nested_gemm_words<HB, LB, MODE, 8, false>;
        constexpr size_t lds = words_lds_bytes<HB, LB, 8>();
        words_grant_lds(k, lds);
        launch_timed(k, grid, dim3(512), lds, st, ev_start, ev_stop, p, WH, WL);
    } else {
        auto k = k_nested_gemm_words<HB, LB, MODE, 4, false>;
        constexpr size_t lds = words_lds_bytes<HB, LB, 4>();
        words_grant_lds(k, lds);
        launch_timed(k, grid, dim3(256), lds, st, ev_start, ev_stop, p, WH, WL);
    }
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
