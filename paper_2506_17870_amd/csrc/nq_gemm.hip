// Host side of the inference entry points: argument checks, residency of the lower-bit
// page (paper Sec. 3.2.3 / 3.3: the caller picks full-bit or part-bit; a paged-out page is
// an error, never a silent downgrade), tile choice and launch.
#include "nq_common.h"
#include "nq_gemm_params.h"

using namespace nq;

namespace {

struct Geometry {
    int64_t M;
    int H, W, Cin, Ho, Wo, KH, KW, stride, pad;
};

int pick_tile(int64_t M, int64_t N)
{
    if (N <= 64) return 0;
    if (M <= 64) return 2;
    return 1;
}

nq_status run(bool full, const int8_t *d_x, const Geometry &g, const nq_weight *w, const nq_epilogue *epi,
              void *d_y, void *stream)
{
    if (!w || !epi) return NQ_ERR_INVALID_ARG;
    nq_status st = check_cfg(&w->cfg);
    if (st != NQ_OK) return st;
    if (w->cfg.layout != NQ_LAYOUT_DENSE) return NQ_ERR_UNSUPPORTED;
    if ((st = check_shape(w->N, w->K)) != NQ_OK) return st;
    if (g.M < 0) return NQ_ERR_INVALID_ARG;
    const int h = w->cfg.n_bits - w->cfg.l_bits, l = w->cfg.l_bits;
    if (full && !w->low_resident) return NQ_ERR_NOT_RESIDENT;
    if (g.M == 0 || w->N == 0) return NQ_OK;
    if (w->K == 0) return NQ_ERR_SHAPE;
    if (!d_x || !d_y || !w->d_high || !w->d_scale || (full && !w->d_low)) return NQ_ERR_INVALID_ARG;
    if (!aligned16(w->d_high) || (full && !aligned16(w->d_low))) return NQ_ERR_ALIGN;
    if (w->high_bytes < nq_packed_bytes(w->N, w->K, h, NQ_LAYOUT_DENSE)) return NQ_ERR_RANGE;
    if (full && w->low_bytes < nq_packed_bytes(w->N, w->K, l, NQ_LAYOUT_DENSE)) return NQ_ERR_RANGE;
    if (g.M > (int64_t(1) << 40) / (w->N > 0 ? w->N : 1)) return NQ_ERR_SHAPE;

    hipStream_t s = (hipStream_t)stream;
    if (full && w->low_event_armed && w->low_event) {
        // the page may still be in flight on the copy stream
        if (hipStreamWaitEvent(s, (hipEvent_t)w->low_event, 0) != hipSuccess) {
            (void)hipGetLastError();
            return NQ_ERR_HIP;
        }
    }

    GemmParams p;
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

    const int tile = pick_tile(g.M, w->N);
    if (ceil_div(g.M, NQ_TILE_BM[tile]) > 0x7fffffffLL || ceil_div(w->N, NQ_TILE_BN[tile]) > 65535)
        return NQ_ERR_SHAPE;
    NQ_DISPATCH_HL(h, l, launch_nested_gemm, full, tile, p, s);
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

}  // namespace

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
