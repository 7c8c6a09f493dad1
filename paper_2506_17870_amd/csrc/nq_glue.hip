// Glue between the nested convolutions of a residual CNN on int8 NHWC activations.  The
// paper only states that the models are CNNs with 8-bit activations (Sec. 4.2); these two
// memory-bound kernels make a whole quantised network runnable on the device.
#include "nq_common.h"

namespace nq {

// One thread per sixteen channels of one output pixel (C a multiple of 16, 16-byte aligned tensors): 16-byte
// loads and stores; the maximum is taken on pairs of bytes moved to the top of 16-bit halves, where the packed
// 16-bit maximum orders them like the signed bytes they are.  grid.x covers one output row (Wo * C / 16
// threads), grid.y the output rows, grid.z the images (strided when there are more than the grid holds).
typedef short p_v2s __attribute__((ext_vector_type(2)));

__global__ void __launch_bounds__(256) k_maxpool_i8_v16(const int8_t *__restrict__ x, int64_t B, int H, int W, int C16,
                                                         int Ho, int Wo, int ksize, int stride, int pad,
                                                         int8_t *__restrict__ y)
{
    const unsigned ix = blockIdx.x * 256u + threadIdx.x;
    if (ix >= (unsigned)(Wo * C16)) return;
    const int ow = (int)(ix / (unsigned)C16), c16 = (int)(ix - (unsigned)ow * (unsigned)C16);
    const int oh = blockIdx.y;
    const uint4 *x4 = reinterpret_cast<const uint4 *>(x);
    uint4 *y4 = reinterpret_cast<uint4 *>(y);
    for (int64_t b = blockIdx.z; b < B; b += gridDim.z) {
        uint32_t even[4], odd[4];            // bytes 0, 2 and bytes 1, 3 of each dword, as value * 256 in 16 bits
#pragma unroll
        for (int i = 0; i < 4; ++i) even[i] = odd[i] = 0x80008000u;       // -128
        for (int kh = 0; kh < ksize; ++kh) {
            const int ih = oh * stride - pad + kh;
            if ((unsigned)ih >= (unsigned)H) continue;
            for (int kw = 0; kw < ksize; ++kw) {
                const int iw = ow * stride - pad + kw;
                if ((unsigned)iw >= (unsigned)W) continue;
                const uint4 v = x4[((b * H + ih) * W + iw) * C16 + c16];
                const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t e = (d[i] << 8) & 0xFF00FF00u, o = d[i] & 0xFF00FF00u;
                    const p_v2s me = __builtin_elementwise_max(__builtin_bit_cast(p_v2s, even[i]), __builtin_bit_cast(p_v2s, e));
                    const p_v2s mo = __builtin_elementwise_max(__builtin_bit_cast(p_v2s, odd[i]), __builtin_bit_cast(p_v2s, o));
                    even[i] = __builtin_bit_cast(uint32_t, me);
                    odd[i] = __builtin_bit_cast(uint32_t, mo);
                }
            }
        }
        uint32_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (odd[i] & 0xFF00FF00u) | ((even[i] >> 8) & 0x00FF00FFu);
        y4[((b * Ho + oh) * Wo + ow) * C16 + c16] = make_uint4(r[0], r[1], r[2], r[3]);
    }
}

// One thread per channel of one output pixel (any C, any alignment).
__global__ void __launch_bounds__(256) k_maxpool_i8(const int8_t *__restrict__ x, int64_t total, int H, int W, int C,
                                                     int Ho, int Wo, int ksize, int stride, int pad,
                                                     int8_t *__restrict__ y)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % C);
    int64_t rest = idx / C;
    const int ow = (int)(rest % Wo); rest /= Wo;
    const int oh = (int)(rest % Ho);
    const int64_t b = rest / Ho;
    int best = -128;
    for (int kh = 0; kh < ksize; ++kh)
        for (int kw = 0; kw < ksize; ++kw) {
            const int ih = oh * stride - pad + kh, iw = ow * stride - pad + kw;
            if ((unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W) {
                const int v = x[((b * H + ih) * W + iw) * C + c];
                best = v > best ? v : best;
            }
        }
    y[idx] = (int8_t)best;
}

// One thread per (image, channel); consecutive threads read consecutive channels.
__global__ void __launch_bounds__(256) k_avgpool_i8(const int8_t *__restrict__ x, int64_t B, int64_t HW, int64_t C,
                                                     float in_scale, float inv_out_scale, int8_t *__restrict__ y)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * C) return;
    const int64_t b = idx / C, c = idx % C;
    int sum = 0;
    for (int64_t p = 0; p < HW; ++p) sum += x[(b * HW + p) * C + c];
    const float k = in_scale / (float)HW;
    const float v = (float)sum * k;
    float q = rintf(v * inv_out_scale);
    q = fminf(fmaxf(q, -128.0f), 127.0f);
    y[idx] = (int8_t)(int)q;
}

}  // namespace nq

using namespace nq;

extern "C" nq_status nq_maxpool_i8(const int8_t *d_x, int64_t B, int64_t H, int64_t W, int64_t C, int ksize,
                                   int stride, int pad, int8_t *d_y, void *stream)
{
    if (B < 0 || H < 1 || W < 1 || C < 1 || ksize < 1 || stride < 1 || pad < 0) return NQ_ERR_INVALID_ARG;
    if (H > 32768 || W > 32768 || C > NQ_MAX_K || ksize > 64 || pad >= ksize) return NQ_ERR_SHAPE;
    if (H + 2 * pad < ksize || W + 2 * pad < ksize) return NQ_ERR_SHAPE;
    const int64_t Ho = (H + 2 * pad - ksize) / stride + 1, Wo = (W + 2 * pad - ksize) / stride + 1;
    const int64_t total = B * Ho * Wo * C;
    if (total == 0) return NQ_OK;
    if (!d_x || !d_y) return NQ_ERR_INVALID_ARG;
    if (C % 16 == 0 && aligned16(d_x) && aligned16(d_y) && Wo * (C / 16) < 0x7fffffffLL && Ho <= 65535) {
        const dim3 grid((unsigned)ceil_div(Wo * (C / 16), 256), (unsigned)Ho, (unsigned)(B < 65535 ? B : 65535));
        hipLaunchKernelGGL(k_maxpool_i8_v16, grid, dim3(256), 0, (hipStream_t)stream, d_x, B, (int)H, (int)W,
                           (int)(C / 16), (int)Ho, (int)Wo, ksize, stride, pad, d_y);
        return launch_status();
    }
    if (ceil_div(total, 256) > 0x7fffffffLL) return NQ_ERR_SHAPE;
    hipLaunchKernelGGL(k_maxpool_i8, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, (hipStream_t)stream, d_x,
                       total, (int)H, (int)W, (int)C, (int)Ho, (int)Wo, ksize, stride, pad, d_y);
    return launch_status();
}

extern "C" nq_status nq_avgpool_i8(const int8_t *d_x, int64_t B, int64_t HW, int64_t C, float in_scale,
                                   float inv_out_scale, int8_t *d_y, void *stream)
{
    if (B < 0 || HW < 1 || C < 1) return NQ_ERR_INVALID_ARG;
    if (HW > (1 << 24)) return NQ_ERR_SHAPE;
    if (B * C == 0) return NQ_OK;
    if (!d_x || !d_y) return NQ_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_avgpool_i8, dim3((unsigned)ceil_div(B * C, 256)), dim3(256), 0, (hipStream_t)stream, d_x, B,
                       HW, C, in_scale, inv_out_scale, d_y);
    return launch_status();
}
