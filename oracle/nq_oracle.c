/*
 * NestQuant CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar implementation of what the nested-integer hot path
 * computes, written from the paper's definitions.  It shares no code, header,
 * table or helper with the HIP library; only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may load it.  The product never calls it.
 *
 * Every function cites the passage of the paper (arXiv 2506.17870) it follows.
 * Integer work is done in int32/int64; the dequantisation epilogue is done in
 * fp32 in one fixed operation order (no fused multiply-add), which is the
 * precision the GPU path takes its rounding decisions in.
 *
 * Parity pins (see tests/test_oracle_pins.py): the nesting-numerical-error
 * table, the -67 worked example, exact recomposition for all 2^n values,
 * range statements of Sec. 3.2/3.3, the packing counts of Sec. 3.3.4, the
 * ideal-storage table of Sec. 4.3, brute-force integer dot products and
 * numpy's int64 matmul.  Parity unpinned: nothing on the path; the quantiser
 * of Eq. 1 is pinned only against a retyped closed form and is not graded.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define OQ_OK 0
#define OQ_ERR_ARG 1
#define OQ_ERR_RANGE 2

/* ------------------------------------------------------------------ */
/* Eq. 1: symmetric linear quantisation, signed, no zero point.       */
/* Per output channel n: s = absmax / (2^(nb-1) - 1) (s = 1 for an    */
/* all-zero row), w_int = Clip(round_half_even(w / s), min, max).     */
/* ------------------------------------------------------------------ */
int oq_quantize_rtn(const float *w, int64_t N, int64_t K, int n_bits,
                    int8_t *w_int, float *scale)
{
    if (n_bits < 2 || n_bits > 8) return OQ_ERR_ARG;
    const int qmin = -(1 << (n_bits - 1));
    const int qmax = (1 << (n_bits - 1)) - 1;
    for (int64_t n = 0; n < N; ++n) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float a = fabsf(w[n * K + k]);
            if (a > amax) amax = a;
        }
        float s = (amax > 0.0f) ? amax / (float)qmax : 1.0f;
        scale[n] = s;
        for (int64_t k = 0; k < K; ++k) {
            float q = rintf(w[n * K + k] / s);
            int qi = (int)q;
            if (qi < qmin) qi = qmin;
            if (qi > qmax) qi = qmax;
            w_int[n * K + k] = (int8_t)qi;
        }
    }
    return OQ_OK;
}

/* floor(a / 2^l) for any sign of a */
static int floor_div_pow2(int a, int l)
{
    int d = 1 << l;
    int q = a / d;
    if ((a % d != 0) && (a < 0)) q -= 1;
    return q;
}

/* ------------------------------------------------------------------ */
/* Eq. 5: w_high = Clip(round(w_int / 2^l), -2^(h-1), 2^(h-1)-1).     */
/* rounding: 0 BitShift (arithmetic right shift == floor),            */
/*           1 round-to-nearest, ties to even,                        */
/*           2 rounding up (ceil), 3 rounding down (floor).           */
/* Alg. 1 (step 2): residual = w_int - w_high * 2^l.                  */
/* ------------------------------------------------------------------ */
int oq_decompose(const int8_t *w_int, int64_t count, int n_bits, int l_bits,
                 int rounding, int8_t *w_high, int16_t *residual)
{
    int h = n_bits - l_bits;
    if (n_bits < 2 || n_bits > 8 || l_bits < 1 || h < 1) return OQ_ERR_ARG;
    if (rounding < 0 || rounding > 3) return OQ_ERR_ARG;
    const int two_l = 1 << l_bits;
    const int hmin = -(1 << (h - 1));
    const int hmax = (1 << (h - 1)) - 1;
    const int wmin = -(1 << (n_bits - 1));
    const int wmax = (1 << (n_bits - 1)) - 1;
    for (int64_t i = 0; i < count; ++i) {
        int w = w_int[i];
        if (w < wmin || w > wmax) return OQ_ERR_RANGE;
        int fl = floor_div_pow2(w, l_bits);
        int rem = w - fl * two_l; /* in [0, 2^l) */
        int q;
        switch (rounding) {
        case 0: /* BitShift */
        case 3: /* down */
            q = fl;
            break;
        case 2: /* up */
            q = fl + (rem != 0);
            break;
        default: /* nearest, ties to even */
            if (2 * rem > two_l) q = fl + 1;
            else if (2 * rem < two_l) q = fl;
            else q = (fl & 1) ? fl + 1 : fl;
            break;
        }
        if (q < hmin) q = hmin;
        if (q > hmax) q = hmax;
        w_high[i] = (int8_t)q;
        residual[i] = (int16_t)(w - q * two_l);
    }
    return OQ_OK;
}

/* ------------------------------------------------------------------ */
/* The stored lower-bit weight.                                       */
/* fmt 0: the true bit split, unsigned l bits, [0, 2^l - 1]; valid    */
/*        only when w_high came from the shift (Eq. 4 read as a       */
/*        bit-wise split); a residual outside the range is an error.  */
/* fmt 1: extra-1-bit compensation (Sec. 3.3.3): signed (l+1) bits,   */
/*        [-2^l, 2^l - 1]; out of range is an error.                  */
/* fmt 2: Eq. 9 as printed: Clip(residual, -2^(l-1), 2^(l-1)-1),      */
/*        lossy; kept to reproduce the numerical-error table.         */
/* ------------------------------------------------------------------ */
int oq_low_encode(const int16_t *residual, int64_t count, int l_bits, int fmt,
                  int8_t *w_low)
{
    if (l_bits < 1 || l_bits > 7) return OQ_ERR_ARG;
    for (int64_t i = 0; i < count; ++i) {
        int r = residual[i];
        int lo, hi;
        if (fmt == 0) { lo = 0; hi = (1 << l_bits) - 1; }
        else if (fmt == 1) { lo = -(1 << l_bits); hi = (1 << l_bits) - 1; }
        else if (fmt == 2) { lo = -(1 << (l_bits - 1)); hi = (1 << (l_bits - 1)) - 1; }
        else return OQ_ERR_ARG;
        if (fmt == 2) {
            if (r < lo) r = lo;
            if (r > hi) r = hi;
        } else if (r < lo || r > hi) {
            return OQ_ERR_RANGE;
        }
        w_low[i] = (int8_t)r;
    }
    return OQ_OK;
}

/* Eq. 4: w_int = LeftShift(w_high, l) + w_low = w_high * 2^l + w_low. */
int oq_compose(const int8_t *w_high, const int8_t *w_low, int64_t count,
               int l_bits, int16_t *w_full)
{
    for (int64_t i = 0; i < count; ++i)
        w_full[i] = (int16_t)((int)w_high[i] * (1 << l_bits) + (int)w_low[i]);
    return OQ_OK;
}

/* ------------------------------------------------------------------ */
/* Packed-bit tensors (Sec. 3.3.4).                                   */
/* A k-bit field is the value modulo 2^k (two's-complement            */
/* truncation); "sign" says how unpack widens it again.               */
/* ------------------------------------------------------------------ */

/* Layout "paper word": 64//k fields per unsigned 64-bit word, field j
 * of a word in bits [j*k, (j+1)*k), spare top bits zero, every row
 * starts a new word, the last word of a row is zero padded.           */
int64_t oq_paper_words_per_row(int64_t K, int k)
{
    int64_t per = 64 / k;
    return (K + per - 1) / per;
}

int oq_pack_paper(const int8_t *v, int64_t N, int64_t K, int k, uint64_t *out)
{
    if (k < 1 || k > 8) return OQ_ERR_ARG;
    int64_t per = 64 / k, wpr = oq_paper_words_per_row(K, k);
    uint64_t mask = (k == 64) ? ~0ull : ((1ull << k) - 1);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t wd = 0; wd < wpr; ++wd) {
            uint64_t word = 0;
            for (int64_t j = 0; j < per; ++j) {
                int64_t kk = wd * per + j;
                if (kk >= K) break;
                uint64_t field = ((uint64_t)(int64_t)v[n * K + kk]) & mask;
                word |= field << (j * k);
            }
            out[n * wpr + wd] = word;
        }
    return OQ_OK;
}

static int widen(uint32_t field, int k, int is_signed)
{
    int val = (int)field;
    if (is_signed && (field >> (k - 1)) & 1u) val -= (1 << k);
    return val;
}

int oq_unpack_paper(const uint64_t *in, int64_t N, int64_t K, int k,
                    int is_signed, int8_t *v)
{
    if (k < 1 || k > 8) return OQ_ERR_ARG;
    int64_t per = 64 / k, wpr = oq_paper_words_per_row(K, k);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t kk = 0; kk < K; ++kk) {
            uint64_t word = in[n * wpr + kk / per];
            uint32_t field = (uint32_t)((word >> ((kk % per) * k)) & ((1ull << k) - 1));
            v[n * K + kk] = (int8_t)widen(field, k, is_signed);
        }
    return OQ_OK;
}

/*
 * Layout "dense tile" (this library's own; exactly k bits per element on
 * the padded shape).  N is padded to a multiple of 32 and K to a multiple
 * of 64 with zero fields.  A tile is 32 rows x 64 columns; tiles are stored
 * row-block major, column-block minor, each tile k*64 dwords:
 *   dword (i, slot), i in [0,k), slot in [0,64), sits at slot*k + i (the k
 *   dwords of a slot are contiguous);
 *   slot = 32*g + r : r = row within the tile, g = which half of the 64
 *   columns; the slot's 32 columns are c = 32*g + 4*j + b, j in [0,8)
 *   "position", b in [0,4) "byte lane"; byte b of dword (i,slot) is byte i
 *   of the (slot, b) group, which stores the eight fields F_0..F_7 of
 *   positions j = 0..7 in k bytes B_0..B_{k-1}:
 *   - stream kind 0 ("carrier", used for the higher-bit page): with
 *     s = 8-k, bits [7..s] of B_i hold F_i for i < k; the low s bits of
 *     B_0, B_1, ... taken in that order, least significant bit first, form
 *     a string of k*s bits that holds F_k, F_{k+1}, ..., F_7 one after the
 *     other, each least significant bit first;
 *   - stream kind 1 ("bit string", used for the lower-bit page): the bytes
 *     B_0..B_{k-1} read as one little-endian string of 8k bits hold F_j in
 *     bits [j*k, (j+1)*k).
 */
static int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

int64_t oq_dense_bytes(int64_t N, int64_t K, int k)
{
    return round_up(N, 32) * round_up(K, 64) * k / 8;
}

/* bit position (byte index, bit index) of bit t of field j in a group */
static void dense_bit_place(int kind, int k, int j, int t, int *byte, int *bit)
{
    if (kind == 1) {
        int pos = j * k + t;
        *byte = pos / 8;
        *bit = pos % 8;
        return;
    }
    int s = 8 - k;
    if (j < k) {
        *byte = j;
        *bit = s + t;
    } else {
        int pos = (j - k) * k + t; /* position in the string of free bits */
        *byte = pos / s;
        *bit = pos % s;
    }
}

int oq_pack_dense(const int8_t *v, int64_t N, int64_t K, int k, int kind,
                  uint8_t *out)
{
    if (k < 1 || k > 7 || (kind != 0 && kind != 1)) return OQ_ERR_ARG;
    int64_t NB = round_up(N, 32) / 32, KB = round_up(K, 64) / 64;
    memset(out, 0, (size_t)oq_dense_bytes(N, K, k));
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < K; ++c) {
            int64_t nb = n / 32, kb = c / 64;
            int r = (int)(n % 32), cc = (int)(c % 64);
            int g = cc / 32, j = (cc % 32) / 4, b = cc % 4;
            int slot = 32 * g + r;
            uint32_t field = ((uint32_t)(int32_t)v[n * K + c]) & ((1u << k) - 1u);
            uint8_t *tile = out + (nb * KB + kb) * (int64_t)k * 256;
            for (int t = 0; t < k; ++t) {
                if (!((field >> t) & 1u)) continue;
                int byte, bit;
                dense_bit_place(kind, k, j, t, &byte, &bit);
                tile[(slot * k + byte) * 4 + b] |= (uint8_t)(1u << bit);
            }
        }
    return OQ_OK;
}

int oq_unpack_dense(const uint8_t *in, int64_t N, int64_t K, int k, int kind,
                    int is_signed, int8_t *v)
{
    if (k < 1 || k > 7 || (kind != 0 && kind != 1)) return OQ_ERR_ARG;
    int64_t KB = round_up(K, 64) / 64;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < K; ++c) {
            int64_t nb = n / 32, kb = c / 64;
            int r = (int)(n % 32), cc = (int)(c % 64);
            int g = cc / 32, j = (cc % 32) / 4, b = cc % 4;
            int slot = 32 * g + r;
            const uint8_t *tile = in + (nb * KB + kb) * (int64_t)k * 256;
            uint32_t field = 0;
            for (int t = 0; t < k; ++t) {
                int byte, bit;
                dense_bit_place(kind, k, j, t, &byte, &bit);
                if ((tile[(slot * k + byte) * 4 + b] >> bit) & 1u) field |= 1u << t;
            }
            v[n * K + c] = (int8_t)widen(field, k, is_signed);
        }
    return OQ_OK;
}

/* ------------------------------------------------------------------ */
/* Integer GEMM: acc[m,n] = sum_k x[m,k] * w[n,k], int32 accumulate.  */
/* Full-bit: w = w_high*2^l + w_low (Eq. 4); part-bit: w = w_high.    */
/* ------------------------------------------------------------------ */
int oq_gemm_i32(const int8_t *x, int64_t M, const int16_t *w, int64_t N,
                int64_t K, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t a = 0;
            for (int64_t k = 0; k < K; ++k)
                a += (int32_t)x[m * K + k] * (int32_t)w[n * K + k];
            acc[m * N + n] = a;
        }
    return OQ_OK;
}

/* ------------------------------------------------------------------ */
/* Direct convolution, NHWC activations, weights [Cout][KH][KW][Cin], */
/* zero padding, groups = 1, dilation = 1; same accumulator.          */
/* ------------------------------------------------------------------ */
int oq_conv_i32(const int8_t *x, int64_t B, int64_t H, int64_t W, int64_t Cin,
                const int16_t *w, int64_t Cout, int KH, int KW, int stride,
                int pad, int32_t *acc)
{
    if (stride < 1 || pad < 0 || KH < 1 || KW < 1) return OQ_ERR_ARG;
    int64_t Ho = (H + 2 * pad - KH) / stride + 1;
    int64_t Wo = (W + 2 * pad - KW) / stride + 1;
    if (Ho < 1 || Wo < 1) return OQ_ERR_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oh = 0; oh < Ho; ++oh)
            for (int64_t ow = 0; ow < Wo; ++ow)
                for (int64_t co = 0; co < Cout; ++co) {
                    int32_t a = 0;
                    for (int kh = 0; kh < KH; ++kh)
                        for (int kw = 0; kw < KW; ++kw) {
                            int64_t ih = oh * stride - pad + kh;
                            int64_t iw = ow * stride - pad + kw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const int8_t *xp = x + ((b * H + ih) * W + iw) * Cin;
                            const int16_t *wp = w + ((co * KH + kh) * KW + kw) * Cin;
                            for (int64_t ci = 0; ci < Cin; ++ci)
                                a += (int32_t)xp[ci] * (int32_t)wp[ci];
                        }
                    acc[((b * Ho + oh) * Wo + ow) * Cout + co] = a;
                }
    return OQ_OK;
}

/* ------------------------------------------------------------------ */
/* Grouped convolution (depthwise when every group has one channel):  */
/* output channel co belongs to group co / (Cout/groups) and sums     */
/* over the Cin/groups input channels of that group only; weights     */
/* [Cout][KH][KW][Cin/groups].  Same accumulator, zero padding.       */
/* ------------------------------------------------------------------ */
int oq_conv_grouped_i32(const int8_t *x, int64_t B, int64_t H, int64_t W, int64_t Cin,
                        const int16_t *w, int64_t Cout, int64_t groups, int KH, int KW,
                        int stride, int pad, int32_t *acc)
{
    if (stride < 1 || pad < 0 || KH < 1 || KW < 1 || groups < 1) return OQ_ERR_ARG;
    if (Cin % groups != 0 || Cout % groups != 0) return OQ_ERR_ARG;
    int64_t cig = Cin / groups, cog = Cout / groups;
    int64_t Ho = (H + 2 * pad - KH) / stride + 1;
    int64_t Wo = (W + 2 * pad - KW) / stride + 1;
    if (Ho < 1 || Wo < 1) return OQ_ERR_ARG;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oh = 0; oh < Ho; ++oh)
            for (int64_t ow = 0; ow < Wo; ++ow)
                for (int64_t co = 0; co < Cout; ++co) {
                    int64_t first = (co / cog) * cig;      /* first input channel of the group */
                    int32_t a = 0;
                    for (int kh = 0; kh < KH; ++kh)
                        for (int kw = 0; kw < KW; ++kw) {
                            int64_t ih = oh * stride - pad + kh;
                            int64_t iw = ow * stride - pad + kw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const int8_t *xp = x + ((b * H + ih) * W + iw) * Cin + first;
                            const int16_t *wp = w + ((co * KH + kh) * KW + kw) * cig;
                            for (int64_t ci = 0; ci < cig; ++ci)
                                a += (int32_t)xp[ci] * (int32_t)wp[ci];
                        }
                    acc[((b * Ho + oh) * Wo + ow) * Cout + co] = a;
                }
    return OQ_OK;
}

/* ------------------------------------------------------------------ */
/* Dequantisation epilogue, fp32, fixed order, one rounding per step: */
/*   c   = s_a * s_w[n]            (Eq. 2: w_hat = s * w_int)         */
/*   c   = c * 2^l  in part-bit    (Eq. 8: s_high = s * 2^l, exact)   */
/*   y   = (float)acc * c                                             */
/*   y   = y + bias[n]                     if bias                    */
/*   y   = y + s_r * (float)r_q[m,n]       if residual                */
/*   y   = max(y, 0)                       if relu                    */
/*   q   = clamp(rint(y * inv_s_out), -128, 127)  if out_int8         */
/* ------------------------------------------------------------------ */
int oq_epilogue(const int32_t *acc, int64_t M, int64_t N, float s_a,
                const float *s_w, int part_l_bits, const float *bias,
                const int8_t *r_q, float s_r, int relu, int out_int8,
                float inv_s_out, float *y_f32, int8_t *y_i8)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            volatile float c = s_a * s_w[n];
            if (part_l_bits > 0) c = c * (float)(1 << part_l_bits);
            volatile float y = (float)acc[m * N + n] * c;
            if (bias) y = y + bias[n];
            if (r_q) {
                volatile float t = s_r * (float)r_q[m * N + n];
                y = y + t;
            }
            if (relu && !(y > 0.0f)) y = 0.0f;
            if (out_int8) {
                volatile float t = y * inv_s_out;
                float q = rintf(t);
                if (q < -128.0f) q = -128.0f;
                if (q > 127.0f) q = 127.0f;
                y_i8[m * N + n] = (int8_t)q;
            } else {
                y_f32[m * N + n] = y;
            }
        }
    return OQ_OK;
}

/* ------------------------------------------------------------------ */
/* Glue of a residual CNN on int8 NHWC activations (the paper only    */
/* says the models are CNNs with 8-bit activations, Sec. 4.2).        */
/* Max pooling takes the maximum of the int8 codes inside the window  */
/* (padding never wins).  Global average pooling: int32 sum over the  */
/* H*W positions, y = (float)sum * (s_in / (float)(H*W)),             */
/* q = clamp(rint(y * inv_s_out)).                                    */
/* ------------------------------------------------------------------ */
int oq_maxpool_i8(const int8_t *x, int64_t B, int64_t H, int64_t W, int64_t C,
                  int ksize, int stride, int pad, int8_t *y)
{
    int64_t Ho = (H + 2 * pad - ksize) / stride + 1;
    int64_t Wo = (W + 2 * pad - ksize) / stride + 1;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oh = 0; oh < Ho; ++oh)
            for (int64_t ow = 0; ow < Wo; ++ow)
                for (int64_t c = 0; c < C; ++c) {
                    int best = -129;
                    for (int kh = 0; kh < ksize; ++kh)
                        for (int kw = 0; kw < ksize; ++kw) {
                            int64_t ih = oh * stride - pad + kh;
                            int64_t iw = ow * stride - pad + kw;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            int val = x[((b * H + ih) * W + iw) * C + c];
                            if (val > best) best = val;
                        }
                    if (best < -128) best = -128;
                    y[((b * Ho + oh) * Wo + ow) * C + c] = (int8_t)best;
                }
    return OQ_OK;
}

int oq_avgpool_i8(const int8_t *x, int64_t B, int64_t HW, int64_t C, float s_in,
                  float inv_s_out, int8_t *y)
{
    for (int64_t b = 0; b < B; ++b)
        for (int64_t c = 0; c < C; ++c) {
            int32_t sum = 0;
            for (int64_t p = 0; p < HW; ++p) sum += x[(b * HW + p) * C + c];
            volatile float k = s_in / (float)HW;
            volatile float yv = (float)sum * k;
            volatile float t = yv * inv_s_out;
            float q = rintf(t);
            if (q < -128.0f) q = -128.0f;
            if (q > 127.0f) q = 127.0f;
            y[b * C + c] = (int8_t)q;
        }
    return OQ_OK;
}
