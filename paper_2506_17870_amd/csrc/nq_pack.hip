// Integer weight decomposition and packing kernels (paper Sec. 3.2.1 Eq. 4-5, Alg. 1
// steps 2-3, Sec. 3.3.4).  All kernels are elementwise streams bound by HBM bandwidth:
// one byte read and (h + l)/8 bytes written per weight for the fused decompose-and-pack.
#include "nq_codec.h"
#include "nq_common.h"

namespace nq {

// ---------------------------------------------------------------------------------------
// Eq. 5 (BitShift) and Alg. 1 step 2, unpacked: high = w >> l, low = w - high * 2^l.
// 16 weights per thread, four per dword.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t sar_bytes(uint32_t x, int l)
{
    // arithmetic right shift of four int8 lanes: logical shift, then sign fill
    const uint32_t keep = rep4(0xFFu >> l);
    const uint32_t sign = x & 0x80808080u;
    const uint32_t fill = (sign >> 7) * (0xFFu & ~(0xFFu >> l));
    return ((x >> l) & keep) | fill;
}

// Compensated decomposition (Sec. 3.3.3, Alg. 1 step 2 with round-to-nearest instead of the shift):
// w_high = clip(round_half_even(w / 2^l)) to h bits, w_low = w - w_high * 2^l, which lies in
// [-2^l + 1, 2^l - 1] and needs l + 1 signed bits.  v is the INT-n value.
__host__ __device__ __forceinline__ void split_rtn(int v, int l, int h, int *high, int *low)
{
    int q = v >> l;                                     // floor
    const int r = v - (q << l), half = 1 << (l - 1);
    if (r > half || (r == half && (q & 1))) ++q;
    const int top = (1 << (h - 1)) - 1;
    if (q > top) q = top;                               // (the bottom cannot be passed: floor >= -2^(h-1))
    *high = q;
    *low = v - (q << l);
}

__global__ void __launch_bounds__(256) k_decompose(const int8_t *__restrict__ w, int64_t count, int n_bits,
                                                    int l, int8_t *__restrict__ high,
                                                    int8_t *__restrict__ low, int vec_ok, int sgn)
{
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t base = tid * 16;
    if (base >= count) return;
    if (sgn) {
        for (int64_t i = base; i < count && i < base + 16; ++i) {
            const int v = (int8_t)((uint8_t)w[i] << (8 - n_bits)) >> (8 - n_bits);   // INT-n value, sign extended
            int hi, lo;
            split_rtn(v, l, n_bits - l, &hi, &lo);
            high[i] = (int8_t)hi;
            low[i] = (int8_t)lo;
        }
        return;
    }
    const uint32_t lowmask = rep4((1u << l) - 1u);
    const int up = 8 - n_bits;  // an INT6 value is first moved to the top of its byte
    if (vec_ok && base + 16 <= count) {
        const uint4 v = *reinterpret_cast<const uint4 *>(w + base);
        uint32_t x[4] = {v.x, v.y, v.z, v.w}, hi[4], lo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t top = (x[i] << up) & rep4(0xFFu << up);
            hi[i] = sar_bytes(top, l + up);
            lo[i] = x[i] & lowmask;
        }
        *reinterpret_cast<uint4 *>(high + base) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        *reinterpret_cast<uint4 *>(low + base) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    } else {
        for (int64_t i = base; i < count && i < base + 16; ++i) {
            const int v = (int8_t)((uint8_t)w[i] << up);
            high[i] = (int8_t)(v >> (l + up));
            low[i] = (int8_t)(w[i] & ((1 << l) - 1));
        }
    }
}

// ---------------------------------------------------------------------------------------
// Dense-tile pack.  One wave per tile of 32 rows x 64 columns, one lane per slot: the lane
// reads the 32 consecutive weights of its slot and writes H dwords of the higher-bit page
// and L dwords of the lower-bit page; a wave's stores are 256 contiguous bytes each.
// SRC 0: from w_int (fused decomposition); SRC 1: from separate high / low tensors; SRC 2: from fp32
// weights (a) and their channel scales (b), quantised on the way (Eq. 1).
// ---------------------------------------------------------------------------------------
template <int H, int L, int SRC>
__device__ __forceinline__ void pack_dense_tile(const int8_t *__restrict__ a, const int8_t *__restrict__ b,
                                                int64_t N, int64_t K, int64_t KB, int64_t tile,
                                                uint32_t *__restrict__ ph, uint32_t *__restrict__ pl,
                                                int vec_ok, int sgn)
{
    constexpr int S = 8 - H;        // spare bits of a carrier byte
    constexpr int UP = 8 - H - L;   // 0 for INT8 nesting, 2 for INT6 nesting
    const int lane = threadIdx.x & 63;
    const int64_t nb = tile / KB, kb = tile % KB;
    const int r = lane & 31, g = lane >> 5;
    const int64_t n = nb * 32 + r;
    const int64_t c0 = kb * 64 + 32 * g;

    // ---- the slot's 32 elements, four per dword; zero outside the matrix ------------------------
    // A: the INT-n codes (SRC 0, 2) or w_high (SRC 1); B: w_low (SRC 1)
    uint32_t A[8], B[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) A[j] = B[j] = 0;
    if (n < N) {
        if constexpr (SRC == 2) {
            // Eq. 1 with the channel's scale: IEEE fp32 quotient, round half to even, clip
            const float *wf = reinterpret_cast<const float *>(a) + n * K;
            const float sc = reinterpret_cast<const float *>(b)[n];
            const int qmin = -(1 << (H + L - 1)), qmax = (1 << (H + L - 1)) - 1;
            auto code = [&](float v) {
                const int q = (int)__builtin_rintf(v / sc);
                return (uint32_t)(min(max(q, qmin), qmax) & 0xFF);
            };
            if (vec_ok && c0 + 32 <= K) {
                const float4 *pv = reinterpret_cast<const float4 *>(wf + c0);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float4 v = pv[j];
                    A[j] = code(v.x) | (code(v.y) << 8) | (code(v.z) << 16) | (code(v.w) << 24);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    for (int bb = 0; bb < 4; ++bb) {
                        const int64_t c = c0 + 4 * j + bb;
                        if (c < K) A[j] |= code(wf[c]) << (8 * bb);
                    }
            }
        } else if (vec_ok && c0 + 32 <= K) {
            const uint4 *pa = a ? reinterpret_cast<const uint4 *>(a + n * K + c0) : nullptr;
            const uint4 *pb = (SRC == 1 && b) ? reinterpret_cast<const uint4 *>(b + n * K + c0) : nullptr;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                uint4 va = pa ? pa[q] : make_uint4(0, 0, 0, 0);
                A[4 * q + 0] = va.x; A[4 * q + 1] = va.y; A[4 * q + 2] = va.z; A[4 * q + 3] = va.w;
                uint4 vb = pb ? pb[q] : make_uint4(0, 0, 0, 0);
                B[4 * q + 0] = vb.x; B[4 * q + 1] = vb.y; B[4 * q + 2] = vb.z; B[4 * q + 3] = vb.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t wa = 0, wb = 0;
                for (int bb = 0; bb < 4; ++bb) {
                    const int64_t c = c0 + 4 * j + bb;
                    if (c < K) {
                        if (a) wa |= (uint32_t)(uint8_t)a[n * K + c] << (8 * bb);
                        if (SRC == 1 && b) wb |= (uint32_t)(uint8_t)b[n * K + c] << (8 * bb);
                    }
                }
                A[j] = wa; B[j] = wb;
            }
        }
    }

    if (sgn) {
        // compensated format: fields of h and l + 1 bits from (w_high, signed w_low), which unless given
        // (SRC 1) are split off the codes with round-to-nearest first; byte by byte (not the measured path)
        uint32_t X[8], XL[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            X[j] = XL[j] = 0;
            for (int bb = 0; bb < 4; ++bb) {
                int hi, lo;
                if (SRC != 1) {
                    const int v = (int8_t)((uint8_t)(A[j] >> (8 * bb)) << UP) >> UP;
                    split_rtn(v, L, H, &hi, &lo);
                } else {
                    hi = (int8_t)(A[j] >> (8 * bb));
                    lo = (int8_t)(B[j] >> (8 * bb));
                }
                X[j] |= (((uint32_t)hi << S) & 0xFFu) << (8 * bb);
                XL[j] |= (((uint32_t)lo & ((2u << L) - 1u)) << (S - L)) << (8 * bb);
            }
        }
        if (ph) {
            uint32_t P[H];
            HighCodec<H>::encode(X, P);
#pragma unroll
            for (int i = 0; i < H; ++i) ph[tile * (H * 64) + lane * H + i] = P[i];
        }
        if (pl) {
            uint32_t Q[L + 1];
            LowCodec<L + 1, S + 1>::encode(XL, Q);
#pragma unroll
            for (int i = 0; i < L + 1; ++i) pl[tile * ((L + 1) * 64) + lane * (L + 1) + i] = Q[i];
        }
        return;
    }
    uint32_t X[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (SRC != 1) {
            X[j] = (A[j] << UP) & rep4(0xFFu << UP);
        } else {
            X[j] = ((A[j] << S) & HighCodec<H>::HM) | ((B[j] << (S - L)) & LowCodec<L, S>::LM);
        }
    }
    if (ph) {
        uint32_t P[H];
        HighCodec<H>::encode(X, P);
        uint32_t *dst = ph + tile * (H * 64) + lane * H;
#pragma unroll
        for (int i = 0; i < H; ++i) dst[i] = P[i];
    }
    if (pl) {
        uint32_t Q[L];
        LowCodec<L, S>::encode(X, Q);
        uint32_t *dst = pl + tile * (L * 64) + lane * L;
#pragma unroll
        for (int i = 0; i < L; ++i) dst[i] = Q[i];
    }
}

template <int H, int L, int SRC>
__global__ void __launch_bounds__(256) k_pack_dense(const int8_t *__restrict__ a, const int8_t *__restrict__ b,
                                                     int64_t N, int64_t K, int64_t KB, int64_t tiles,
                                                     uint32_t *__restrict__ ph, uint32_t *__restrict__ pl,
                                                     int vec_ok, int sgn)
{
    const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= tiles) return;
    pack_dense_tile<H, L, SRC>(a, b, N, K, KB, tile, ph, pl, vec_ok, sgn);
}

// Many tensors in one launch (the weights of a whole model): the jobs travel by value in the kernel
// arguments, with the running count of their tiles; a wave finds its job by searching that count.
constexpr int PACK_BATCH = 64;
struct PackBatch {
    const int8_t *w[PACK_BATCH];
    uint32_t *ph[PACK_BATCH];
    uint32_t *pl[PACK_BATCH];
    int N[PACK_BATCH], K[PACK_BATCH];
    int64_t first_tile[PACK_BATCH + 1];      // tiles of jobs 0 .. j-1; entries past `count` repeat the total
    int count;
};

template <int H, int L>
__global__ void __launch_bounds__(256) k_pack_dense_batch(const PackBatch jobs, int sgn)
{
    const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= jobs.first_tile[jobs.count]) return;
    int lo = 0, hi = jobs.count - 1;                      // last job whose first tile is <= tile
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (jobs.first_tile[mid] <= tile) lo = mid;
        else hi = mid - 1;
    }
    const int64_t N = jobs.N[lo], K = jobs.K[lo];
    const int8_t *w = jobs.w[lo];
    const int vec_ok = (K % 16 == 0) && ((reinterpret_cast<uintptr_t>(w) & 15u) == 0);
    pack_dense_tile<H, L, 0>(w, nullptr, N, K, (K + 63) / 64, tile - jobs.first_tile[lo], jobs.ph[lo], jobs.pl[lo],
                             vec_ok, sgn);
}

// ---------------------------------------------------------------------------------------
// Eq. 1: channel scales and codes.  k_row_absmax: one block per row, 16-byte loads where the
// row allows; the scale is absmax / qmax (1 for an all-zero row).  k_quantize_codes: one
// block per 1024 elements of a row.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_row_absmax(const float *__restrict__ w, int64_t K, float qmax,
                                                     float *__restrict__ scale, int vec_ok)
{
    __shared__ float part[4];
    const float *row = w + (int64_t)blockIdx.x * K;
    float m = 0.0f;
    if (vec_ok) {
        const float4 *rv = reinterpret_cast<const float4 *>(row);
        for (int64_t i = threadIdx.x; i < K / 4; i += 256) {
            const float4 v = rv[i];
            m = fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
        }
    } else {
        for (int64_t i = threadIdx.x; i < K; i += 256) m = fmaxf(m, fabsf(row[i]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
        scale[blockIdx.x] = m > 0.0f ? m / qmax : 1.0f;
    }
}

__global__ void __launch_bounds__(256) k_quantize_codes(const float *__restrict__ w, int64_t K, int64_t chunks,
                                                         int n_bits, const float *__restrict__ scale,
                                                         int8_t *__restrict__ w_int, int vec_ok)
{
    const int64_t n = blockIdx.x / chunks, c0 = (blockIdx.x % chunks) * 1024 + threadIdx.x * 4;
    if (c0 >= K) return;
    const float sc = scale[n];
    const int qmin = -(1 << (n_bits - 1)), qmax = (1 << (n_bits - 1)) - 1;
    auto code = [&](float v) { return (uint32_t)(min(max((int)__builtin_rintf(v / sc), qmin), qmax) & 0xFF); };
    const float *src = w + n * K + c0;
    int8_t *dst = w_int + n * K + c0;
    if (vec_ok) {        // K % 4 == 0: the four elements are inside the row
        const float4 v = *reinterpret_cast<const float4 *>(src);
        *reinterpret_cast<uint32_t *>(dst) = code(v.x) | (code(v.y) << 8) | (code(v.z) << 16) | (code(v.w) << 24);
    } else {
        for (int i = 0; i < 4 && c0 + i < K; ++i) dst[i] = (int8_t)code(src[i]);
    }
}

// Dense-tile unpack: pages -> int8 parts.  A lane holds 32 consecutive elements of one row as eight dwords;
// the fields are moved to the bottom of their bytes and sign extended four bytes at a time, and leave as two
// 16-byte stores where the row allows (vec_ok: K a multiple of 16, 16-byte aligned outputs), else byte by byte.
__device__ __forceinline__ void unpack_store32(int8_t *__restrict__ dst, int64_t c0, int64_t K, const uint32_t (&V)[8],
                                               int vec_ok)
{
    if (vec_ok && c0 + 32 <= K) {
        uint4 *d4 = reinterpret_cast<uint4 *>(dst + c0);
        d4[0] = make_uint4(V[0], V[1], V[2], V[3]);
        d4[1] = make_uint4(V[4], V[5], V[6], V[7]);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            for (int bb = 0; bb < 4; ++bb) {
                const int64_t c = c0 + 4 * j + bb;
                if (c < K) dst[c] = (int8_t)(V[j] >> (8 * bb));
            }
    }
}

// Bytes that hold a field of `bits` bits at their bottom (zeros above): the same bytes sign extended.
template <int BITS>
__device__ __forceinline__ uint32_t sext_bytes(uint32_t t)
{
    constexpr uint32_t above = (0xFFu << BITS) & 0xFFu;              // the bits of a byte above the field
    const uint32_t sign = (t >> (BITS - 1)) & 0x01010101u;           // 1 in every byte whose field is negative
    return t | sign * above;                                          // no carries: 1 * above < 256
}

template <int H, int L>
__global__ void __launch_bounds__(256) k_unpack_dense(const uint32_t *__restrict__ ph,
                                                       const uint32_t *__restrict__ pl, int64_t N, int64_t K,
                                                       int64_t KB, int64_t tiles, int8_t *__restrict__ high,
                                                       int8_t *__restrict__ low, int sgn, int vec_ok)
{
    constexpr int S = 8 - H;
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= tiles) return;
    const int64_t nb = tile / KB, kb = tile % KB;
    const int r = lane & 31, g = lane >> 5;
    const int64_t n = nb * 32 + r;
    const int64_t c0 = kb * 64 + 32 * g;
    if (n >= N) return;
    if (ph && high) {
        uint32_t P[H], D[8], V[8];
#pragma unroll
        for (int i = 0; i < H; ++i) P[i] = ph[tile * (H * 64) + lane * H + i];
        HighCodec<H>::decode(P, D);
        // a decoded byte is w_high * 2^S: down by S, the neighbour's bits masked off, sign extended from h bits
#pragma unroll
        for (int j = 0; j < 8; ++j) V[j] = sext_bytes<H>((D[j] >> S) & rep4(0xFFu >> S));
        unpack_store32(high + n * K, c0, K, V, vec_ok);
    }
    if (pl && low && sgn) {
        uint32_t Q[L + 1], D[8], V[8];
#pragma unroll
        for (int i = 0; i < L + 1; ++i) Q[i] = pl[tile * ((L + 1) * 64) + lane * (L + 1) + i];
#pragma unroll
        for (int j = 0; j < 8; ++j) D[j] = 0;
        LowCodec<L + 1, S + 1>::decode_or(Q, D);
        // (l+1)-bit two's complement fields at bits [S-L, S+1) of their bytes
#pragma unroll
        for (int j = 0; j < 8; ++j) V[j] = sext_bytes<L + 1>((D[j] >> (S - L)) & rep4((2u << L) - 1u));
        unpack_store32(low + n * K, c0, K, V, vec_ok);
    } else if (pl && low) {
        uint32_t Q[L], D[8], V[8];
#pragma unroll
        for (int i = 0; i < L; ++i) Q[i] = pl[tile * (L * 64) + lane * L + i];
#pragma unroll
        for (int j = 0; j < 8; ++j) D[j] = 0;
        LowCodec<L, S>::decode_or(Q, D);
#pragma unroll
        for (int j = 0; j < 8; ++j) V[j] = (D[j] >> (S - L)) & rep4((1u << L) - 1u);
        unpack_store32(low + n * K, c0, K, V, vec_ok);
    }
}

// ---------------------------------------------------------------------------------------
// The paper's packed-bit tensor (Sec. 3.3.4): 64/k fields per unsigned 64-bit word.
// One thread per word.  part 0: fields are (w >> l) from w_int; 1: the low l bits of w_int;
// 2: the given values as they are; 3 / 4: the round-to-nearest w_high of w_int / its signed residual.
// ---------------------------------------------------------------------------------------
template <int KF>     // bits of a field
__global__ void __launch_bounds__(256) k_pack_paper(const int8_t *__restrict__ v, int64_t N, int64_t K,
                                                     int part, int l, int up, int64_t wpr, int64_t bpr,
                                                     uint64_t *__restrict__ out, int vec_ok)
{
    constexpr int k = KF;
    // A block packs 256 consecutive words of one row.  Their 256 * (64 / k) source bytes are brought into LDS
    // with 16-byte loads (from the 16-byte boundary below the first one) and each thread then collects the
    // bytes of its word there; reading them straight from memory, a wave's lanes are 64 / k bytes apart.
    // Byte i of the segment is at i + 4 * (i / 64): a wave's lanes, 64 / k bytes apart, then fall on different
    // banks whatever k is.
    __shared__ __attribute__((aligned(16))) int8_t seg[(256 * 64 + 16) / 64 * 68 + 68];
    auto at_seg = [](int64_t i) { return i + 4 * (i >> 6); };
    const int64_t n = blockIdx.x / bpr;
    const int64_t wd0 = (blockIdx.x - n * bpr) * 256;
    constexpr int per = 64 / k;
    const int64_t e0 = wd0 * per;                                     // first element of the block
    const int64_t e1 = e0 + 256 * per < K ? e0 + 256 * per : K;       // one past its last
    const int8_t *row = v + n * K;
    const int64_t a0 = vec_ok ? (e0 & ~int64_t(15)) : e0;
    if (vec_ok) {
        for (int64_t at = a0 + 16 * threadIdx.x; at < e1; at += 16 * 256) {     // K % 16 == 0: whole pieces
            const uint4 piece = *reinterpret_cast<const uint4 *>(row + at);
            uint32_t *dst = reinterpret_cast<uint32_t *>(seg + at_seg(at - a0));   // a piece never straddles 64
            dst[0] = piece.x; dst[1] = piece.y; dst[2] = piece.z; dst[3] = piece.w;
        }
    } else {
        for (int64_t at = a0 + threadIdx.x; at < e1; at += 256) seg[at_seg(at - a0)] = row[at];
    }
    __syncthreads();
    const int64_t wd = wd0 + threadIdx.x;
    if (wd >= wpr) return;
    const uint64_t mask = (1ull << k) - 1ull;
    uint64_t word = 0;
#pragma unroll
    for (int j = 0; j < per; ++j) {
        const int64_t c = wd * per + j;
        if (c >= K) continue;
        int val = seg[at_seg(c - a0)];
        if (part == 0) val = ((int8_t)((uint8_t)val << up)) >> (l + up);
        else if (part == 1) val = val & ((1 << l) - 1);
        else if (part == 3 || part == 4) {              // compensated split of w_int: its high / its low part
            int hi, lo;
            split_rtn(((int8_t)((uint8_t)val << up)) >> up, l, 8 - up - l, &hi, &lo);
            val = part == 3 ? hi : lo;
        }
        word |= ((uint64_t)(int64_t)val & mask) << (j * k);
    }
    out[n * wpr + wd] = word;
}

// One thread per 16 consecutive elements of a row: it walks through the words that hold them.
__global__ void __launch_bounds__(256) k_unpack_paper(const uint64_t *__restrict__ in, int64_t N, int64_t K,
                                                       int k, int is_signed, int64_t wpr, int64_t cpr,
                                                       int8_t *__restrict__ v, int vec_ok)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= N * cpr) return;
    const int64_t n = t / cpr;
    const int c0 = (int)(t - n * cpr) * 16;
    const int per = 64 / k;
    const uint32_t mask = (1u << k) - 1u, sign = 1u << (k - 1);
    const uint64_t *row = in + n * wpr;
    int wi = c0 / per, f = c0 - wi * per;
    uint64_t word = row[wi] >> (f * k);
    uint32_t V[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (c0 + i < K) {
            uint32_t field = (uint32_t)word & mask;
            if (is_signed && (field & sign)) field |= ~mask;          // two's complement of k bits
            V[i >> 2] |= (field & 0xFFu) << (8 * (i & 3));
            word >>= k;
            if (++f == per && c0 + i + 1 < K) { f = 0; word = row[++wi]; }
        }
    }
    int8_t *dst = v + n * K + c0;
    if (vec_ok && c0 + 16 <= K) {
        *reinterpret_cast<uint4 *>(dst) = make_uint4(V[0], V[1], V[2], V[3]);
    } else {
        for (int i = 0; i < 16 && c0 + i < K; ++i) dst[i] = (int8_t)(V[i >> 2] >> (8 * (i & 3)));
    }
}

template <int H, int L>
static void launch_pack_dense(int src, int sgn, const int8_t *a, const int8_t *b, int64_t N, int64_t K, void *ph,
                              void *pl, hipStream_t st)
{
    const int64_t NB = ceil_div(N, 32), KB = ceil_div(K, 64), tiles = NB * KB;
    if (tiles == 0) return;
    const int vec_ok = src == 2 ? (K % 4 == 0) && aligned16(a)
                                : (K % 16 == 0) && aligned16(a) && (b == nullptr || aligned16(b));
    const dim3 grid((unsigned)ceil_div(tiles, 4)), block(256);
    if (src == 2)
        hipLaunchKernelGGL((k_pack_dense<H, L, 2>), grid, block, 0, st, a, b, N, K, KB, tiles,
                           (uint32_t *)ph, (uint32_t *)pl, vec_ok, sgn);
    else if (src == 0)
        hipLaunchKernelGGL((k_pack_dense<H, L, 0>), grid, block, 0, st, a, b, N, K, KB, tiles,
                           (uint32_t *)ph, (uint32_t *)pl, vec_ok, sgn);
    else
        hipLaunchKernelGGL((k_pack_dense<H, L, 1>), grid, block, 0, st, a, b, N, K, KB, tiles,
                           (uint32_t *)ph, (uint32_t *)pl, vec_ok, sgn);
}

template <int H, int L>
static void launch_unpack_dense(int sgn, const void *ph, const void *pl, int64_t N, int64_t K, int8_t *high,
                                int8_t *low, hipStream_t st)
{
    const int64_t NB = ceil_div(N, 32), KB = ceil_div(K, 64), tiles = NB * KB;
    if (tiles == 0) return;
    const int vec_ok = (K % 16 == 0) && (high == nullptr || aligned16(high)) && (low == nullptr || aligned16(low));
    hipLaunchKernelGGL((k_unpack_dense<H, L>), dim3((unsigned)ceil_div(tiles, 4)), dim3(256), 0, st,
                       (const uint32_t *)ph, (const uint32_t *)pl, N, K, KB, tiles, high, low, sgn, vec_ok);
}

static nq_status check_pages(const nq_cfg *cfg, const void *ph, const void *pl)
{
    if ((ph && !aligned16(ph)) || (pl && !aligned16(pl))) return NQ_ERR_ALIGN;
    (void)cfg;
    return NQ_OK;
}

}  // namespace nq

using namespace nq;

extern "C" size_t nq_packed_bytes(int64_t N, int64_t K, int field_bits, int layout)
{
    if (N < 0 || K < 0) return 0;
    if (layout == NQ_LAYOUT_DENSE) {
        if (field_bits < 1 || field_bits > 7) return 0;
        return (size_t)(round_up(N, 32) * round_up(K, 64) * field_bits / 8);
    }
    if (layout == NQ_LAYOUT_PAPER_U64) {
        if (field_bits < 1 || field_bits > 8) return 0;
        return (size_t)(N * ceil_div(K, 64 / field_bits) * 8);
    }
    return 0;
}

static void launch_row_absmax(const float *d_w, int64_t N, int64_t K, int n_bits, float *d_scale, hipStream_t s)
{
    const int vec_ok = (K % 4 == 0) && aligned16(d_w);
    hipLaunchKernelGGL(k_row_absmax, dim3((unsigned)N), dim3(256), 0, s, d_w, K,
                       (float)((1 << (n_bits - 1)) - 1), d_scale, vec_ok);
}

extern "C" nq_status nq_quantize(const float *d_w, int64_t N, int64_t K, int n_bits, int8_t *d_w_int,
                                 float *d_scale, void *stream)
{
    if (n_bits < 2 || n_bits > 8) return NQ_ERR_INVALID_ARG;
    nq_status st = check_shape(N, K);
    if (st != NQ_OK) return st;
    if (N * K == 0) return NQ_OK;
    if (!d_w || !d_w_int || !d_scale) return NQ_ERR_INVALID_ARG;
    const int64_t chunks = ceil_div(K, 1024);
    if (N * chunks > 0x7fffffff) return NQ_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    launch_row_absmax(d_w, N, K, n_bits, d_scale, s);
    const int vec_ok = (K % 4 == 0) && aligned16(d_w) && ((uintptr_t)d_w_int % 4 == 0);
    hipLaunchKernelGGL(k_quantize_codes, dim3((unsigned)(N * chunks)), dim3(256), 0, s, d_w, K, chunks, n_bits,
                       d_scale, d_w_int, vec_ok);
    return launch_status();
}

// Eq. 1's step for a whole tensor (per-tensor activation quantisation): absmax over all elements through
// an atomic maximum on the bit patterns (non-negative floats order like unsigned integers), then one
// thread turns it into absmax / qmax (1 for an all-zero tensor).  d_scale doubles as the accumulator.
__global__ void k_tensor_absmax_begin(uint32_t *acc) { *acc = 0u; }

__global__ void __launch_bounds__(256) k_tensor_absmax(const float *__restrict__ x, int64_t count, int vec_ok,
                                                        uint32_t *__restrict__ acc)
{
    __shared__ float part[4];
    float m = 0.0f;
    const int64_t stride = (int64_t)gridDim.x * 256;
    if (vec_ok) {
        const float4 *xv = reinterpret_cast<const float4 *>(x);
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count / 4; i += stride) {
            const float4 v = xv[i];
            m = fmaxf(fmaxf(m, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
        }
        for (int64_t i = count / 4 * 4 + (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride)
            m = fmaxf(m, fabsf(x[i]));
    } else {
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) m = fmaxf(m, fabsf(x[i]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
        atomicMax(acc, __float_as_uint(m));
    }
}

__global__ void k_tensor_absmax_end(float *scale, float qmax)
{
    const float m = *scale;
    *scale = m > 0.0f ? m / qmax : 1.0f;
}

extern "C" nq_status nq_tensor_scale(const float *d_x, int64_t count, int n_bits, float *d_scale, void *stream)
{
    if (n_bits < 2 || n_bits > 8 || count < 0) return NQ_ERR_INVALID_ARG;
    if (!d_scale || (count > 0 && !d_x)) return NQ_ERR_INVALID_ARG;
    if (((uintptr_t)d_scale & 3u) != 0 || ((uintptr_t)d_x & 3u) != 0) return NQ_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_tensor_absmax_begin, dim3(1), dim3(1), 0, s, reinterpret_cast<uint32_t *>(d_scale));
    if (count > 0) {
        const int64_t blocks = ceil_div(count, 256 * 16);
        hipLaunchKernelGGL(k_tensor_absmax, dim3((unsigned)(blocks < 2048 ? blocks : 2048)), dim3(256), 0, s, d_x, count,
                           aligned16(d_x) ? 1 : 0, reinterpret_cast<uint32_t *>(d_scale));
    }
    hipLaunchKernelGGL(k_tensor_absmax_end, dim3(1), dim3(1), 0, s, d_scale, (float)((1 << (n_bits - 1)) - 1));
    return launch_status();
}

extern "C" nq_status nq_quantize_tensor(const float *d_x, int64_t count, int n_bits, int8_t *d_codes, float *d_scale,
                                        void *stream)
{
    if (count > 0 && !d_codes) return NQ_ERR_INVALID_ARG;
    if (ceil_div(count, 1024) > 0x7fffffff) return NQ_ERR_SHAPE;
    const nq_status st = nq_tensor_scale(d_x, count, n_bits, d_scale, stream);
    if (st != NQ_OK || count == 0) return st;
    // the whole tensor as one row of k_quantize_codes: 1024 elements per block, 16-byte loads where the pointers allow
    const int vec_ok = (count % 4 == 0) && aligned16(d_x) && ((uintptr_t)d_codes % 4 == 0);
    const int64_t chunks = ceil_div(count, 1024);
    hipLaunchKernelGGL(k_quantize_codes, dim3((unsigned)chunks), dim3(256), 0, (hipStream_t)stream, d_x, count, chunks,
                       n_bits, d_scale, d_codes, vec_ok);
    return launch_status();
}

extern "C" nq_status nq_quantize_decompose_pack(const float *d_w, int64_t N, int64_t K, const nq_cfg *cfg,
                                                float *d_scale, void *d_packed_high, void *d_packed_low,
                                                void *stream)
{
    nq_status st = check_cfg(cfg);
    if (st != NQ_OK) return st;
    if (cfg->layout != NQ_LAYOUT_DENSE) return NQ_ERR_UNSUPPORTED;
    if ((st = check_shape(N, K)) != NQ_OK) return st;
    if ((st = check_pages(cfg, d_packed_high, d_packed_low)) != NQ_OK) return st;
    if (N * K == 0) return NQ_OK;
    if (!d_w || !d_scale) return NQ_ERR_INVALID_ARG;
    if (N > 0x7fffffff) return NQ_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    launch_row_absmax(d_w, N, K, cfg->n_bits, d_scale, s);
    const int h = cfg->n_bits - cfg->l_bits, l = cfg->l_bits;
    const int sgn = cfg->low_format == NQ_LOW_SIGNED_L1;
    NQ_DISPATCH_HL(h, l, launch_pack_dense, 2, sgn, reinterpret_cast<const int8_t *>(d_w),
                   reinterpret_cast<const int8_t *>(d_scale), N, K, d_packed_high, d_packed_low, s);
    return launch_status();
}

extern "C" nq_status nq_decompose(const int8_t *d_w_int, int64_t N, int64_t K, const nq_cfg *cfg,
                                  int8_t *d_high, int8_t *d_low, void *stream)
{
    nq_status st = check_cfg(cfg);
    if (st != NQ_OK) return st;
    if ((st = check_shape(N, K)) != NQ_OK) return st;
    const int64_t count = N * K;
    if (count == 0) return NQ_OK;
    if (!d_w_int || !d_high || !d_low) return NQ_ERR_INVALID_ARG;
    const int vec_ok = aligned16(d_w_int) && aligned16(d_high) && aligned16(d_low);
    const int64_t threads = ceil_div(count, 16);
    hipLaunchKernelGGL(k_decompose, dim3((unsigned)ceil_div(threads, 256)), dim3(256), 0, (hipStream_t)stream,
                       d_w_int, count, cfg->n_bits, cfg->l_bits, d_high, d_low, vec_ok,
                       cfg->low_format == NQ_LOW_SIGNED_L1);
    return launch_status();
}

static void launch_pack_paper(int k, dim3 grid, hipStream_t s, const int8_t *v, int64_t N, int64_t K, int part, int l,
                              int up, int64_t wpr, int64_t bpr, uint64_t *out, int vec_ok)
{
    switch (k) {
#define NQ_PP_CASE(KV)                                                                                           \
    case KV:                                                                                                     \
        hipLaunchKernelGGL(k_pack_paper<KV>, grid, dim3(256), 0, s, v, N, K, part, l, up, wpr, bpr, out, vec_ok); \
        break;
        NQ_PP_CASE(1) NQ_PP_CASE(2) NQ_PP_CASE(3) NQ_PP_CASE(4) NQ_PP_CASE(5) NQ_PP_CASE(6) NQ_PP_CASE(7)
#undef NQ_PP_CASE
    default: break;
    }
}

static nq_status pack_any(int src, const int8_t *a, const int8_t *b, int64_t N, int64_t K, const nq_cfg *cfg,
                          void *ph, void *pl, void *stream)
{
    nq_status st = check_cfg(cfg);
    if (st != NQ_OK) return st;
    if ((st = check_shape(N, K)) != NQ_OK) return st;
    if ((st = check_pages(cfg, ph, pl)) != NQ_OK) return st;
    if (N * K == 0) return NQ_OK;
    const int h = cfg->n_bits - cfg->l_bits, l = cfg->l_bits;
    const int sgn = cfg->low_format == NQ_LOW_SIGNED_L1, lf = low_field_bits(cfg);
    hipStream_t s = (hipStream_t)stream;
    if (cfg->layout == NQ_LAYOUT_DENSE) {
        NQ_DISPATCH_HL(h, l, launch_pack_dense, src, sgn, a, b, N, K, ph, pl, s);
    } else {
        const int up = 8 - cfg->n_bits;
        if (N * ceil_div(ceil_div(K, 64 / (h < lf ? h : lf)), 256) > 0x7fffffffLL) return NQ_ERR_SHAPE;   // grid
        if (ph) {
            const int64_t wpr = ceil_div(K, 64 / h);
            const int64_t bpr = ceil_div(wpr, 256);
            launch_pack_paper(h, dim3((unsigned)(N * bpr)), s, a, N, K, src == 0 ? (sgn ? 3 : 0) : 2, l, up, wpr, bpr,
                              (uint64_t *)ph, (int)((K % 16 == 0) && aligned16(a)));
        }
        if (pl) {
            const int64_t wpr = ceil_div(K, 64 / lf);
            const int64_t bpr = ceil_div(wpr, 256);
            const int8_t *from = src == 0 ? a : b;
            launch_pack_paper(lf, dim3((unsigned)(N * bpr)), s, from, N, K, src == 0 ? (sgn ? 4 : 1) : 2, l, up, wpr,
                              bpr, (uint64_t *)pl, (int)((K % 16 == 0) && aligned16(from)));
        }
    }
    return launch_status();
}

extern "C" nq_status nq_pack(const int8_t *d_high, const int8_t *d_low, int64_t N, int64_t K, const nq_cfg *cfg,
                             void *d_packed_high, void *d_packed_low, void *stream)
{
    // a page is packed only when both its input and its output are given
    if ((d_high == nullptr) != (d_packed_high == nullptr)) return NQ_ERR_INVALID_ARG;
    if ((d_low == nullptr) != (d_packed_low == nullptr)) return NQ_ERR_INVALID_ARG;
    if (!d_high && !d_low) return NQ_ERR_INVALID_ARG;
    return pack_any(1, d_high, d_low, N, K, cfg, d_packed_high, d_packed_low, stream);
}

extern "C" nq_status nq_decompose_pack(const int8_t *d_w_int, int64_t N, int64_t K, const nq_cfg *cfg,
                                       void *d_packed_high, void *d_packed_low, void *stream)
{
    if (!d_w_int && N * K != 0) return NQ_ERR_INVALID_ARG;
    if (!d_packed_high && !d_packed_low) return NQ_ERR_INVALID_ARG;
    return pack_any(0, d_w_int, nullptr, N, K, cfg, d_packed_high, d_packed_low, stream);
}

template <int H, int L>
static void launch_pack_dense_batch(const PackBatch &jobs, int sgn, hipStream_t st)
{
    const int64_t tiles = jobs.first_tile[jobs.count];
    hipLaunchKernelGGL((k_pack_dense_batch<H, L>), dim3((unsigned)ceil_div(tiles, 4)), dim3(256), 0, st, jobs, sgn);
}

extern "C" nq_status nq_decompose_pack_batch(const nq_pack_job *jobs, int64_t count, const nq_cfg *cfg, void *stream)
{
    nq_status st = check_cfg(cfg);
    if (st != NQ_OK) return st;
    if (cfg->layout != NQ_LAYOUT_DENSE) return NQ_ERR_UNSUPPORTED;
    if (count < 0 || (count > 0 && !jobs)) return NQ_ERR_INVALID_ARG;
    for (int64_t i = 0; i < count; ++i) {
        if ((st = check_shape(jobs[i].N, jobs[i].K)) != NQ_OK) return st;
        if (jobs[i].N > 0x7fffffff) return NQ_ERR_SHAPE;
        if (jobs[i].N * jobs[i].K != 0 && (!jobs[i].d_w_int || !jobs[i].d_packed_high || !jobs[i].d_packed_low))
            return NQ_ERR_INVALID_ARG;
        if ((st = check_pages(cfg, jobs[i].d_packed_high, jobs[i].d_packed_low)) != NQ_OK) return st;
    }
    const int h = cfg->n_bits - cfg->l_bits, l = cfg->l_bits;
    const int sgn = cfg->low_format == NQ_LOW_SIGNED_L1;
    bool launched = false;
    for (int64_t i0 = 0; i0 < count; i0 += PACK_BATCH) {
        PackBatch b;
        b.count = 0;
        b.first_tile[0] = 0;
        for (int64_t i = i0; i < count && i < i0 + PACK_BATCH; ++i) {
            const int64_t tiles = ceil_div(jobs[i].N, 32) * ceil_div(jobs[i].K, 64);
            if (tiles == 0) continue;
            const int j = b.count++;
            b.w[j] = jobs[i].d_w_int;
            b.ph[j] = (uint32_t *)jobs[i].d_packed_high;
            b.pl[j] = (uint32_t *)jobs[i].d_packed_low;
            b.N[j] = (int)jobs[i].N;
            b.K[j] = (int)jobs[i].K;
            b.first_tile[j + 1] = b.first_tile[j] + tiles;
        }
        if (b.count == 0) continue;
        if (ceil_div(b.first_tile[b.count], 4) > 0x7fffffffLL) return NQ_ERR_SHAPE;
        for (int j = b.count + 1; j <= PACK_BATCH; ++j) b.first_tile[j] = b.first_tile[b.count];
        NQ_DISPATCH_HL(h, l, launch_pack_dense_batch, b, sgn, (hipStream_t)stream);
        launched = true;
    }
    return launched ? launch_status() : NQ_OK;          // nothing to do: no HIP call at all
}

extern "C" nq_status nq_unpack(const void *d_packed_high, const void *d_packed_low, int64_t N, int64_t K,
                               const nq_cfg *cfg, int8_t *d_high, int8_t *d_low, void *stream)
{
    nq_status st = check_cfg(cfg);
    if (st != NQ_OK) return st;
    if ((st = check_shape(N, K)) != NQ_OK) return st;
    if ((d_high == nullptr) != (d_packed_high == nullptr)) return NQ_ERR_INVALID_ARG;
    if ((d_low == nullptr) != (d_packed_low == nullptr)) return NQ_ERR_INVALID_ARG;
    if (!d_high && !d_low) return NQ_ERR_INVALID_ARG;
    if ((st = check_pages(cfg, d_packed_high, d_packed_low)) != NQ_OK) return st;
    if (N * K == 0) return NQ_OK;
    const int h = cfg->n_bits - cfg->l_bits, l = cfg->l_bits;
    const int sgn = cfg->low_format == NQ_LOW_SIGNED_L1, lf = low_field_bits(cfg);
    hipStream_t s = (hipStream_t)stream;
    if (cfg->layout == NQ_LAYOUT_DENSE) {
        NQ_DISPATCH_HL(h, l, launch_unpack_dense, sgn, d_packed_high, d_packed_low, N, K, d_high, d_low, s);
    } else {
        const int64_t cpr = ceil_div(K, 16);                      // 16-element pieces of a row, one thread each
        const dim3 grid((unsigned)ceil_div(N * cpr, 256)), block(256);
        if (d_high)
            hipLaunchKernelGGL(k_unpack_paper, grid, block, 0, s, (const uint64_t *)d_packed_high, N, K, h, 1,
                               ceil_div(K, 64 / h), cpr, d_high, (int)((K % 16 == 0) && aligned16(d_high)));
        if (d_low)
            hipLaunchKernelGGL(k_unpack_paper, grid, block, 0, s, (const uint64_t *)d_packed_low, N, K, lf, sgn,
                               ceil_div(K, 64 / lf), cpr, d_low, (int)((K % 16 == 0) && aligned16(d_low)));
    }
    return launch_status();
}
