// Bit-field codec of the dense-tile page layout, on dwords (four byte lanes at once).
//
// A "unit" is the 32 weights one slot of a tile holds: eight dwords X[0..7], byte b of
// X[j] being the weight at column 4*j + b of the slot.  The codec works on the operand
// form of a weight byte: the INT-n value shifted to the top of the byte, w * 2^(8-n), so
// that bits [7..S] (S = 8-H) are the higher-bit field and bits [S-1..S-L] the lower-bit
// field.  With the lower-bit field cleared the byte is w_high * 2^S, which is what the
// part-bit kernels feed to the matrix cores (Eq. 8 of the paper: the factor 2^l moves
// into the scale); with both fields it is w_int * 2^(8-n) (Eq. 4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nq {

__host__ __device__ constexpr uint32_t rep4(uint32_t byte) { return (byte & 0xFFu) * 0x01010101u; }
__host__ __device__ constexpr int cmin(int a, int b) { return a < b ? a : b; }

template <int H>
struct HighCodec {
    static constexpr int S = 8 - H;
    static constexpr uint32_t HM = rep4(0xFFu << S);

    // P[0..H-1] -> D[0..7] with the lower S bits of every byte zero.
    __device__ __forceinline__ static void decode(const uint32_t (&P)[H], uint32_t (&D)[8])
    {
#pragma unroll
        for (int i = 0; i < H; ++i) D[i] = P[i] & HM;
#pragma unroll
        for (int j = H; j < 8; ++j) {
            uint32_t d = 0;
#pragma unroll
            for (int t = 0; t < H; ++t) {
                const int pos = (j - H) * H + t;   // place in the string of spare bits
                const int byte = pos / S, bit = pos % S;
                if (t == 0 || bit == 0) {          // a run of field bits inside one byte
                    const int len = cmin(S - bit, H - t);
                    const uint32_t mask = rep4(((1u << len) - 1u) << (S + t));
                    d |= (P[byte] << (S + t - bit)) & mask;
                }
            }
            D[j] = d;
        }
    }

    // X[0..7] (higher-bit fields in bits [7..S]) -> P[0..H-1].
    __device__ __forceinline__ static void encode(const uint32_t (&X)[8], uint32_t (&P)[H])
    {
#pragma unroll
        for (int i = 0; i < H; ++i) P[i] = X[i] & HM;
#pragma unroll
        for (int j = H; j < 8; ++j) {
#pragma unroll
            for (int t = 0; t < H; ++t) {
                const int pos = (j - H) * H + t;
                const int byte = pos / S, bit = pos % S;
                if (t == 0 || bit == 0) {
                    const int len = cmin(S - bit, H - t);
                    const uint32_t mask = rep4(((1u << len) - 1u) << bit);
                    P[byte] |= (X[j] >> (S + t - bit)) & mask;
                }
            }
        }
    }
};

// The lower-bit field of L bits sits at bits [S-1..S-L] of the operand byte.
template <int L, int S>
struct LowCodec {
    static constexpr int P0 = S - L;
    static constexpr uint32_t LM = rep4(((1u << L) - 1u) << P0);

    // ORs the lower-bit fields of Q[0..L-1] into D[0..7].
    __device__ __forceinline__ static void decode_or(const uint32_t (&Q)[L], uint32_t (&D)[8])
    {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
#pragma unroll
            for (int t = 0; t < L; ++t) {
                const int pos = j * L + t;
                const int byte = pos / 8, bit = pos % 8;
                if (t == 0 || bit == 0) {
                    const int len = cmin(8 - bit, L - t);
                    const int target = P0 + t;
                    const uint32_t mask = rep4(((1u << len) - 1u) << target);
                    const uint32_t q = Q[byte];
                    const uint32_t moved = (target >= bit) ? (q << (target >= bit ? target - bit : 0))
                                                           : (q >> (bit > target ? bit - target : 0));
                    D[j] |= moved & mask;
                }
            }
        }
    }

    __device__ __forceinline__ static void encode(const uint32_t (&X)[8], uint32_t (&Q)[L])
    {
#pragma unroll
        for (int i = 0; i < L; ++i) Q[i] = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
#pragma unroll
            for (int t = 0; t < L; ++t) {
                const int pos = j * L + t;
                const int byte = pos / 8, bit = pos % 8;
                if (t == 0 || bit == 0) {
                    const int len = cmin(8 - bit, L - t);
                    const int source = P0 + t;
                    const uint32_t mask = rep4(((1u << len) - 1u) << bit);
                    const uint32_t x = X[j];
                    const uint32_t moved = (source >= bit) ? (x >> (source >= bit ? source - bit : 0))
                                                           : (x << (bit > source ? bit - source : 0));
                    Q[byte] |= moved & mask;
                }
            }
        }
    }
};

// The compensated lower-bit part of the paper (Sec. 3.3.3: one extra bit, signed): fields of L + 1
// bits in two's complement, stored as the same kind of bit string as the unsigned part.  Full-bit
// recomposition is shift-ADD, w = w_high * 2^l + w_low (Eq. 4), no longer a concatenation.  Per byte
// lane: the top bit s of the field says w_low < 0, and then w = (w_high - 1) * 2^l + (w_low mod 2^l),
// so the operand byte is the higher-bit byte minus s at bit S (a subtraction that must not borrow
// from the neighbouring lane) with the low l bits of the field ORed in below.
template <int L, int S>
struct SignedLowCodec {
    using Raw = LowCodec<L + 1, S + 1>;                       // field at bits [S-L, S]
    static constexpr uint32_t TOP = rep4(1u << S);             // its sign bit
    static constexpr uint32_t LOW = rep4(((1u << L) - 1u) << (S - L));

    // D[0..7]: higher-bit bytes (lower S bits zero) -> full-bit operand bytes.
    __device__ __forceinline__ static void decode_add(const uint32_t (&Q)[L + 1], uint32_t (&D)[8])
    {
        uint32_t T[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) T[j] = 0;
        Raw::decode_or(Q, T);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // byte-wise a - b for b < 128: force the top bit of a so that no lane borrows, then put
            // the top bit right (it flips exactly where a's was clear)
            const uint32_t a = D[j], b = T[j] & TOP;
            const uint32_t r = ((a | 0x80808080u) - b) ^ (~a & 0x80808080u);
            D[j] = r | (T[j] & LOW);
        }
    }
};

// The lower-bit page as the GEMM / convolution kernels see it.  MODE 0: not read (part-bit model);
// 1: unsigned l-bit part, concatenated below the higher-bit field; 2: compensated signed (l+1)-bit
// part, added.  DW = packed dwords per slot of a tile.
template <int L, int S, int MODE>
struct LowPage {
    static constexpr int DW = MODE == 2 ? L + 1 : (MODE == 1 ? L : 0);
    static constexpr int ARR = DW ? DW : 1;                   // array extent (never zero)
    __device__ __forceinline__ static void apply(const uint32_t (&Q)[ARR], uint32_t (&D)[8])
    {
        if constexpr (MODE == 1) LowCodec<L, S>::decode_or(Q, D);
        if constexpr (MODE == 2) SignedLowCodec<L, S>::decode_add(Q, D);
    }
};

}  // namespace nq
