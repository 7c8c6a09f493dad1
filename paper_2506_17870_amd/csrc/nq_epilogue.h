// Fused dequantisation epilogue of the nested GEMM / convolution kernels (paper Eq. 2:
// w_hat = s * w_int; Eq. 8: s_high = s * 2^l), applied to one 32x32 accumulator tile of
// v_mfma_i32_32x32x32_i8.  fp32, fixed operation order, one rounding per step:
//   y = (float)acc * c;  y = y + bias;  y = y + s_r * (float)r;  y = max(y, lo);  store or
//   q = clamp(rint(y * inv_s_out)).
//
// Two register layouts, chosen per kernel instantiation so that the stores of a wave are as
// contiguous as the output type allows:
//
//  EPI_F32 (fp32 output, no residual): activations are the matrix core's row operand, weights its
//    column operand.  Lane (col = lane & 31, rg = lane >> 5) holds channel col of the tile rows
//    8*(r >> 2) + 4*rg + (r & 3); a store instruction writes two runs of 128 contiguous bytes.
//
//  EPI_I8 / EPI_ANY (int8 output, residual, everything else): the operands are swapped, so a lane
//    holds one pixel (lane & 31) and sixteen channels.  Which channels is the kernel's choice:
//    the lane that feeds operand row a fetches the weights of channel epi_weight_slot() of the
//    tile, and with that permutation register r of half-wave rg is channel 16*rg + r.  A lane
//    then owns 16 consecutive channels of one pixel: 16 contiguous bytes of an int8 output or of
//    the residual, moved with single 16-byte accesses instead of sixteen byte accesses.
//    EPI_I8 needs N to be a multiple of 16 and 16-byte aligned pointers (checked by the host);
//    EPI_ANY works element by element for any N, any alignment, either output type, and writes
//    the accumulator dump.
//
// A tile is named by (m0, rows, nt0): the global output row of tile row 0, how many of the 32
// tile rows are real outputs, and the first channel of the tile.  The per-lane bodies of the swapped
// layouts (epi_cols16, epi_row16: sixteen consecutive channels of one output row) are also what the
// depthwise / grouped kernel calls, whose 16 x 16 accumulator tiles map lanes to pixels differently.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_gemm_params.h"

namespace nq {

typedef int e_v16i __attribute__((ext_vector_type(16)));
typedef int e_v4i __attribute__((ext_vector_type(4)));
typedef float e_v4f __attribute__((ext_vector_type(4)));

constexpr int EPI_F32 = 0, EPI_I8 = 1, EPI_ANY = 2;

// Slot of a dense weight tile (32*g + row) that lane `lane` fetches.  In the swapped layouts the
// matrix core puts operand row 8*j + 4*rg + i (j < 4, i < 4) into register 4*j + i of half-wave
// rg; fetching channel 16*rg + 4*j + i for that row makes the registers of a lane consecutive
// channels.
template <int EPI>
__device__ __forceinline__ int epi_weight_slot(int lane)
{
    if constexpr (EPI == EPI_F32) return lane;
    const int a = lane & 31;
    return (lane & 32) | (((a >> 2) & 1) << 4) | ((a >> 3) << 2) | (a & 3);
}

// One matrix-core step with the operand order of the layout.
template <int EPI>
__device__ __forceinline__ e_v16i epi_mfma(const e_v4i wfrag, const e_v4i xfrag, const e_v16i acc)
{
    if constexpr (EPI == EPI_F32) return __builtin_amdgcn_mfma_i32_32x32x32_i8(xfrag, wfrag, acc, 0, 0, 0);
    else return __builtin_amdgcn_mfma_i32_32x32x32_i8(wfrag, xfrag, acc, 0, 0, 0);
}

// Per-channel constants of the lane's channels (one in EPI_F32, sixteen otherwise).  Adding a
// zero bias and clamping at -inf leave y unchanged, so the optional steps need no branch per
// element.
template <int EPI>
struct EpiCols {
    static constexpr int NC = EPI == EPI_F32 ? 1 : 16;
    float c[NC];     // act_scale * scale[n] (* 2^l in part-bit mode)
    float bias[NC];  // bias[n] or 0
};

// EPI_I8: the scale and bias of the sixteen channels nl0 .. nl0 + 15 as they come from memory, so that a kernel can
// request them long before it needs the constants made from them (epi_cols16_finish).
struct EpiRaw16 {
    e_v4f s[4], b[4];
};
__device__ __forceinline__ void epi_cols16_fetch(const GemmParams &p, int nl0, EpiRaw16 &raw)
{
    const int n = nl0 < p.N ? nl0 : 0;
    const e_v4f *s4 = reinterpret_cast<const e_v4f *>(p.scale + n);
    const e_v4f *b4 = reinterpret_cast<const e_v4f *>(p.bias + n);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        raw.s[j] = s4[j];
        raw.b[j] = e_v4f{0.0f, 0.0f, 0.0f, 0.0f};
        if (p.bias) raw.b[j] = b4[j];
    }
}
__device__ __forceinline__ void epi_cols16_finish(const GemmParams &p, bool full, const EpiRaw16 &raw, EpiCols<EPI_I8> &e)
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float c = p.act_scale * raw.s[j][i];
            if (!full) c = c * p.part_mul;
            e.c[4 * j + i] = c;
            e.bias[4 * j + i] = raw.b[j][i];
        }
}

// Constants of the sixteen channels nl0 .. nl0 + 15 (swapped layouts).
template <int EPI>
__device__ __forceinline__ void epi_cols16(const GemmParams &p, int nl0, bool full, EpiCols<EPI> &e)
{
    static_assert(EPI != EPI_F32, "sixteen channels per lane: swapped layouts only");
    if constexpr (EPI == EPI_I8) {
        EpiRaw16 raw;
        epi_cols16_fetch(p, nl0, raw);
        epi_cols16_finish(p, full, raw, e);
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = nl0 + r < p.N;
            float c = p.act_scale * (ok ? p.scale[nl0 + r] : 0.0f);
            if (!full) c = c * p.part_mul;
            e.c[r] = c;
            e.bias[r] = (ok && p.bias) ? p.bias[nl0 + r] : 0.0f;
        }
    }
}

template <int EPI>
__device__ __forceinline__ void epi_cols(const GemmParams &p, int nt0, int lane, bool full, EpiCols<EPI> &e)
{
    if constexpr (EPI == EPI_F32) {
        const int n = nt0 + (lane & 31);
        const bool ok = n < p.N;
        float c = p.act_scale * (ok ? p.scale[n] : 0.0f);
        if (!full) c = c * p.part_mul;
        e.c[0] = c;
        e.bias[0] = (ok && p.bias) ? p.bias[n] : 0.0f;
    } else {
        epi_cols16<EPI>(p, nt0 + 16 * (lane >> 5), full, e);
    }
}

// Requests the residual codes of the lane's sixteen channels (EPI_I8; EPI_ANY reads them element
// by element inside epi_tile, EPI_F32 has none).  Kernels call this for all their tiles before the
// first epi_tile, so that the loads of every tile are in flight together.
template <int EPI>
__device__ __forceinline__ void epi_resid_load(const GemmParams &p, int64_t m0, int rows, int nt0, int lane, e_v4i &res)
{
    res = e_v4i{0, 0, 0, 0};
    if constexpr (EPI == EPI_I8) {
        const int nl0 = nt0 + 16 * (lane >> 5);
        if (p.resid && (lane & 31) < rows && nl0 < p.N)
            res = *reinterpret_cast<const e_v4i *>(p.resid + (m0 + (lane & 31)) * p.N + nl0);
    }
}

// Waits until every outstanding load has landed, and tells the compiler so.  Kernels call it once between the
// last load of their epilogue and its first store: after it no register is the target of a load in flight, so
// the compiler has no reason to wait on the memory counter again, which, once stores are in flight, would be
// a wait for their acknowledgements (loads and stores share the counter and are counted in order).
__device__ __forceinline__ void epi_join()
{
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0f70);                   // vmcnt(0); the other counters are left alone
    __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ float epi_quantise(float y, float inv_out_scale)
{
    const float q = rintf(y * inv_out_scale);
    return fminf(fmaxf(q, -128.0f), 127.0f);
}

// EPI_F32 body.  WHOLE: all 32 tile rows are real outputs, so no test per element.
template <bool WHOLE>
__device__ __forceinline__ void epi_tile_f32(const GemmParams &p, const e_v16i acc, int shift, const EpiCols<EPI_F32> &e,
                                             int64_t o_tile, unsigned o_lane, int rg, int rows)
{
    // Opaque to the optimiser: otherwise the sixteen row offsets of every tile are hoisted out of
    // the caller's loops and held in registers for the whole kernel.
    asm volatile("" : "+v"(o_lane));
    const float lo = p.relu ? 0.0f : -__builtin_inff();
    float *yf = reinterpret_cast<float *>(p.y) + o_tile;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + (r & 3);          // relative to tile row 4*rg
        if (WHOLE || row + 4 * rg < rows) {
            float y = (float)(acc[r] >> shift) * e.c[0];
            y = y + e.bias[0];
            yf[o_lane + (unsigned)(row * p.N)] = fmaxf(y, lo);
        }
    }
}

// EPI_I8 arithmetic of one output row's sixteen channels: the requantised codes, packed, not stored.
__device__ __forceinline__ e_v4i epi_codes16(const GemmParams &p, const e_v16i acc, int shift, const EpiCols<EPI_I8> &e,
                                             const e_v4i &res)
{
    const float lo = p.relu ? 0.0f : -__builtin_inff();
    float y[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        y[r] = (float)(acc[r] >> shift) * e.c[r];
        y[r] = y[r] + e.bias[r];
    }
    if (p.resid) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int code = (int)(int8_t)((unsigned)res[r >> 2] >> (8 * (r & 3)));
            const float rv = p.resid_scale * (float)code;
            y[r] = y[r] + rv;
        }
    }
    e_v4i q;
    if (p.relu && p.inv_out_scale > 0.0f) {
        // With a ReLU and a positive output scale, clamp(rint(max(y, 0) * inv), -128, 127) is
        // rint(med3(y * inv, 0, 127)): rounding and a positive factor keep the order and map 0 to 0, so
        // the ReLU can be taken after the scaling, where it is the lower end of one three-operand clamp,
        // and rounding commutes with a clamp to whole numbers.  The rounding itself (to nearest, ties to
        // even) is done by the float -> unsigned byte pack.
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            unsigned d = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float v = __builtin_amdgcn_fmed3f(y[4 * j + i] * p.inv_out_scale, 0.0f, 127.0f);
                d = __builtin_amdgcn_cvt_pk_u8_f32(v, i, d);
            }
            q[j] = (int)d;
        }
    } else {
        // The rounded code plus 128 goes through the saturating float -> unsigned byte pack, which
        // clamps it to [0, 255] (the clamp of the code to [-128, 127]); the offset is taken off
        // again by flipping the top bit of every byte.  The sum is exact for every code that is
        // not clamped anyway.
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            unsigned d = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float v = rintf(fmaxf(y[4 * j + i], lo) * p.inv_out_scale) + 128.0f;
                d = __builtin_amdgcn_cvt_pk_u8_f32(v, i, d);
            }
            q[j] = (int)(d ^ 0x80808080u);
        }
    }
    return q;
}

// Swapped layouts: the lane's sixteen consecutive channels nl0 .. nl0 + 15 of output row o / N; o is the
// element offset of channel nl0 in that row.  res: the residual codes from epi_resid_load (EPI_I8).
template <int EPI>
__device__ __forceinline__ void epi_row16(const GemmParams &p, const e_v16i acc, int shift, const EpiCols<EPI> &e,
                                          int64_t o, int nl0, const e_v4i &res)
{
    static_assert(EPI != EPI_F32, "sixteen channels per lane: swapped layouts only");
    const float lo = p.relu ? 0.0f : -__builtin_inff();
    if constexpr (EPI == EPI_ANY) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (nl0 + r < p.N) {
                const int a = acc[r] >> shift;
                if (p.acc_dump) p.acc_dump[o + r] = a;
                float y = (float)a * e.c[r];
                y = y + e.bias[r];
                if (p.resid) {
                    const float rv = p.resid_scale * (float)p.resid[o + r];
                    y = y + rv;
                }
                y = fmaxf(y, lo);
                if (p.out_int8)
                    reinterpret_cast<int8_t *>(p.y)[o + r] = (int8_t)(int)epi_quantise(y, p.inv_out_scale);
                else
                    reinterpret_cast<float *>(p.y)[o + r] = y;
            }
        }
    } else {
        if (nl0 >= p.N) return;
        *reinterpret_cast<e_v4i *>(reinterpret_cast<int8_t *>(p.y) + o) = epi_codes16(p, acc, shift, e, res);
    }
}

// One tile of the block's output.
template <int EPI>
__device__ __forceinline__ void epi_tile(const GemmParams &p, const e_v16i acc, int shift, const EpiCols<EPI> &e,
                                         int64_t m0, int rows, int nt0, int lane, const e_v4i &res)
{
    const int rg = lane >> 5;
    if constexpr (EPI == EPI_F32) {
        const int col = lane & 31;
        if (nt0 + col >= p.N) return;
        // the tile's address is the same for the whole wave: a scalar base plus a 32-bit lane offset
        if (rows >= 32) epi_tile_f32<true>(p, acc, shift, e, m0 * p.N + nt0, (unsigned)(4 * rg * p.N + col), rg, rows);
        else if (rows > 0) epi_tile_f32<false>(p, acc, shift, e, m0 * p.N + nt0, (unsigned)(4 * rg * p.N + col), rg, rows);
    } else {
        const int nl0 = nt0 + 16 * rg;
        if ((lane & 31) >= rows) return;
        epi_row16<EPI>(p, acc, shift, e, (m0 + (lane & 31)) * p.N + nl0, nl0, res);
    }
}

// Which layout a problem gets (host side).
inline int epi_mode(const GemmParams &p) { return p.general ? EPI_ANY : (p.out_int8 ? EPI_I8 : EPI_F32); }

}  // namespace nq
