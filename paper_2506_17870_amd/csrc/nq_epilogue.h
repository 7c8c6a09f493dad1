// Fused dequantisation epilogue of the nested GEMM / convolution kernels (paper Eq. 2:
// w_hat = s * w_int; Eq. 8: s_high = s * 2^l), applied to one 32x32 accumulator tile of
// v_mfma_i32_32x32x32_i8.  fp32, fixed operation order, one rounding per step:
//   y = (float)acc * c;  y = y + bias;  y = y + s_r * (float)r;  y = max(y, lo);  store or
//   q = clamp(rint(y * inv_s_out)).
// Lane (col = lane & 31, rg = lane >> 5) holds in register r the tile row
// 8*(r >> 2) + 4*rg + (r & 3) of column col.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nq_gemm_params.h"

namespace nq {

typedef int e_v16i __attribute__((ext_vector_type(16)));

// Per-column constants of the epilogue.  Adding a zero bias and clamping at -inf leave y
// unchanged, so the optional steps need no branch per element.
struct EpiColumn {
    float c;     // act_scale * scale[n] (* 2^l in part-bit mode)
    float bias;  // bias[n] or 0
};

__device__ __forceinline__ EpiColumn epi_column(const GemmParams &p, int n, bool full)
{
    EpiColumn e;
    const bool ok = n < p.N;
    e.c = p.act_scale * (ok ? p.scale[n] : 0.0f);
    if (!full) e.c = e.c * p.part_mul;
    e.bias = (ok && p.bias) ? p.bias[n] : 0.0f;
    return e;
}

// o_tile: element index (row * N + n) of tile row 0, column 0 -- the same for the whole wave, so
// the address is a scalar base plus a 32-bit lane offset; o_lane = 4*rg*N + column; rows_left:
// how many tile rows, counted from tile row 0, are real outputs.
template <bool OUT8, bool RESID, bool DUMP, bool WHOLE>
__device__ __forceinline__ void epi_tile_rows(const GemmParams &p, const e_v16i acc, int shift, const EpiColumn &e,
                                              int64_t o_tile, unsigned o_lane, int rg, int rows_left,
                                              const int (&res)[16])
{
    // Opaque to the optimiser: otherwise the sixteen row offsets of every specialisation are
    // hoisted out of the caller's loops and held in registers for the whole kernel.
    asm volatile("" : "+v"(o_lane));
    const float lo = p.relu ? 0.0f : -__builtin_inff();
    float *yf = reinterpret_cast<float *>(p.y) + o_tile;
    int8_t *yq = reinterpret_cast<int8_t *>(p.y) + o_tile;
    int32_t *dq = p.acc_dump + o_tile;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + (r & 3);          // relative to tile row 4*rg
        if (WHOLE || row + 4 * rg < rows_left) {
            const unsigned off = o_lane + (unsigned)(row * p.N);
            const int a = acc[r] >> shift;
            if (DUMP) dq[off] = a;
            float y = (float)a * e.c;
            y = y + e.bias;
            if (RESID) {
                const float rv = p.resid_scale * (float)res[r];
                y = y + rv;
            }
            y = fmaxf(y, lo);
            if (OUT8) {
                float q = rintf(y * p.inv_out_scale);
                q = fminf(fmaxf(q, -128.0f), 127.0f);
                yq[off] = (int8_t)(int)q;
            } else {
                yf[off] = y;
            }
        }
    }
}

// A tile whose 32 rows are all real outputs (the usual case) carries no per-element test.  The
// general kernels use the tested form only: with both forms of all their bodies the unrolled
// epilogue of a block would exceed what the compiler is willing to unroll, and accumulators
// indexed by a loop variable would fall out of the registers.
template <bool OUT8, bool RESID, bool DUMP, bool BOTH_FORMS>
__device__ __forceinline__ void epi_tile_impl(const GemmParams &p, const e_v16i acc, int shift, const EpiColumn &e,
                                              int64_t o_tile, unsigned o_lane, int rg, int rows_left,
                                              const int (&res)[16])
{
    if (BOTH_FORMS && rows_left >= 32)
        epi_tile_rows<OUT8, RESID, DUMP, true>(p, acc, shift, e, o_tile, o_lane, rg, rows_left, res);
    else if (rows_left > 0)
        epi_tile_rows<OUT8, RESID, DUMP, false>(p, acc, shift, e, o_tile, o_lane, rg, rows_left, res);
}

// Requests the residual codes of one tile (general kernels only).  Kernels call this for all
// their tiles before the first epi_tile, so that the loads of every tile are in flight together
// instead of one memory latency being paid per tile.
template <bool GENERAL>
__device__ __forceinline__ void epi_resid_load(const GemmParams &p, int64_t o_tile, unsigned o_lane, int rg,
                                               int rows_left, int (&res)[16])
{
    if constexpr (GENERAL) {
        if (p.resid) {
            const int8_t *rq = p.resid + o_tile;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + (r & 3);
                res[r] = 0;
                if (row + 4 * rg < rows_left) res[r] = rq[o_lane + (unsigned)(row * p.N)];
            }
        }
    }
}

// Test aid: the raw int32 accumulators of a tile (after the exact shift), predicated per row.
__device__ __forceinline__ void epi_dump(const GemmParams &p, const e_v16i acc, int shift, int64_t o_tile,
                                         unsigned o_lane, int rg, int rows_left)
{
    int32_t *dq = p.acc_dump + o_tile;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + (r & 3);
        if (row + 4 * rg < rows_left) dq[o_lane + (unsigned)(row * p.N)] = acc[r] >> shift;
    }
}

// Chooses the specialisation once per tile (uniform branches), not once per element.
// GENERAL = false: the kernel was launched for a plain epilogue (fp32 or int8 output, no
// residual, no accumulator dump) and carries only those two bodies, which keeps the hot kernels
// short of register pressure; GENERAL = true kernels add the residual bodies and the dump pass.
template <bool GENERAL>
__device__ __forceinline__ void epi_tile(const GemmParams &p, const e_v16i acc, int shift, const EpiColumn &e,
                                         int64_t o_tile, unsigned o_lane, int rg, int rows_left,
                                         const int (&res)[16])
{
    if constexpr (GENERAL) {
        if (p.acc_dump) epi_dump(p, acc, shift, o_tile, o_lane, rg, rows_left);
        if (p.resid) {
            if (p.out_int8) epi_tile_impl<true, true, false, false>(p, acc, shift, e, o_tile, o_lane, rg, rows_left, res);
            else epi_tile_impl<false, true, false, false>(p, acc, shift, e, o_tile, o_lane, rg, rows_left, res);
            return;
        }
    }
    if (p.out_int8) epi_tile_impl<true, false, false, !GENERAL>(p, acc, shift, e, o_tile, o_lane, rg, rows_left, res);
    else epi_tile_impl<false, false, false, !GENERAL>(p, acc, shift, e, o_tile, o_lane, rg, rows_left, res);
}

}  // namespace nq
