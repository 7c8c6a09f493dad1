// Host-side helpers shared by the translation units of libnq: argument checks, the
// (h, l) dispatch and HIP error handling.  Internal; the public interface is include/nq.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/nq.h"

namespace nq {

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// n in {8,6}, 1 <= l <= n-2 (Sec. 3.3.1 considers INT(8|h), h in 3..7 and INT(6|h), h in 3..5).
inline nq_status check_cfg(const nq_cfg *cfg)
{
    if (!cfg) return NQ_ERR_INVALID_ARG;
    if (cfg->n_bits != 8 && cfg->n_bits != 6) return NQ_ERR_UNSUPPORTED;
    if (cfg->l_bits < 1 || cfg->l_bits > cfg->n_bits - 2) return NQ_ERR_UNSUPPORTED;
    if (cfg->layout != NQ_LAYOUT_DENSE && cfg->layout != NQ_LAYOUT_PAPER_U64) return NQ_ERR_INVALID_ARG;
    if (cfg->low_format != NQ_LOW_UNSIGNED_L && cfg->low_format != NQ_LOW_SIGNED_L1) return NQ_ERR_INVALID_ARG;
    return NQ_OK;
}

// Field width of the lower-bit page: l, or l + 1 for the compensated signed part (Sec. 3.3.3).
inline int low_field_bits(const nq_cfg *cfg) { return cfg->l_bits + (cfg->low_format == NQ_LOW_SIGNED_L1 ? 1 : 0); }

inline nq_status check_shape(int64_t N, int64_t K)
{
    if (N < 0 || K < 0) return NQ_ERR_INVALID_ARG;
    if (K > NQ_MAX_K || N > (int64_t(1) << 31)) return NQ_ERR_SHAPE;
    return NQ_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Turns the status of the last launch into an nq_status and clears HIP's sticky flag.
inline nq_status launch_status()
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? NQ_OK : NQ_ERR_HIP;
}

}  // namespace nq

// Calls F<H, L>(args...) for the supported (h, l) pairs; h + l is 8 or 6.
#define NQ_DISPATCH_HL(h, l, F, ...)                       \
    switch ((h) * 8 + (l)) {                               \
    case 7 * 8 + 1: F<7, 1>(__VA_ARGS__); break;           \
    case 6 * 8 + 2: F<6, 2>(__VA_ARGS__); break;           \
    case 5 * 8 + 3: F<5, 3>(__VA_ARGS__); break;           \
    case 4 * 8 + 4: F<4, 4>(__VA_ARGS__); break;           \
    case 3 * 8 + 5: F<3, 5>(__VA_ARGS__); break;           \
    case 2 * 8 + 6: F<2, 6>(__VA_ARGS__); break;           \
    case 5 * 8 + 1: F<5, 1>(__VA_ARGS__); break;           \
    case 4 * 8 + 2: F<4, 2>(__VA_ARGS__); break;           \
    case 3 * 8 + 3: F<3, 3>(__VA_ARGS__); break;           \
    case 2 * 8 + 4: F<2, 4>(__VA_ARGS__); break;           \
    default: break;                                        \
    }
