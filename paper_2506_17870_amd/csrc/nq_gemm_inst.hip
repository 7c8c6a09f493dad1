// Four translation units per nesting, compiled with -DNQ_INST_H=<h> -DNQ_INST_L=<l> and
// -DNQ_INST_PART=0 (generic, windowed, register-stationary and few-channel kernels), 1 (large-GEMM kernels),
// 2 (depthwise / grouped convolution) or 3 (stationary-weights GEMM), so that the units build in parallel.
#if NQ_INST_PART == 0
#include "nq_conv_rowstream.h"
#include "nq_conv_smallcin.h"
#include "nq_conv_window.h"
#include "nq_gemm_kernel.h"
#include "nq_gemm_skinny.h"

namespace nq {
template void launch_nested_gemm_skinny<NQ_INST_H, NQ_INST_L>(bool, const GemmParams &, hipStream_t, void *, void *);
template void launch_nested_gemm_skinny_batch<NQ_INST_H, NQ_INST_L>(int, int, bool, bool, const GemmParams *, const int *,
                                                                    int, int, hipStream_t, void *, void *);
template void launch_nested_gemm<NQ_INST_H, NQ_INST_L>(bool, int, const GemmParams &, hipStream_t, void *, void *);
template void launch_nested_conv_window<NQ_INST_H, NQ_INST_L>(bool, int, const GemmParams &, const WindowGeom &,
                                                              size_t, hipStream_t, void *, void *);
template void launch_nested_conv_rowstream<NQ_INST_H, NQ_INST_L>(bool, const GemmParams &, const StreamGeom &, int,
                                                                 hipStream_t, void *, void *);
template void launch_nested_conv_smallcin<NQ_INST_H, NQ_INST_L>(bool, const GemmParams &, const SmallCinGeom &,
                                                                hipStream_t, void *, void *);
}
#elif NQ_INST_PART == 2
#include "nq_conv_grouped.h"
#include "nq_conv_grouped_any.h"

namespace nq {
template void launch_nested_conv_grouped<NQ_INST_H, NQ_INST_L>(bool, const GemmParams &, const GroupGeom &,
                                                               hipStream_t, void *, void *);
template void launch_nested_conv_grouped_any<NQ_INST_H, NQ_INST_L>(bool, const GemmParams &, int, int, int, hipStream_t,
                                                                   void *, void *);
}
#elif NQ_INST_PART == 3
#include "nq_gemm_stat.h"

namespace nq {
template void launch_nested_gemm_stat<NQ_INST_H, NQ_INST_L>(bool, const GemmParams &, const StatGeom &, hipStream_t,
                                                            void *, void *);
}
#else
#include "nq_gemm_big.h"

namespace nq {
template void launch_nested_gemm_big<NQ_INST_H, NQ_INST_L>(bool, const GemmParams &, int, int *, hipStream_t, void *,
                                                           void *);
}
#endif
