// One translation unit per nesting: compiled with -DNQ_INST_H=<h> -DNQ_INST_L=<l>.
#include "nq_gemm_kernel.h"

namespace nq {
template void launch_nested_gemm<NQ_INST_H, NQ_INST_L>(bool, int, const GemmParams &, hipStream_t);
}
