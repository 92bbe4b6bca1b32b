// One (dtype, layout) family of GEMM kernels per object file, so the families compile in parallel.
// Built several times with -DCHN_GEMM_T=<float|bf16_raw> -DCHN_GEMM_AKC=<0|1> -DCHN_GEMM_BKC=<0|1>
// -DCHN_GEMM_NAME=<symbol>.
#include "gemm_kernel.h"

namespace chn {
namespace gemm {

chn_status CHN_GEMM_NAME(GemmArgs &g, hipStream_t st) {
  return launch_layout<CHN_GEMM_T, CHN_GEMM_AKC != 0, CHN_GEMM_BKC != 0>(g, st);
}

}  // namespace gemm
}  // namespace chn
