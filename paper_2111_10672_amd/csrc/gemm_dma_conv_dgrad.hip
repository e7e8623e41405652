// One operand-layout combination of the direct-to-LDS bfloat16 product (see gemm_dma_impl.h), in a file of
// its own so that the combinations compile side by side.
#include "gemm_dma_impl.h"

namespace spb {
hipError_t launch_gemm_dma_conv_dgrad(const GemmProblem& p, hipStream_t stream) {
  return gemm_dma_detail::launch_layouts<Layout::RowK, Layout::KRow, Gather::ConvRows, Gather::ConvWeightT>(p, stream);
}
}  // namespace spb
