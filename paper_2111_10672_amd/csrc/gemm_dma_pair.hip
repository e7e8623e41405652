// The input-gradient and the weight-gradient product of one dense layer in a single launch of the
// small-product kernel (see gemm_dma_impl.h): both read the same output gradient and neither reads the
// other's result, so on small layers, where a launch costs as much as the product, they share one.
#include "gemm_dma_impl.h"

namespace spb {
namespace gemm_dma_detail {
namespace {

template <int BM1, int BN1, int BM2, int BN2>
hipError_t launch_pair_tiles(const GemmProblem& d, const GemmProblem& w, hipStream_t stream) {
  const GemmParams p1 = make_params(d, BM1, BN1), p2 = make_params(w, BM2, BN2);
  auto kernel = gemm_bf16_small_pair_kernel<BM1, BN1, Layout::RowK, Layout::KRow, BM2, BN2, Layout::KRow, Layout::KRow>;
  constexpr size_t lds_bytes = small_pair_lds<BM1, BN1, BM2, BN2>();  // at most half a CU's LDS
  static_assert(lds_bytes <= 80 * 1024, "two workgroups per CU");
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kernel), (size_t)lds_bytes); e != hipSuccess) return e;
  const int blocks = p1.tiles_m * p1.tiles_n + p2.tiles_m * p2.tiles_n;
  hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), lds_bytes, stream, p1, p2);
  return hipGetLastError();
}

}  // namespace
}  // namespace gemm_dma_detail

bool gemm_dma_pair_accepts(const GemmProblem& d, const GemmProblem& w) {
  using namespace gemm_dma_detail;
  auto plain = [](const GemmProblem& q) { return q.batch == 1 && q.k_splits == 1 && small_product_fits(q); };
  return d.a_layout == Layout::RowK && d.b_layout == Layout::KRow && w.a_layout == Layout::KRow && w.b_layout == Layout::KRow &&
         plain(d) && plain(w);
}

hipError_t launch_gemm_dma_pair(const GemmProblem& d, const GemmProblem& w, hipStream_t stream) {
  using namespace gemm_dma_detail;
  if (!gemm_dma_pair_accepts(d, w)) return hipErrorInvalidValue;
  const bool d64 = small_product_tile64(d), w64 = small_product_tile64(w);
  if (d64 && w64) return launch_pair_tiles<64, 64, 64, 64>(d, w, stream);
  if (d64) return launch_pair_tiles<64, 64, 32, 32>(d, w, stream);
  if (w64) return launch_pair_tiles<32, 32, 64, 64>(d, w, stream);
  return launch_pair_tiles<32, 32, 32, 32>(d, w, stream);
}

}  // namespace spb
