// bfloat16 products on the gfx950 matrix cores with direct-to-LDS operand loads.
//
//   C[m, n] = sum_k A(m, k) * B(n, k),   float32 accumulation
//
// Same three products as gemm.hip (forward, input gradient, weight gradient of a dense layer), built
// around two CDNA4 facilities:
//   * global_load_lds_dwordx4: every lane fetches 16 bytes from its own global address and the wave's
//     64 chunks land in one contiguous KiB of LDS, without passing through registers.  Several tiles
//     can therefore be in flight at once (STAGES-deep ring); which chunk a lane fetches is chosen so
//     that the KiB it fills is already in the bank-friendly order the matrix-core reads want.
//   * ds_read_b64_tr_b16: a transposing LDS read.  An operand whose *row* index is contiguous in memory
//     (the layout of both weight-gradient operands and of W in the input-gradient product) is copied to
//     LDS as it lies and transposed on the way to the registers.  Within 16 lanes, lane j receives
//     element (j % 4) of the 8-byte words read by lanes j/4, j/4 + 4, j/4 + 8, j/4 + 12; pointing lane j'
//     at 4 consecutive rows starting at row 4 * (j' % 4) of k-row j'/4 gives lane j four consecutive k
//     of row j, which is the MFMA operand layout.
// Tile loop: wait for tile t (s_waitcnt vmcnt leaves the younger tiles' loads in flight), one barrier,
// issue tile t + STAGES - 1 into the buffer tile t - 1 used, multiply tile t.
#include "gemm_common.h"

namespace spb {

hipError_t launch_gemm_dma_rr(const GemmProblem& p, hipStream_t stream);
hipError_t launch_gemm_dma_rk(const GemmProblem& p, hipStream_t stream);
hipError_t launch_gemm_dma_kk(const GemmProblem& p, hipStream_t stream);
hipError_t launch_gemm_dma_conv_fwd(const GemmProblem& p, hipStream_t stream);
hipError_t launch_gemm_dma_conv_dgrad(const GemmProblem& p, hipStream_t stream);
hipError_t launch_gemm_dma_conv_wgrad(const GemmProblem& p, hipStream_t stream);

bool gemm_dma_accepts(const GemmProblem& p) {
  if (p.dtype != DType::BF16) return false;
  // A partly filled 16-byte chunk along the contiguous index is fetched whole: allowed only where the
  // owner of the buffer keeps the rest of the chunk zero.
  auto ok = [&](Layout l, int rows, bool pad_zero) { return ((l == Layout::RowK ? p.K : rows) % 8 == 0) || pad_zero; };
  if (!ok(p.a_layout, p.M, p.a_pad_zero) || !ok(p.b_layout, p.N, p.b_pad_zero)) return false;
  // The epilogue moves 16 bytes at a time along n.
  auto a16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
  const int per_out = p.epilogue == Epilogue::StoreF32 ? 4 : 8;
  if (p.ldc % per_out || !a16(p.C)) return false;
  if (p.bias && !a16(p.bias)) return false;
  const bool reads_mask = p.epilogue == Epilogue::MaskStore || p.epilogue == Epilogue::ScaleStore;
  if (reads_mask && (!p.mask || p.ldmask % 8 || !a16(p.mask))) return false;
  if (p.epilogue == Epilogue::AffineBwdStore &&
      (!p.mask || p.ldmask % 8 || !a16(p.mask) || !p.affine_y || p.ldaffine_y % 8 || !a16(p.affine_y) || !p.col_scale || !p.col_partial ||
       p.N % 8 || p.k_splits != 1 || p.batch != 1 || p.bias))
    return false;
  if (p.residual && (p.ldres % 8 || !a16(p.residual))) return false;
  if (p.aux_out && (p.ldaux % 8 || !a16(p.aux_out))) return false;
  if (p.col_scale && !a16(p.col_scale)) return false;
  if (p.k_splits < 1 || p.k_splits > 65535 || (p.k_splits > 1 && (p.epilogue != Epilogue::StoreF32 || p.batch != 1 || p.bias || p.a_row_sum))) return false;
  if (p.a_gather != Gather::None || p.b_gather != Gather::None) {
    const ConvGeom& c = p.conv;
    if (c.sc % 8 || c.r * c.s > 255 || (c.stride != 1 && c.stride != 2) || c.rh <= 0 || c.rw <= 0 || c.rh * c.rw > 65535) return false;
    if (p.b_gather == Gather::ConvWeightT && (c.w_cin % 8 || c.w_cout % 8)) return false;
  }
  if (p.batch < 1 || p.batch > 65535 || (p.batch > 1 && p.a_row_sum)) return false;
  // batch offsets must keep every operand 16-byte aligned
  for (const BatchStride* b : {&p.a_batch, &p.b_batch, &p.c_batch})
    if (b->inner_count < 1 || b->outer % 8 || b->inner % 8) return false;
  return true;
}

hipError_t launch_gemm_dma(const GemmProblem& p, hipStream_t stream) {
  if (p.a_gather == Gather::ConvRows && p.b_gather == Gather::None && p.b_layout == Layout::RowK) return launch_gemm_dma_conv_fwd(p, stream);
  if (p.a_gather == Gather::ConvRows && p.b_gather == Gather::ConvWeightT) return launch_gemm_dma_conv_dgrad(p, stream);
  if (p.a_gather == Gather::None && p.a_layout == Layout::KRow && p.b_gather == Gather::ConvPatchT) return launch_gemm_dma_conv_wgrad(p, stream);
  if (p.a_gather != Gather::None || p.b_gather != Gather::None) return hipErrorInvalidValue;
  if (p.a_layout == Layout::RowK && p.b_layout == Layout::RowK) return launch_gemm_dma_rr(p, stream);
  if (p.a_layout == Layout::RowK && p.b_layout == Layout::KRow) return launch_gemm_dma_rk(p, stream);
  if (p.a_layout == Layout::KRow && p.b_layout == Layout::KRow) return launch_gemm_dma_kk(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace spb
