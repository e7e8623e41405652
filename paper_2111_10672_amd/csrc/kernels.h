// Host-side launch interface of the HIP kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace spb {

enum class DType : int { F32 = 0, BF16 = 1 };

inline size_t dtype_size(DType t) { return t == DType::F32 ? 4 : 2; }

// How an operand of the product C[m, n] = sum_k A(m, k) * B(n, k) lies in memory.
enum class Layout : int {
  RowK = 0,  // element (row, k) at base[row * ld + k]: the reduction index is contiguous
  KRow = 1,  // element (row, k) at base[k * ld + row]: the row index is contiguous
};

enum class Epilogue : int {
  StoreF32 = 0,      // C float32 = acc (+ bias[n])
  BiasAct = 1,       // C (T) = act(acc + bias[n]); act = ReLU if relu else identity
  MaskStore = 2,     // C (T) = mask[m, n] > 0 ? acc : 0   (ReLU backward fused into the input-gradient product)
};

struct GemmProblem {
  DType dtype = DType::BF16;      // storage type of A, B, bias, mask and of C unless the epilogue stores float32
  Layout a_layout = Layout::RowK, b_layout = Layout::RowK;
  Epilogue epilogue = Epilogue::StoreF32;
  int M = 0, N = 0, K = 0;
  const void* A = nullptr; int lda = 0;
  const void* B = nullptr; int ldb = 0;
  void* C = nullptr; int ldc = 0;
  const void* bias = nullptr;     // [N], dtype
  int relu = 0;
  const void* mask = nullptr; int ldmask = 0;   // [M, N], dtype
  // The buffer's owner keeps zeros between the end of each row's data and the next multiple of 8 elements
  // along the contiguous index (lets a kernel fetch whole 16-byte chunks).
  bool a_pad_zero = false, b_pad_zero = false;
  float* a_row_sum = nullptr;     // optional [M]: sum_k A(m, k), written once by the tiles of column block 0
  const char* name = "gemm";
};

// Checks shapes and alignment on the host, then enqueues one kernel.  Returns hipSuccess,
// hipErrorInvalidValue for a problem the kernel cannot take, or the launch error.
hipError_t launch_gemm(const GemmProblem& p, hipStream_t stream);
bool gemm_dma_accepts(const GemmProblem& p);
hipError_t launch_gemm_dma(const GemmProblem& p, hipStream_t stream);
double gemm_flops(const GemmProblem& p);
double gemm_bytes(const GemmProblem& p);

// Softmax cross-entropy over `rows` rows of float32 logits [rows, ldz], `classes` used columns.
// Writes dz (dtype, [rows, lddz]) = (softmax - onehot) / rows with zeros in columns classes..lddz-1,
// row_loss[rows] (float32), then a
// second kernel adds row_loss up in a fixed order into loss_out[0] = mean.
hipError_t launch_softmax_xent(const float* logits, int ldz, const int32_t* labels, int rows, int classes,
                               void* dz, int lddz, DType dz_dtype, float* row_loss, float* loss_out,
                               hipStream_t stream);

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t stream);

}  // namespace spb
