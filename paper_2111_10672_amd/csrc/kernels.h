// Host-side launch interface of the HIP kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <map>
#include <mutex>
#include <utility>

#include "bf16_round.h"

namespace spb {

enum class DType : int { F32 = 0, BF16 = 1 };

inline size_t dtype_size(DType t) { return t == DType::F32 ? 4 : 2; }

// How an operand of the product C[m, n] = sum_k A(m, k) * B(n, k) lies in memory.
enum class Layout : int {
  RowK = 0,  // element (row, k) at base[row * ld + k]: the reduction index is contiguous
  KRow = 1,  // element (row, k) at base[k * ld + row]: the row index is contiguous
};

enum class Epilogue : int {
  StoreF32 = 0,      // C float32 = alpha * acc (+ bias[n])
  BiasAct = 1,       // v = alpha * acc * col_scale[n] + bias[n]; aux_out (T) = v if given; C (T) = act(v + residual[m, n])
  MaskStore = 2,     // C (T) = mask[m, n] > 0 ? acc : 0          (ReLU backward fused into the input-gradient product)
  ScaleStore = 3,    // C (T) = acc * mask[m, n]                  (GELU backward; mask holds gelu'(pre-activation) as the forward pass stored it)
  // Backward of "per-channel affine, then ReLU" fused into the input-gradient product that forms the gradient at the
  // ReLU's output: d = acc rounded to T (what a separate pass would have read back), dz = mask[m, n] > 0 ? d : 0,
  // C (T) = col_scale[n] * dz, and per tile row of the product col_partial[tile_m][0][n] = sum over its rows of
  // dz * affine_y[m, n], col_partial[tile_m][1][n] = sum of dz (float32; reduce_pairs adds the tile rows up).
  // With residual: d = acc + residual[m, n] before the rounding; with aux_out: aux_out (T) = dz.
  AffineBwdStore = 4,
};

enum class Act : int { None = 0, Relu = 1, Gelu = 2 };

// An operand that is not a stored matrix but a view of an NHWC tensor (implicit GEMM of a convolution).
enum class Gather : int {
  None = 0,
  ConvRows = 1,     // A, RowK: row m = pixel (n, a, b) of a [N, RH, RW] grid; k = (tap, channel) of the gathered tensor
  ConvWeightT = 2,  // B, KRow: weights [Cout][R*S][Cin] read as B(ci, (tap, co))            (input-gradient product)
  ConvPatchT = 3,   // B, KRow: B((tap, ci), m) = x[pixel(m) shifted by tap][ci]             (weight-gradient product)
};

struct ConvGeom {
  int n = 0, sh = 0, sw = 0, sc = 0;  // the gathered tensor: [n, sh, sw, sc], NHWC
  int rh = 0, rw = 0;                 // spatial size of the grid the implicit matrix's pixel index runs over
  int r = 1, s = 1, stride = 1, pad = 0;
  int transposed = 0;                 // 0: source = grid * stride + tap - pad; 1: source = (grid + pad - tap) / stride if divisible
  int w_cin = 0, w_cout = 0;          // ConvWeightT: the weight tensor is [w_cout][r * s][w_cin]
};

// Element offset of batch entry z of an operand: (z / inner_count) * outer + (z % inner_count) * inner.
struct BatchStride {
  long long outer = 0, inner = 0;
  int inner_count = 1;
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
  int relu = 0;                   // shorthand for act = Relu
  Act act = Act::None;
  float alpha = 1.f;
  const void* residual = nullptr; int ldres = 0;   // [M, N], dtype, added to the biased value BEFORE the activation (BiasAct): C = act(v + residual)
  void* aux_out = nullptr; int ldaux = 0;          // [M, N], dtype, receives the pre-activation (BiasAct)
  const void* col_scale = nullptr;                 // [N], dtype: v = alpha * acc * col_scale[n] + bias[n]   (BiasAct)
  int aux_raw = 0;                                 // aux_out receives alpha * acc instead of the pre-activation
  int aux_act_grad = 0;                            // act = Gelu: aux_out receives gelu'(v) instead of v (all the backward pass needs of v)
  int batch = 1;                  // independent products launched together (attention heads)
  BatchStride a_batch, b_batch, c_batch;
  Gather a_gather = Gather::None, b_gather = Gather::None;
  ConvGeom conv;
  // > 1: the k range is cut into k_splits slices; slice z writes its float32 partial product to C + z * M * ldc
  // (StoreF32 only); the caller adds the slices up.
  int k_splits = 1;
  const void* mask = nullptr; int ldmask = 0;   // [M, N], dtype
  // The buffer's owner keeps zeros between the end of each row's data and the next multiple of 8 elements
  // along the contiguous index (lets a kernel fetch whole 16-byte chunks).
  bool a_pad_zero = false, b_pad_zero = false;
  // The product runs beside workgroups of another stream: where the tile choice is between one 128 x 128 workgroup
  // that takes most of a CU's LDS and one that leaves room for a neighbour, take the latter.
  bool share_cu = false;
  float* a_row_sum = nullptr;     // optional [M]: sum_k A(m, k), written once by the tiles of column block 0
  // AffineBwdStore: the affine's input (pre-affine convolution output), the partial column sums [tile rows][2][N]
  // (room for (M + 63) / 64 tile rows) and where the launcher reports how many tile rows it wrote
  const void* affine_y = nullptr;
  int ldaffine_y = 0;
  float* col_partial = nullptr;
  int* col_partial_rows = nullptr;
  const char* name = "gemm";
};

// A kernel that wants more than 64 KiB of dynamic LDS has to ask once.  The answer is kept per kernel (and per
// device: each device has its own copy of the function), behind a lock: models on several host threads launch the
// same instantiations.
inline hipError_t raise_lds_limit(const void* kernel, size_t lds_bytes) {
  static std::mutex lock;
  static std::map<std::pair<const void*, int>, hipError_t> done;
  int device = 0;
  if (hipError_t e = hipGetDevice(&device); e != hipSuccess) return e;
  std::lock_guard<std::mutex> guard(lock);
  auto key = std::make_pair(kernel, device);
  auto it = done.find(key);
  if (it != done.end()) return it->second;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e == hipSuccess) done.emplace(key, e);
  return e;
}

// Checks shapes and alignment on the host, then enqueues one kernel.  Returns hipSuccess,
// hipErrorInvalidValue for a problem the kernel cannot take, or the launch error.
hipError_t launch_gemm(const GemmProblem& p, hipStream_t stream);
bool gemm_dma_accepts(const GemmProblem& p);
hipError_t launch_gemm_dma(const GemmProblem& p, hipStream_t stream);
// float32 products of small dense layers (latency-bound): see gemm_f32_small.hip
bool gemm_f32_small_accepts(const GemmProblem& p);
hipError_t launch_gemm_f32_small(const GemmProblem& p, hipStream_t stream);
// The input-gradient product d (RowK x KRow) and the weight-gradient product w (KRow x KRow) of one dense layer,
// which do not depend on each other: one launch when both are small enough for the small-product kernel
// (gemm_pair_shares_launch says whether), otherwise w and then d, one launch each.
bool gemm_pair_shares_launch(const GemmProblem& d, const GemmProblem& w);
hipError_t launch_gemm_pair(const GemmProblem& d, const GemmProblem& w, hipStream_t stream);
bool gemm_dma_pair_accepts(const GemmProblem& d, const GemmProblem& w);
hipError_t launch_gemm_dma_pair(const GemmProblem& d, const GemmProblem& w, hipStream_t stream);
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

// ---- memory-bound kernels of the residual-CNN units (NHWC bfloat16, channels % 8 == 0, <= 2048) ----
// Backward of "per-channel affine, then optional ReLU whose output is act": dz = dout * [act > 0] (dz = dout if act is
// null); dy = scale * dz; dsum = dz (optional); dscale[c] = sum dz * y; dshift[c] = sum dz (float32, overwritten).
// partial: scratch of affine_partial_floats(rows, channels) floats.
// With `deferred` the column sums stay per-workgroup partial sums and *deferred describes the reduction that finishes
// them (for launch_unit_reduce); dscale and dshift are written by that reduction.
size_t affine_partial_floats(long long rows, int channels);
// One small fixed-order reduction: kPairs = the column sums of an affine backward pass (partial [count][2][width] ->
// out [width], out_b [width]); kSlices / kSlices4 = the k-slices of a weight gradient (see launch_splitk_reduce;
// kSlices4 counts in groups of four floats).  blocks = workgroups it takes.
struct ReduceTask {
  enum Kind { kPairs = 0, kSlices4 = 1, kSlices = 2 };
  int kind = kPairs;
  const float* partial = nullptr;
  int count = 0, width = 0;
  long long stride = 0, numel = 0;
  float* out = nullptr;
  float* out_b = nullptr;
  int cin = 0, cin_padded = 0;
  unsigned blocks = 0;
};
inline unsigned reduce_pairs_blocks(int width) { return (unsigned)((2 * width + 15) / 16); }   // workgroups of a kPairs task
struct ReduceTable {
  static constexpr int kMax = 32;
  int n = 0;
  unsigned end_block[kMax] = {};
  ReduceTask task[kMax];
};
hipError_t launch_affine_relu_bwd(const void* dout, const void* act, const void* y, const void* scale, void* dy, void* dsum,
                                  float* partial, float* dscale, float* dshift, long long rows, int channels, hipStream_t s,
                                  ReduceTask* deferred = nullptr);
// The reduction launch_splitk_reduce would run, as a task; false if the arguments are not valid.
bool make_splitk_reduce_task(const float* partial, int slices, long long slice_stride, float* out, long long numel, int cin, int cin_padded,
                             ReduceTask* task);
// All of the tasks in one launch (several if there are more than ReduceTable::kMax), same bits as one launch each.
hipError_t launch_unit_reduce(const ReduceTask* tasks, int n, hipStream_t s);
// out[j] = sum over slices of partial[slice * slice_stride + map(j)], j < numel; map(j) = j, or with cin < cin_padded
// (j / cin) * cin_padded + j % cin (drops the zero channels a 3-channel input was padded with).
hipError_t launch_splitk_reduce(const float* partial, int slices, long long slice_stride, float* out, long long numel, int cin, int cin_padded,
                                hipStream_t s);
// out[j] (bfloat16) = sum over slices of partial[slice * slice_stride + j], j < numel; numel a multiple of 8, 16-byte aligned.
hipError_t launch_splitk_reduce_bf16(const float* partial, int slices, long long slice_stride, void* out, long long numel, hipStream_t s);
// 3x3 / stride 2 / padding 1 max-pool of x [n, h, w, c]; which (optional, [n, oh, ow, c]) records the winning window position.
hipError_t launch_maxpool_fwd(const void* x, void* out, uint8_t* which, int n, int h, int w, int c, hipStream_t s);
hipError_t launch_maxpool_bwd(const void* dout, const uint8_t* which, void* da, int n, int h, int w, int c, hipStream_t s);
// global average pool of x [n, hw, c] -> pooled [n, c], and its backward (broadcast / hw)
hipError_t launch_avgpool_fwd(const void* x, void* pooled, int n, int hw, int c, hipStream_t s);
hipError_t launch_avgpool_bwd(const void* dpooled, void* dx, int n, int hw, int c, hipStream_t s);
// out[row, :] = in[row, :c_in] followed by zeros up to c_out
hipError_t launch_pad_channels(const void* in, void* out, long long rows, int c_in, int c_out, hipStream_t s);

// ---- row-wise kernels of the encoder units (bfloat16 rows of `width` elements, width % 8 == 0, <= 2048) ----
// y[r] = LayerNorm(x[rows ? rows[r] : r]) for r < n_rows; stats[r] = (mean, 1 / sqrt(var + 1e-5)).
hipError_t launch_layernorm_fwd(const void* x, int ldx, const int32_t* rows, int n_rows, int width, const void* gamma, const void* beta,
                                void* y, int ldy, float* stats, hipStream_t s);
// LayerNorm backward.  dy and stats are indexed by r, x and dx by rows ? rows[r] : r.  dx (optional) receives the input
// gradient plus res[r] (optional).  dgamma/dbeta (float32 [width]) are overwritten; partial is scratch of
// layernorm_partial_floats(n_rows, width) floats.  With `deferred` the column sums are not added up here: the task
// describes that reduction for a later launch_unit_reduce, and `partial` must stay untouched until then.
size_t layernorm_partial_floats(int n_rows, int width);
hipError_t launch_layernorm_bwd(const void* dy, int lddy, const void* x, int ldx, const int32_t* rows, const float* stats,
                                const void* gamma, const void* res, int ldres, void* dx, int lddx, float* partial,
                                float* dgamma, float* dbeta, int n_rows, int width, hipStream_t s, ReduceTask* deferred = nullptr);
// prob (bfloat16) = softmax of each row of scores (float32), rows of `len` contiguous entries.
hipError_t launch_softmax_fwd(const float* scores, void* prob, long long n_rows, int len, hipStream_t s);
// dscore (bfloat16) = prob * (dprob - sum(dprob * prob)) * scale per row.
hipError_t launch_softmax_bwd(const float* dprob, const void* prob, void* dscore, long long n_rows, int len, float scale, hipStream_t s);
// out[m] = tok[ids[m]] + pos[m % seq];  gradients: dtok (float32 [vocab, width], overwritten), dpos (float32 [seq, width]).
hipError_t launch_embedding_fwd(const int32_t* ids, const void* tok, const void* pos, void* out, int ldo, int n_rows, int seq, int vocab,
                                int width, hipStream_t s);
hipError_t launch_embedding_bwd(const int32_t* ids, const void* dx, int lddx, float* dtok, float* dpos, int batch, int seq, int vocab,
                                int width, hipStream_t s);

// Fused attention forward (attention.hip): per (batch entry, head), ctx = softmax(Q K^T * scale) V with Q, K, V the
// three column blocks of qkv [batch * seq, 3 * heads * head_dim]; prob [batch * heads, seq, seq] (bfloat16) is
// written only when non-null.  attention_fused_accepts says which shapes it takes (head_dim 64, seq <= 128, ...).
bool attention_fused_accepts(int seq, int head_dim, int ld_qkv, int ld_ctx);
hipError_t launch_attention_fwd(const void* qkv, int ld_qkv, void* prob, void* ctx, int ld_ctx, int batch, int heads, int seq,
                                int head_dim, float scale, hipStream_t stream);

// Its backward: dqkv [batch * seq, 3 * heads * head_dim] receives dQ, dK, dV from prob (as the forward wrote it),
// qkv and dctx [batch * seq, heads * head_dim].
hipError_t launch_attention_bwd(const void* qkv, int ld_qkv, const void* prob, const void* dctx, int ld_ctx, void* dqkv, int batch,
                                int heads, int seq, int head_dim, float scale, hipStream_t stream);

// Server-side aggregation and update (aggregate.hip): for each tensor, g = mean of `count` float32 worker
// gradients (added in the order given), v = momentum * v + g + weight_decay * w, w = w - rate * v.  w is in
// param_dtype (bfloat16 parameters are rounded to nearest-even after the float32 update), v is float32.
constexpr int kMaxAggWorkers = 8;
struct AggregateTensor {
  void* w = nullptr;
  float* v = nullptr;
  const float* g[kMaxAggWorkers] = {};
  long long numel = 0;
  int count = 0;
  float rate = 0.f;
};
hipError_t launch_aggregate_update(const AggregateTensor* tensors, int n_tensors, DType param_dtype, float momentum,
                                   float weight_decay, hipStream_t stream);

}  // namespace spb

