// Pieces shared by the GEMM kernels: vector types, bfloat16 storage helpers, kernel parameters, epilogue.
#pragma once
#include <utility>

#include "kernels.h"

namespace spb {
namespace gemm_detail {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct bf16_t { uint16_t bits; };

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose index is a constant expression
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

constexpr int kThreads = 256;
constexpr int kRowBytes = 128;  // bytes of k per LDS row and per tile step
constexpr int kChunks = 8;      // 16-byte chunks per LDS row

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int kPerChunk = 4; static constexpr int kTileK = 32; };
template <> struct Elem<bf16_t> { static constexpr int kPerChunk = 8; static constexpr int kTileK = 64; };

// Where 16-byte chunk `chunk` (8 bf16 of k) of row `row` of a RowK tile lies: rows of 128 bytes whose chunks are
// permuted by the row's low five bits, so that the 32 rows one matrix-core operand read touches fall into different
// banks.  Only the position of the row inside its 32-row fragment enters, which makes a fragment's address the
// address of fragment 0 plus a constant.
__device__ __forceinline__ int lds_offset(int row, int chunk) {
  return row * kRowBytes + (((chunk ^ row ^ ((row >> 3) & 3)) & 7) << 4);
}

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float(((uint32_t)v.bits) << 16); }

__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(bf16_t* p, float v) {
  p->bits = bf16_round(v);
}

struct GemmParams {
  const void* A; const void* B; void* C;
  const void* bias; const void* mask; float* a_row_sum;
  const void* residual; void* aux_out; const void* col_scale;
  const void* affine_y; float* col_partial; int ldy;
  int M, N, K, lda, ldb, ldc, ldmask, ldres, ldaux;
  int epilogue, act, aux_raw, aux_act_grad;
  float alpha;
  int k_tiles_per_split;  // 0: blockIdx.y is a batch entry; > 0: blockIdx.y is a slice of the k range
  // k-slices in multiples of 8: the grid is (slices, tiles), so that workgroup x + 8 i - slice x - runs on XCD x % 8.
  // The tiles of a slice read the same k range of both operands and belong behind one L2 (the encoder head's input
  // gradient, 30 tiles x 8 slices: 460 MB fetched with the slices dealt over all XCDs, against 84 MB of operands).
  int slice_in_x;
  ConvGeom conv;
  int tiles_m, tiles_n;
  BatchStride a_batch, b_batch, c_batch;
};

__device__ __forceinline__ long long batch_offset(const BatchStride& b, int z) {
  return (long long)(z / b.inner_count) * b.outer + (long long)(z % b.inner_count) * b.inner;
}

// erf by the five-term formula 7.1.26 of Abramowitz and Stegun, 1 - (a1 t + ... + a5 t^5) exp(-x^2) with
// t = 1 / (1 + p |x|): absolute error below 1.5e-7 everywhere, no branch, a dozen instructions.  The GELU
// epilogues evaluate it once per output element, which is what bounds them, so the library erf (several times
// the instructions, two divergent ranges) is not used.
// erf_parts(u): t-polynomial and exp(-u^2) of the formula, for u >= 0.
__device__ __forceinline__ void erf_parts(float au, float& pt, float& e) {
  const float t = __frcp_rn(fmaf(0.3275911f, au, 1.f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  pt = poly * t;
  e = __expf(-au * au);
}
__device__ __forceinline__ float gelu_f(float x) {
  float pt, e;
  erf_parts(fabsf(x) * 0.70710678118654752f, pt, e);
  const float erf_u = copysignf(fmaf(-pt, e, 1.f), x);
  return 0.5f * x * (1.f + erf_u);
}
// gelu(x) and gelu'(x) from one evaluation of the erf formula (the forward epilogue that stashes the derivative).
__device__ __forceinline__ void gelu_both_f(float x, float& y, float& dy) {
  float pt, e;
  erf_parts(fabsf(x) * 0.70710678118654752f, pt, e);
  const float cdf = 0.5f * (1.f + copysignf(fmaf(-pt, e, 1.f), x));
  y = x * cdf;
  dy = fmaf(x * 0.3989422804014327f, e, cdf);
}

// Accumulator register r of lane l of a 32x32 MFMA block holds C[8*(r/4) + 4*(l/32) + r%4][l%32].
template <typename T, int TM, int TN>
__device__ __forceinline__ void store_tile(const GemmParams& p, f32x16 (&acc)[TM][TN], int row_base, int col_base, int lane) {
  const T* bias = static_cast<const T*>(p.bias);
  const T* mask = static_cast<const T*>(p.mask);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = col_base + j * 32 + (lane & 31);
      if (n >= p.N) continue;
      const float bv = bias ? to_float(bias[n]) : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = row_base + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m >= p.M) continue;
        float v = acc[i][j][r];
        if (p.epilogue == (int)Epilogue::StoreF32) {
          static_cast<float*>(p.C)[(size_t)m * p.ldc + n] = v + bv;
        } else if (p.epilogue == (int)Epilogue::BiasAct) {
          v += bv;
          if (p.act == (int)Act::Relu) v = fmaxf(v, 0.f);
          store_elem(static_cast<T*>(p.C) + (size_t)m * p.ldc + n, v);
        } else {
          if (!(to_float(mask[(size_t)m * p.ldmask + n]) > 0.f)) v = 0.f;
          store_elem(static_cast<T*>(p.C) + (size_t)m * p.ldc + n, v);
        }
      }
    }
  }
}

inline GemmParams make_params(const GemmProblem& q, int bm, int bn) {
  GemmParams p;
  p.A = q.A; p.B = q.B; p.C = q.C; p.bias = q.bias; p.mask = q.mask; p.a_row_sum = q.a_row_sum;
  p.M = q.M; p.N = q.N; p.K = q.K; p.lda = q.lda; p.ldb = q.ldb; p.ldc = q.ldc; p.ldmask = q.ldmask;
  p.residual = q.residual; p.aux_out = q.aux_out; p.ldres = q.ldres; p.ldaux = q.ldaux;
  p.epilogue = (int)q.epilogue; p.act = q.relu ? (int)Act::Relu : (int)q.act;
  p.alpha = q.alpha; p.col_scale = q.col_scale; p.aux_raw = q.aux_raw; p.aux_act_grad = q.aux_act_grad;
  p.conv = q.conv;
  p.affine_y = q.affine_y; p.ldy = q.ldaffine_y; p.col_partial = q.col_partial;
  if (q.col_partial_rows) *q.col_partial_rows = (q.M + bm - 1) / bm;
  p.k_tiles_per_split = 0; p.slice_in_x = 0;
  p.a_batch = q.a_batch; p.b_batch = q.b_batch; p.c_batch = q.c_batch;
  p.tiles_m = (q.M + bm - 1) / bm;
  p.tiles_n = (q.N + bn - 1) / bn;
  return p;
}

// Consecutive workgroup ids land on different XCDs (round-robin over 8); give each XCD a contiguous
// run of tiles so that neighbours in a run share operand rows in that XCD's L2.
__device__ __forceinline__ int xcd_tile(int block, int n_tiles) {
  return n_tiles % 8 == 0 ? (block & 7) * (n_tiles >> 3) + (block >> 3) : block;
}

// The same run of tiles per XCD, but walked in groups of kTileGroupM tile rows (down a group's rows first, then to
// the next tile column), so that the tiles an XCD has in flight at one time form a compact block of the result:
// they share few operand row panels, and the XCD's L2 fills stay near (rows + columns) instead of (all rows + 1).
constexpr int kTileGroupM = 8;
__device__ __forceinline__ void xcd_tile_grouped(int block, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  const int run = xcd_tile(block, tiles_m * tiles_n);
  const int per_group = kTileGroupM * tiles_n;
  const int group = run / per_group, r = run - group * per_group;
  const int first_m = group * kTileGroupM;
  const int gm = min(tiles_m - first_m, kTileGroupM);
  tile_n = r / gm;
  tile_m = first_m + (r - tile_n * gm);
}

}  // namespace gemm_detail
}  // namespace spb
