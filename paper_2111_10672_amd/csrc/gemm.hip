// Dense products on the matrix cores of gfx950 (CDNA4), float32 accumulation.
//
//   C[m, n] = sum_k A(m, k) * B(n, k)
//
// serves the three products of a fully connected layer (Sec. 2 of the paper, the forward pass and
// the backward pass over the units above the cut):
//   forward          Z  = X  * W^T      A = X  (RowK)   B = W (RowK)
//   input gradient   dX = dZ * W        A = dZ (RowK)   B = W (KRow)
//   weight gradient  dW = dZ^T * X      A = dZ (KRow)   B = X (KRow)   (+ bias gradient = row sums of A)
//
// One workgroup of 256 threads (4 wavefronts of 64) computes a BM x BN tile.  Both operands are
// staged through LDS as [row][128 bytes of k], so that every MFMA operand is one 16-byte LDS read
// per lane; operands whose rows are the contiguous index in memory are transposed on the way in
// (four 16-byte global loads per thread, a register transpose, short LDS writes).  The 16-byte
// chunks of an LDS row are XOR-swizzled by the row number so that neither the MFMA reads (32
// consecutive rows, same chunk) nor the transposed writes (rows 8 apart) pile onto one bank group.
// Global loads for tile t+1 are in flight while tile t is multiplied (register prefetch, two LDS
// buffers, one barrier per tile).
#include "gemm_common.h"

namespace spb {
using namespace gemm_detail;
namespace {

// ---- operand loaders: global -> registers -> LDS [row][k] ------------------------------------

// Reduction index contiguous in memory: 16-byte chunks go straight through.
template <typename T, int ROWS>
struct RowKLoader {
  static constexpr int kPer = Elem<T>::kPerChunk;
  static constexpr int kItems = ROWS * kChunks / kThreads;
  static_assert(ROWS * kChunks % kThreads == 0, "tile rows must fill the workgroup");
  u32x4 reg[kItems];

  __device__ __forceinline__ void load(const T* base, int ld, int row0, int nrows, int k0, int K) {
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int c = threadIdx.x + i * kThreads;
      const int gr = row0 + (c >> 3), gk = k0 + (c & 7) * kPer;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (gr < nrows && gk < K) {
        v = *reinterpret_cast<const u32x4*>(base + (size_t)gr * ld + gk);
        if (gk + kPer > K) {  // ragged last chunk of k: the pitch covers it, its contents are not data
          const int keep = K - gk;
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            if constexpr (sizeof(T) == 4) {
              if (d >= keep) v[d] = 0u;
            } else {
              if (2 * d >= keep) v[d] = 0u;
              else if (2 * d + 1 >= keep) v[d] &= 0xFFFFu;
            }
          }
        }
      }
      reg[i] = v;
    }
  }
  __device__ __forceinline__ void store(char* lds) const {
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int c = threadIdx.x + i * kThreads;
      *reinterpret_cast<u32x4*>(lds + lds_offset(c >> 3, c & 7)) = reg[i];
    }
  }
};

// Row index contiguous in memory: each thread takes a block of 4 k-rows x one 16-byte chunk of rows
// and writes it transposed.
template <typename T, int ROWS>
struct KRowLoader {
  static constexpr int kPer = Elem<T>::kPerChunk;
  static constexpr int kRowChunks = ROWS / kPer;
  static constexpr int kQuads = Elem<T>::kTileK / 4;
  static constexpr int kBlocks = kRowChunks * kQuads;
  static constexpr int kItems = (kBlocks + kThreads - 1) / kThreads;
  u32x4 reg[kItems][4];

  __device__ __forceinline__ void load(const T* base, int ld, int row0, int nrows, int k0, int K) {
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int id = threadIdx.x + i * kThreads;
      const int rc = id % kRowChunks, kq = id / kRowChunks;
      const int gr = row0 + rc * kPer;
      const bool live = (kBlocks % kThreads == 0 || id < kBlocks) && gr < nrows;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int gk = k0 + kq * 4 + j;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (live && gk < K) v = *reinterpret_cast<const u32x4*>(base + (size_t)gk * ld + gr);
        reg[i][j] = v;
      }
      if (live && gr + kPer > nrows) {  // ragged last chunk of rows: clear what lies beyond the matrix
        const int keep = nrows - gr;    // 1 .. kPer-1 elements are real
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            uint32_t w = reg[i][j][d];
            if constexpr (sizeof(T) == 4) {
              if (d >= keep) w = 0u;
            } else {
              if (2 * d >= keep) w = 0u;
              else if (2 * d + 1 >= keep) w &= 0xFFFFu;
            }
            reg[i][j][d] = w;
          }
        }
      }
    }
  }
  __device__ __forceinline__ void store(char* lds) const {
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int id = threadIdx.x + i * kThreads;
      if (kBlocks % kThreads != 0 && id >= kBlocks) break;
      const int rc = id % kRowChunks, kq = id / kRowChunks;
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        const int row = rc * kPer + e;
        if constexpr (sizeof(T) == 4) {
          u32x4 o = {reg[i][0][e], reg[i][1][e], reg[i][2][e], reg[i][3][e]};
          *reinterpret_cast<u32x4*>(lds + lds_offset(row, kq)) = o;
        } else {
          const int d = e >> 1;
          uint32_t lo, hi;
          if ((e & 1) == 0) {
            lo = (reg[i][0][d] & 0xFFFFu) | (reg[i][1][d] << 16);
            hi = (reg[i][2][d] & 0xFFFFu) | (reg[i][3][d] << 16);
          } else {
            lo = (reg[i][0][d] >> 16) | (reg[i][1][d] & 0xFFFF0000u);
            hi = (reg[i][2][d] >> 16) | (reg[i][3][d] & 0xFFFF0000u);
          }
          uint2 o = make_uint2(lo, hi);
          *reinterpret_cast<uint2*>(lds + lds_offset(row, kq >> 1) + (kq & 1) * 8) = o;
        }
      }
    }
  }
};

template <typename T, int ROWS, Layout L> struct LoaderOf;
template <typename T, int ROWS> struct LoaderOf<T, ROWS, Layout::RowK> { using type = RowKLoader<T, ROWS>; };
template <typename T, int ROWS> struct LoaderOf<T, ROWS, Layout::KRow> { using type = KRowLoader<T, ROWS>; };

// ---- matrix-core step: one 16-byte chunk pair per lane ---------------------------------------
// 32x32 MFMA: lane l supplies row (l % 32) of each operand and the k-slice selected by l / 32.
__device__ __forceinline__ f32x16 mma(bf16_t, u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mma(float, u32x4 a, u32x4 b, f32x16 c) {
  // four k-steps of 2; lanes 0-31 and 32-63 hold different chunks, the same pairing for A and B
#pragma unroll
  for (int e = 0; e < 4; ++e)
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[e]), __uint_as_float(b[e]), c, 0, 0, 0);
  return c;
}

template <typename T, int BM, int BN, int WAVES_M, int WAVES_N, Layout LA, Layout LB>
__global__ __launch_bounds__(kThreads) void gemm_kernel(GemmParams p) {
  static_assert(WAVES_M * WAVES_N == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1 && WM % 32 == 0 && WN % 32 == 0, "wave tile is a multiple of 32x32");
  constexpr int TILE_K = Elem<T>::kTileK;

  extern __shared__ __attribute__((aligned(16))) char lds[];
  auto a_buf = [&](int i) { return lds + i * (BM * kRowBytes); };
  auto b_buf = [&](int i) { return lds + 2 * BM * kRowBytes + i * (BN * kRowBytes); };

  const int tile = xcd_tile(blockIdx.x, p.tiles_m * p.tiles_n);
  const int tile_m = tile % p.tiles_m, tile_n = tile / p.tiles_m;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;

  typename LoaderOf<T, BM, LA>::type la;
  typename LoaderOf<T, BN, LB>::type lb;
  const T* A = static_cast<const T*>(p.A);
  const T* B = static_cast<const T*>(p.B);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const bool want_row_sum = p.a_row_sum != nullptr && tile_n == 0;
  float row_sum = 0.f;

  const int n_steps = (p.K + TILE_K - 1) / TILE_K;
  la.load(A, p.lda, m0, p.M, 0, p.K);
  lb.load(B, p.ldb, n0, p.N, 0, p.K);
  la.store(a_buf(0));
  lb.store(b_buf(0));
  __syncthreads();

  for (int t = 0; t < n_steps; ++t) {
    const int cur = t & 1;
    if (t + 1 < n_steps) {
      la.load(A, p.lda, m0, p.M, (t + 1) * TILE_K, p.K);
      lb.load(B, p.ldb, n0, p.N, (t + 1) * TILE_K, p.K);
    }
    const char* as = a_buf(cur);
    const char* bs = b_buf(cur);
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) {
      const int chunk = 2 * kg + (lane >> 5);
      u32x4 a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const u32x4*>(as + lds_offset(wm * WM + i * 32 + (lane & 31), chunk));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const u32x4*>(bs + lds_offset(wn * WN + j * 32 + (lane & 31), chunk));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mma(T{}, a[i], b[j], acc[i][j]);
    }
    if (want_row_sum && threadIdx.x < BM) {
#pragma unroll
      for (int c = 0; c < kChunks; ++c) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(as + lds_offset(threadIdx.x, c));
        if constexpr (sizeof(T) == 4) {
#pragma unroll
          for (int d = 0; d < 4; ++d) row_sum += __uint_as_float(v[d]);
        } else {
#pragma unroll
          for (int d = 0; d < 4; ++d) row_sum += __uint_as_float(v[d] << 16) + __uint_as_float(v[d] & 0xFFFF0000u);
        }
      }
    }
    if (t + 1 < n_steps) {
      la.store(a_buf(cur ^ 1));
      lb.store(b_buf(cur ^ 1));
    }
    __syncthreads();
  }

  if (want_row_sum && threadIdx.x < BM && m0 + (int)threadIdx.x < p.M) p.a_row_sum[m0 + threadIdx.x] = row_sum;

  store_tile<T, TM, TN>(p, acc, m0 + wm * WM, n0 + wn * WN, lane);
}

template <typename T, int BM, int BN, int WAVES_M, int WAVES_N, Layout LA, Layout LB>
hipError_t launch_tile(const GemmProblem& q, hipStream_t stream) {
  GemmParams p = make_params(q, BM, BN);
  const size_t lds_bytes = (size_t)2 * (BM + BN) * kRowBytes;
  auto kernel = gemm_kernel<T, BM, BN, WAVES_M, WAVES_N, LA, LB>;
  if (lds_bytes > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kernel, dim3(p.tiles_m * p.tiles_n), dim3(kThreads), lds_bytes, stream, p);
  return hipGetLastError();
}

template <typename T, Layout LA, Layout LB>
hipError_t launch_layouts(const GemmProblem& q, hipStream_t stream) {
  const long big_tiles = (long)((q.M + 127) / 128) * ((q.N + 127) / 128);
  if (big_tiles >= 192) return launch_tile<T, 128, 128, 2, 2, LA, LB>(q, stream);
  return launch_tile<T, 64, 64, 2, 2, LA, LB>(q, stream);
}

template <typename T>
hipError_t launch_typed(const GemmProblem& q, hipStream_t stream) {
  if (q.a_layout == Layout::RowK && q.b_layout == Layout::RowK) return launch_layouts<T, Layout::RowK, Layout::RowK>(q, stream);
  if (q.a_layout == Layout::RowK && q.b_layout == Layout::KRow) return launch_layouts<T, Layout::RowK, Layout::KRow>(q, stream);
  if (q.a_layout == Layout::KRow && q.b_layout == Layout::KRow) return launch_layouts<T, Layout::KRow, Layout::KRow>(q, stream);
  return hipErrorInvalidValue;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

double gemm_flops(const GemmProblem& p) { return 2.0 * p.M * p.N * p.K * p.batch; }

double gemm_bytes(const GemmProblem& p) {
  const double es = (double)dtype_size(p.dtype);
  const double out = p.epilogue == Epilogue::StoreF32 ? 4.0 : es;
  // an implicit-GEMM operand is the tensor it is gathered from, read once, not its unrolled matrix
  const double tensor = (double)p.conv.n * p.conv.sh * p.conv.sw * p.conv.sc;
  const double a = p.a_gather == Gather::ConvRows ? tensor : (double)p.M * p.K;
  const double bm = p.b_gather == Gather::ConvPatchT ? tensor
                  : p.b_gather == Gather::ConvWeightT ? (double)p.conv.w_cout * p.conv.r * p.conv.s * p.conv.w_cin : (double)p.N * p.K;
  double b = es * (a + bm) + out * (double)p.M * p.N * p.k_splits;
  if (p.mask) b += es * (double)p.M * p.N;
  if (p.residual) b += es * (double)p.M * p.N;
  if (p.aux_out) b += es * (double)p.M * p.N;
  return b * p.batch;
}

namespace {
// what every product must satisfy, whichever kernel takes it
bool operands_valid(const GemmProblem& p) {
  const int per = p.dtype == DType::F32 ? 4 : 8;  // elements per 16-byte chunk
  if (p.M <= 0 || p.N <= 0 || p.K <= 0 || !p.A || !p.B || !p.C) return false;
  if (!aligned16(p.A) || !aligned16(p.B)) return false;
  // Vector loads: the contiguous extent of each operand must be whole 16-byte chunks inside its pitch.
  if (p.lda % per || p.ldb % per) return false;
  auto extent_ok = [&](Layout l, int rows, int ld) {
    const int extent = l == Layout::RowK ? p.K : rows;
    return (extent + per - 1) / per * per <= ld;
  };
  if (!extent_ok(p.a_layout, p.M, p.lda) || !extent_ok(p.b_layout, p.N, p.ldb)) return false;
  if (p.ldc < p.N) return false;
  if (p.epilogue == Epilogue::MaskStore && (!p.mask || p.ldmask < p.N)) return false;
  return true;
}
}  // namespace

hipError_t launch_gemm(const GemmProblem& p, hipStream_t stream) {
  if (!operands_valid(p)) return hipErrorInvalidValue;
  if (p.dtype == DType::BF16 && gemm_dma_accepts(p)) return launch_gemm_dma(p, stream);
  if (p.dtype == DType::F32 && gemm_f32_small_accepts(p)) return launch_gemm_f32_small(p, stream);
  // the register-staged kernel below knows only the dense-layer epilogues of a single product
  if (p.batch != 1 || p.alpha != 1.f || p.residual || p.aux_out || p.act == Act::Gelu || p.epilogue == Epilogue::ScaleStore ||
      p.epilogue == Epilogue::AffineBwdStore ||
      p.col_scale || p.a_gather != Gather::None || p.b_gather != Gather::None || p.k_splits != 1)
    return hipErrorInvalidValue;
  if (p.dtype == DType::F32) return launch_typed<float>(p, stream);
  return launch_typed<bf16_t>(p, stream);
}

bool gemm_pair_shares_launch(const GemmProblem& d, const GemmProblem& w) {
  return d.dtype == DType::BF16 && w.dtype == DType::BF16 && operands_valid(d) && operands_valid(w) && gemm_dma_accepts(d) &&
         gemm_dma_accepts(w) && gemm_dma_pair_accepts(d, w);
}

hipError_t launch_gemm_pair(const GemmProblem& d, const GemmProblem& w, hipStream_t stream) {
  if (gemm_pair_shares_launch(d, w)) return launch_gemm_dma_pair(d, w, stream);
  hipError_t e = launch_gemm(w, stream);
  if (e != hipSuccess) return e;
  return launch_gemm(d, stream);
}

}  // namespace spb
