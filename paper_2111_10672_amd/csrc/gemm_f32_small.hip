// float32 products of small dense layers (the perceptron configurations), C[m, n] = sum_k A(m, k) * B(n, k).
//
// Same scheme as the bfloat16 small-product kernel: such a product is a chain of latencies, so a workgroup owns
// one 32 x 32 tile, its four waves split the k range into four contiguous parts, each wave streams its part
// through a tile ring of its own in LDS with direct-to-LDS loads and waits only on its own loads (no barrier in
// the tile loop), and the four partial tiles are added up through LDS at the end, each wave finishing 8 rows.
// A tile is 32 values of k (128 bytes per row).  The matrix-core instruction is v_mfma_f32_32x32x2_f32: a lane
// supplies one value of A (row lane % 32) and one of B per instruction, and WHICH two values of k an instruction
// multiplies is free as long as both operands agree, so the lanes of half h take k = 4 h + e in instruction e and
// a fragment of four instructions is one 16-byte LDS read per operand (RowK) or four 4-byte reads (KRow).
#include "gemm_common.h"

namespace spb {
namespace {
using namespace gemm_detail;

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* global_ptr_t;

static __device__ const uint32_t kZeroChunk32[4] = {0u, 0u, 0u, 0u};

constexpr int kTile = 32;      // values of k per tile
constexpr int kRing = 4;       // tiles per wave in flight
constexpr int kStage = 64 * kRowBytes;  // A tile (32 rows) + B tile (32 rows)
constexpr int kLoads = 8;      // direct-to-LDS instructions per tile
constexpr int kPitch = 36;     // floats per parked row; column 32 carries the row sum of A

constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 15) << 8); }
template <int VM>
__device__ __forceinline__ void wait_own_loads() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(VM, 15));
  asm volatile("" ::: "memory");
}

// One lane's four 16-byte chunks of a 32-row operand tile: source pointers for the wave's first tile, stepped
// from tile to tile.  A chunk outside the matrix is fetched from a chunk of zeros.
template <Layout L>
struct Source32 {
  const char* ptr[4];
  int k_in_tile[4];
  bool in_rows[4];
  size_t tile_step;
  __device__ __forceinline__ void init(const float* base, int ld, int row0, int nrows, int lane, int t0) {
    tile_step = L == Layout::RowK ? (size_t)kTile * 4 : (size_t)kTile * ld * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int slot = i * 64 + lane;
      int gr, k;
      if constexpr (L == Layout::RowK) {
        const int row = slot >> 3, pc = slot & 7;
        gr = row0 + row;
        k = ((pc ^ row ^ (row >> 3)) & 7) << 2;
      } else {
        k = slot >> 3;
        gr = row0 + ((slot & 7) << 2);
      }
      k_in_tile[i] = k;
      in_rows[i] = gr < nrows;
      ptr[i] = reinterpret_cast<const char*>(L == Layout::RowK ? base + (size_t)gr * ld + k : base + (size_t)k * ld + gr) + (size_t)t0 * tile_step;
    }
  }
  __device__ __forceinline__ void issue(int t, int K, char* tile) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const char* src = in_rows[i] && t * kTile + k_in_tile[i] < K ? ptr[i] : reinterpret_cast<const char*>(kZeroChunk32);
      ptr[i] += tile_step;
      __builtin_amdgcn_global_load_lds((global_ptr_t)src, (lds_ptr_t)(tile + i * 1024), 16, 0, 0);
    }
  }
};

// The four values a lane supplies to the four MFMAs of k-group g (8 values of k): k = 8 g + 4 (lane / 32) + e.
template <Layout L>
__device__ __forceinline__ f32x4 read_fragment32(const char* tile, int g, int lane) {
  if constexpr (L == Layout::RowK) {
    return *reinterpret_cast<const f32x4*>(tile + lds_offset(lane & 31, 2 * g + (lane >> 5)));
  } else {
    f32x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = *reinterpret_cast<const float*>(tile + (8 * g + 4 * (lane >> 5) + e) * kRowBytes + (lane & 31) * 4);
    return v;
  }
}

template <Layout LA, Layout LB>
__global__ __launch_bounds__(256) void gemm_f32_small_kernel(GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tile = xcd_tile(blockIdx.x, p.tiles_m * p.tiles_n);
  const int tile_m = tile % p.tiles_m, tile_n = tile / p.tiles_m;
  const int m0 = tile_m * 32, n0 = tile_n * 32;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* ring = lds + wave * (kRing * kStage);

  const int tiles = (p.K + kTile - 1) / kTile;
  const int per_wave = (tiles + 3) / 4;
  const int my_first = wave * per_wave;
  const int n = max(min(tiles, my_first + per_wave) - my_first, 0);  // tiles of this wave

  Source32<LA> src_a;
  Source32<LB> src_b;
  src_a.init(static_cast<const float*>(p.A), p.lda, m0, p.M, lane, my_first);
  src_b.init(static_cast<const float*>(p.B), p.ldb, n0, p.N, lane, my_first);
  auto issue = [&](int i) {
    char* stage = ring + (i % kRing) * kStage;
    src_a.issue(my_first + i, p.K, stage);
    src_b.issue(my_first + i, p.K, stage + 32 * kRowBytes);
  };
#pragma unroll
  for (int s = 0; s < kRing; ++s)
    if (s < n) issue(s);

  f32x16 acc, acc_sum;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[r] = 0.f; acc_sum[r] = 0.f; }
  // bias gradient of a weight-gradient product: row sums of A, as one more MFMA against ones
  const bool want_row_sum = p.a_row_sum != nullptr && tile_n == 0;

  for (int i = 0; i < n; ++i) {
    const int younger = min(kRing - 1, n - 1 - i);  // tiles issued after tile i that may still be in flight
    if (younger == 3) wait_own_loads<3 * kLoads>();
    else if (younger == 2) wait_own_loads<2 * kLoads>();
    else if (younger == 1) wait_own_loads<1 * kLoads>();
    else wait_own_loads<0>();
    const char* as = ring + (i % kRing) * kStage;
    const char* bs = as + 32 * kRowBytes;
    f32x4 a[4], b[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) { a[g] = read_fragment32<LA>(as, g, lane); b[g] = read_fragment32<LB>(bs, g, lane); }
    // the reads must have returned before the slot is handed to the next tile's loads
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int g = 0; g < 4; ++g) { asm volatile("" : "+v"(a[g])); asm volatile("" : "+v"(b[g])); }
    if (i + kRing < n) issue(i + kRing);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][e], b[g][e], acc, 0, 0, 0);
        if (want_row_sum) acc_sum = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][e], 1.0f, acc_sum, 0, 0, 0);
      }
    }
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
  __syncthreads();  // every wave is done with its ring: park the partial tiles there

  float* red = reinterpret_cast<float*>(lds);
  float* mine = red + wave * (32 * kPitch);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    mine[row * kPitch + (lane & 31)] = acc[r];
    if (want_row_sum && (lane & 31) == 0) mine[row * kPitch + 32] = acc_sum[r];
  }
  __syncthreads();

  // wave w finishes rows 8 w .. 8 w + 7: lane -> (row, 4 columns)
  const int row = 8 * wave + (lane >> 3), c = (lane & 7) * 4;
  const int m = m0 + row, nn = n0 + c;
  if (want_row_sum && lane < 8) {
    const float* at = red + (8 * wave + lane) * kPitch + 32;
    const float v = ((at[0] + at[32 * kPitch]) + at[2 * 32 * kPitch]) + at[3 * 32 * kPitch];
    if (m0 + 8 * wave + lane < p.M) p.a_row_sum[m0 + 8 * wave + lane] = v;
  }
  if (m >= p.M || nn >= p.N) return;
  const float* at = red + row * kPitch + c;
  f32x4 v = *reinterpret_cast<const f32x4*>(at);
#pragma unroll
  for (int w = 1; w < 4; ++w) v += *reinterpret_cast<const f32x4*>(at + w * (32 * kPitch));
  const float* bias = static_cast<const float*>(p.bias);
  const float* mask = static_cast<const float*>(p.mask);
  float* out = static_cast<float*>(p.C) + (size_t)m * p.ldc + nn;
  float o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float x = v[e];
    if (nn + e < p.N) {
      if (p.epilogue == (int)Epilogue::MaskStore) {
        if (!(mask[(size_t)m * p.ldmask + nn + e] > 0.f)) x = 0.f;
      } else {
        x += bias ? bias[nn + e] : 0.f;
        if (p.epilogue == (int)Epilogue::BiasAct && p.act == (int)Act::Relu) x = fmaxf(x, 0.f);
      }
    }
    o[e] = x;
  }
  if (nn + 4 <= p.N && (p.ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(p.C) & 15) == 0) {
    *reinterpret_cast<f32x4*>(out) = f32x4{o[0], o[1], o[2], o[3]};
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (nn + e < p.N) out[e] = o[e];
  }
}

template <Layout LA, Layout LB>
hipError_t launch(const GemmProblem& q, hipStream_t stream) {
  const GemmParams p = make_params(q, 32, 32);
  constexpr size_t lds_bytes = (size_t)4 * kRing * kStage;  // 128 KiB; the parked partial tiles (18 KiB) overlay it
  auto kernel = gemm_f32_small_kernel<LA, LB>;
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kernel), (size_t)lds_bytes); e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(p.tiles_m * p.tiles_n), dim3(256), lds_bytes, stream, p);
  return hipGetLastError();
}

}  // namespace

// Products this kernel takes: float32, one product, the dense-layer epilogues, at most a few tiles per CU, and
// operands whose partly filled 16-byte chunks (a k or row count that is not a multiple of 4) are zero-padded.
bool gemm_f32_small_accepts(const GemmProblem& p) {
  if (p.dtype != DType::F32 || p.batch != 1 || p.k_splits != 1 || p.alpha != 1.f || p.residual || p.aux_out || p.col_scale) return false;
  if (p.a_gather != Gather::None || p.b_gather != Gather::None) return false;
  if (p.act == Act::Gelu || p.epilogue == Epilogue::ScaleStore) return false;
  if (p.a_layout == Layout::KRow && p.b_layout == Layout::RowK) return false;
  auto ok = [&](Layout l, int rows, bool pad_zero) { return ((l == Layout::RowK ? p.K : rows) % 4 == 0) || pad_zero; };
  if (!ok(p.a_layout, p.M, p.a_pad_zero) || !ok(p.b_layout, p.N, p.b_pad_zero)) return false;
  return (long)((p.M + 31) / 32) * ((p.N + 31) / 32) <= 2048;
}

hipError_t launch_gemm_f32_small(const GemmProblem& p, hipStream_t stream) {
  if (!gemm_f32_small_accepts(p)) return hipErrorInvalidValue;
  if (p.a_layout == Layout::RowK && p.b_layout == Layout::RowK) return launch<Layout::RowK, Layout::RowK>(p, stream);
  if (p.a_layout == Layout::RowK && p.b_layout == Layout::KRow) return launch<Layout::RowK, Layout::KRow>(p, stream);
  return launch<Layout::KRow, Layout::KRow>(p, stream);
}

}  // namespace spb
