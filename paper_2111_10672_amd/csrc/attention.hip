// Attention of one (batch entry, head) in one workgroup: S = Q K^T / sqrt(d), P = softmax over keys, ctx = P V, for
// sequences of at most 128 positions and heads of 64 features (the encoder configuration).  The unfused path
// writes the float32 scores to HBM, reads them back for the softmax, writes P and reads it back for the second
// product; here Q, K and V are fetched once into LDS, the scores never leave the accumulators, and P goes to HBM
// only when the backward pass will read it (it is the stash of the unit, in bfloat16, and the same bfloat16
// values feed the second product, as in the unfused path).
//
// Four waves, each owning 32 query rows from start to end: after the one barrier that publishes the tiles no wave
// waits for another.  Both products run with the MFMA operands exchanged, which puts a query's row of scores into
// two lanes (row-wise maximum and sum need one exchange) and lets the second product take P from the registers;
// P passes through LDS only on its way to HBM.
#include "gemm_dma_impl.h"

namespace spb {
namespace {
using namespace gemm_dma_detail;

constexpr int kSeqMax = 128, kHeadDim = 64;
constexpr int kQBytes = kSeqMax * kRowBytes;          // Q tile, RowK: 128 rows x 64 features
constexpr int kVBytes = 2 * kHeadDim * kRowBytes;     // V, KRow: two k tiles (64 keys each) x 64 feature rows
constexpr int kPWave = 2 * 32 * kRowBytes;            // one wave's P: two k tiles (64 keys each) x 32 query rows
constexpr int kAttnLds = 2 * kQBytes + kVBytes + 4 * kPWave;

// Rotation of the KRow dS tile (see the kernel): by 2 chunks per k-row, modulo 8 k-rows.
__device__ __forceinline__ int dsk_rot(int k) { return (k & 7) << 1; }

// One MFMA operand out of a KRow tile, like read_fragment, with two options: OWN_ROT reads a tile laid out with
// dsk_rot instead of the loader's rotation; SPLIT_K fetches, for half-wave hh, k = 16 kg + 4 hh + (0..3) and
// 16 kg + 8 + 4 hh + (0..3) instead of 16 kg + 8 hh + (0..7), the order of k of an A fragment that comes straight
// from exchanged-operand accumulators.  Valid only after fragments_ready().
template <int ROWS, bool OWN_ROT, bool SPLIT_K>
__device__ __forceinline__ u32x4 read_krow(const char* tile, int frag_row0, int kg, int lane) {
  constexpr int kRowChunks = ROWS / 8;
  const int j = lane & 15, g = lane >> 4;
  const int row = frag_row0 + 16 * (g & 1) + 4 * (j & 3);
  u32x4 out;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int k = 16 * kg + (SPLIT_K ? 4 * (g >> 1) + 8 * h : 8 * (g >> 1) + 4 * h) + (j >> 2);
    const int pc = ((row >> 3) + (OWN_ROT ? dsk_rot(k) : krow_rot<ROWS>(k))) % kRowChunks;
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_ptr_t)(tile + k * (ROWS * 2) + pc * 16 + (row & 7) * 2);
    uint2 w;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(w) : "v"(lds_addr));
    out[2 * h] = w.x;
    out[2 * h + 1] = w.y;
  }
  return out;
}

__global__ __launch_bounds__(256) void attention_fwd_kernel(const bf16_t* __restrict__ qkv, int ld_qkv, bf16_t* __restrict__ prob,
                                                            bf16_t* __restrict__ ctx, int ld_ctx, int heads, int seq, float scale) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  char* q_tile = lds;
  char* k_tile = lds + kQBytes;
  char* v_tile = lds + 2 * kQBytes;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* p_tile = lds + 2 * kQBytes + kVBytes + wave * kPWave;
  const int z = blockIdx.x, b = z / heads, h = z - b * heads;
  const int hidden = heads * kHeadDim;
  const bf16_t* base = qkv + (size_t)b * seq * ld_qkv + h * kHeadDim;
  ConvGeom none{};

  TileSource<kSeqMax, Layout::RowK, Gather::None, 4> src_q, src_k;
  TileSource<kHeadDim, Layout::KRow, Gather::None, 4> src_v;
  src_q.init(base, ld_qkv, 0, seq, wave, lane, 0, none);
  src_k.init(base + hidden, ld_qkv, 0, seq, wave, lane, 0, none);
  src_v.init(base + 2 * hidden, ld_qkv, 0, kHeadDim, wave, lane, 0, none);
  src_q.issue(0, kHeadDim, q_tile, wave, ld_qkv, none);
  src_k.issue(0, kHeadDim, k_tile, wave, ld_qkv, none);
  src_v.issue(0, seq, v_tile, wave, ld_qkv, none);
  src_v.issue(1, seq, v_tile + kHeadDim * kRowBytes, wave, ld_qkv, none);
  wait_loads_and_barrier<0>();

  // Scores of this wave's 32 queries against all keys, multiplied with the MFMA operands exchanged: lane l holds, of
  // query q0 + l % 32, the keys 32 j + 8 (r / 4) + 4 (l / 32) + r % 4 of key block j.  A row of the softmax then lies
  // in two lanes (maximum and sum are 63 in-lane operations and one exchange), four consecutive registers are four
  // consecutive keys (P parks in LDS with 8-byte writes) and eight consecutive registers are, up to the order of k,
  // an A fragment of ctx = P V, which therefore comes straight from the registers.
  const int q0 = 32 * wave, qi = lane & 31, hh = lane >> 5;
  f32x16 s[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s[j][r] = 0.f;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const u32x4 a = read_fragment<kSeqMax, Layout::RowK>(q_tile, q0, g, lane);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32x4 kb = read_fragment<kSeqMax, Layout::RowK>(k_tile, 32 * j, g, lane);
      s[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kb), __builtin_bit_cast(bf16x8, a), s[j], 0, 0, 0);
    }
  }
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[j][r] = 32 * j + 8 * (r >> 2) + 4 * hh + (r & 3) < seq ? s[j][r] * scale : -INFINITY;
      m = fmaxf(m, s[j][r]);
    }
  m = fmaxf(m, __shfl_xor(m, 32, 64));
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[j][r] = __expf(s[j][r] - m); sum += s[j][r]; }   // the hardware exponential: P is rounded to bfloat16 next
  sum += __shfl_xor(sum, 32, 64);
  const float inv = 1.f / sum;
  // P, rounded to bfloat16 and packed two keys to a word: pp[j][4 g + e] holds keys 32 j + 8 g + 4 hh + 2 e, + 1
  uint32_t pp[4][8];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) pp[j][e] = pack_bf16(s[j][2 * e] * inv, s[j][2 * e + 1] * inv);
  // ctx = P V: the A fragment of k-group g of key tile kt is pp[2 kt + g / 2][4 (g % 2) ..]; V's fragments are
  // fetched in the same order of k (see read_krow)
  f32x16 o[2];
#pragma unroll
  for (int n = 0; n < 2; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[n][r] = 0.f;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x4 a[1], vb[2];
      const int j = 2 * kt + (g >> 1), e0 = 4 * (g & 1);
      a[0] = u32x4{pp[j][e0], pp[j][e0 + 1], pp[j][e0 + 2], pp[j][e0 + 3]};
      vb[0] = read_krow<kHeadDim, false, true>(v_tile + kt * (kHeadDim * kRowBytes), 0, g, lane);
      vb[1] = read_krow<kHeadDim, false, true>(v_tile + kt * (kHeadDim * kRowBytes), 32, g, lane);
      fragments_ready(a, vb);
#pragma unroll
      for (int n = 0; n < 2; ++n)
        o[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vb[n]), __builtin_bit_cast(bf16x8, a[0]), o[n], 0, 0, 0);
    }
  }
  // P to HBM (only when it is kept): parked per wave as RowK tiles (two k tiles of 64 keys x 32 query rows) with
  // 8-byte writes, read back as 16-byte chunks so that whole rows leave; LDS operations of a wave run in order
  if (prob) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int key = 32 * j + 8 * g + 4 * hh;
        *reinterpret_cast<uint2*>(p_tile + (key >> 6) * (32 * kRowBytes) + lds_offset(qi, (key & 63) >> 3) + (key & 7) * 2) = uint2{pp[j][2 * g], pp[j][2 * g + 1]};
      }
    asm volatile("" ::: "memory");  // read back through pointers of another type
    bf16_t* dst = prob + (size_t)z * seq * seq;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int idx = it * 64 + lane, row = idx >> 4, chunk = idx & 15;   // 32 rows x 16 chunks of 8 keys
      if (q0 + row < seq && chunk * 8 < seq) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(p_tile + (chunk >> 3) * (32 * kRowBytes) + lds_offset(row, chunk & 7));
        *reinterpret_cast<u32x4*>(dst + (size_t)(q0 + row) * seq + chunk * 8) = v;
      }
    }
  }
  asm volatile("" ::: "memory");
  // ctx through the same LDS region (P is dead once its copy is read): 32 rows x 64 floats, four consecutive
  // features per 16-byte write, the 16 chunks of a row permuted by row % 16 (see the backward kernel's write_out)
  float* stage = reinterpret_cast<float*>(p_tile);
  constexpr int kPitch = kHeadDim;  // no padding: the region is exactly 32 x 64 floats
  static_assert(32 * kPitch * 4 <= kPWave, "ctx staging fits in the wave's P region");
#pragma unroll
  for (int n = 0; n < 2; ++n)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int chunk = (8 * n + 2 * g + hh) ^ (qi & 15);
      *reinterpret_cast<f32x4*>(stage + qi * kPitch + chunk * 4) = f32x4{o[n][4 * g], o[n][4 * g + 1], o[n][4 * g + 2], o[n][4 * g + 3]};
    }
  asm volatile("" ::: "memory");
  bf16_t* out = ctx + (size_t)b * seq * ld_ctx + h * kHeadDim;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = it * 8 + (lane >> 3), c = (lane & 7) * 2;
    if (q0 + row < seq) {
      float v[8];
      const f32x4 v0 = *reinterpret_cast<const f32x4*>(stage + row * kPitch + (c ^ (row & 15)) * 4);
      const f32x4 v1 = *reinterpret_cast<const f32x4*>(stage + row * kPitch + ((c + 1) ^ (row & 15)) * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[e] = v0[e]; v[4 + e] = v1[e]; }
      *reinterpret_cast<u32x4*>(out + (size_t)(q0 + row) * ld_ctx + c * 4) = pack_bf16x8(v);
    }
  }
}

// Backward of the same attention, one workgroup per (batch entry, head):
//   dP = dctx V^T;  dS = P * (dP - rowsum(dP * P)) * scale (rounded to bfloat16, as the unfused path stores it);
//   dQ = dS K;  dK = dS^T Q;  dV = P^T dctx.
// Phase 1 is row-wise: wave w forms dP and dS of its 32 queries in the accumulators (P comes straight from HBM in
// that layout) and writes dS once, into a workgroup-wide KRow tile (k = query) that dK reads; its own dQ product
// takes dS from the registers.  After one barrier, phase 2: wave w produces rows 32 w .. of dQ, dK and dV, three
// products of 16 MFMAs each, with K, Q and dctx read through transposing LDS reads and P as a KRow tile that came
// in by direct-to-LDS loads.  LDS: dctx twice (RowK for dP, KRow for dV), V (RowK), K, Q (KRow), P (KRow), the KRow dS
// tile, which takes over the space of dctx-RowK and V once dP is done, and 8 KB per wave through which results leave.
constexpr int kDsK = kSeqMax * 2 * kSeqMax;  // dS as KRow tiles: two k tiles of 64 queries x 128 key rows
constexpr int kBwdLds = kQBytes /*dctx RowK*/ + kQBytes /*V RowK*/ + 3 * kVBytes /*dctx, K, Q as KRow*/ + kDsK /*P KRow*/ + 4 * kPWave;
static_assert(2 * kQBytes == kDsK, "the KRow dS tile reuses the dctx and V tiles of phase 1");

__global__ __launch_bounds__(256) void attention_bwd_kernel(const bf16_t* __restrict__ qkv, int ld_qkv, const bf16_t* __restrict__ prob,
                                                            const bf16_t* __restrict__ dctx, int ld_ctx, bf16_t* __restrict__ dqkv,
                                                            int heads, int seq, float scale) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  char* dctx_r = lds;                           // phase 1; then, with v_r, the KRow dS tile
  char* v_r = lds + kQBytes;
  char* ds_k = lds;
  char* dctx_k = lds + 2 * kQBytes;
  char* k_k = dctx_k + kVBytes;
  char* q_k = k_k + kVBytes;
  char* p_k = q_k + kVBytes;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* out_stage = p_k + kDsK + wave * kPWave;   // this wave's 32 x 64 floats on their way out
  const int z = blockIdx.x, b = z / heads, h = z - b * heads;
  const int hidden = heads * kHeadDim;
  const bf16_t* base = qkv + (size_t)b * seq * ld_qkv + h * kHeadDim;
  const bf16_t* dc = dctx + (size_t)b * seq * ld_ctx + h * kHeadDim;
  const bf16_t* pz = prob + (size_t)z * seq * seq;
  ConvGeom none{};

  {
    TileSource<kSeqMax, Layout::RowK, Gather::None, 4> src_dc, src_v;
    TileSource<kHeadDim, Layout::KRow, Gather::None, 4> src_dck, src_k, src_q;
    TileSource<kSeqMax, Layout::KRow, Gather::None, 4> src_p;
    src_dc.init(dc, ld_ctx, 0, seq, wave, lane, 0, none);
    src_v.init(base + 2 * hidden, ld_qkv, 0, seq, wave, lane, 0, none);
    src_dck.init(dc, ld_ctx, 0, kHeadDim, wave, lane, 0, none);
    src_k.init(base + hidden, ld_qkv, 0, kHeadDim, wave, lane, 0, none);
    src_q.init(base, ld_qkv, 0, kHeadDim, wave, lane, 0, none);
    src_p.init(pz, seq, 0, seq, wave, lane, 0, none);
    src_dc.issue(0, kHeadDim, dctx_r, wave, ld_ctx, none);
    src_v.issue(0, kHeadDim, v_r, wave, ld_qkv, none);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      src_dck.issue(t, seq, dctx_k + t * (kHeadDim * kRowBytes), wave, ld_ctx, none);
      src_k.issue(t, seq, k_k + t * (kHeadDim * kRowBytes), wave, ld_qkv, none);
      src_q.issue(t, seq, q_k + t * (kHeadDim * kRowBytes), wave, ld_qkv, none);
      src_p.issue(t, seq, p_k + t * (kSeqMax * kRowBytes), wave, seq, none);
    }
  }
  // P of this wave's queries, four consecutive keys at a time, straight from HBM while the tiles are in flight.
  // Phase 1 multiplies with the MFMA operands exchanged, so lane l holds, of query q0 + l % 32, the keys
  // 32 j + 8 (r / 4) + 4 (l / 32) + r % 4 of key block j: a query's row lies in two lanes (one exchange for the row
  // sum instead of a shuffle tree per register), four consecutive registers are four consecutive keys (8-byte loads
  // of P, 8-byte LDS writes of dS), and eight consecutive registers are, up to the order of k, an A fragment of
  // dQ = dS K, which therefore never goes through LDS.
  const int q0 = 32 * wave, qi = lane & 31, hh = lane >> 5, q = q0 + qi;
  // Requested as 16-byte pieces (keys 8 c .. 8 c + 7), the lower half-wave the even c and the upper the odd ones;
  // two v_permlane32_swap per pair of pieces then hand each lane its half of both.
  u32x4 praw[8];
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const int key = 8 * (2 * m + hh);
    praw[m] = (q < seq && key < seq) ? *reinterpret_cast<const u32x4*>(pz + (size_t)q * seq + key) : u32x4{0u, 0u, 0u, 0u};
  }
  wait_loads_and_barrier<0>();
  uint2 pw[4][4];   // pw[j][g]: keys 32 j + 8 g + 4 hh + (0..3)
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const auto x = __builtin_amdgcn_permlane32_swap(praw[m][0], praw[m][2], false, false);
    const auto y = __builtin_amdgcn_permlane32_swap(praw[m][1], praw[m][3], false, false);
    pw[m >> 1][2 * (m & 1)] = uint2{x[0], y[0]};
    pw[m >> 1][2 * (m & 1) + 1] = uint2{x[1], y[1]};
  }

  // phase 1: dP = dctx V^T for this wave's queries
  f32x16 dp[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) dp[j][r] = 0.f;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const u32x4 a = read_fragment<kSeqMax, Layout::RowK>(dctx_r, q0, g, lane);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32x4 vb = read_fragment<kSeqMax, Layout::RowK>(v_r, 32 * j, g, lane);
      dp[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vb), __builtin_bit_cast(bf16x8, a), dp[j], 0, 0, 0);
    }
  }
  // dS, rounded to bfloat16 and packed two keys to a word: ds[j][4 g + e] holds keys 32 j + 8 g + 4 hh + 2 e, + 1
  uint32_t ds[4][8];
  {
    float pv[4][16];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        pv[j][4 * g] = __uint_as_float(pw[j][g].x << 16); pv[j][4 * g + 1] = __uint_as_float(pw[j][g].x & 0xFFFF0000u);
        pv[j][4 * g + 2] = __uint_as_float(pw[j][g].y << 16); pv[j][4 * g + 3] = __uint_as_float(pw[j][g].y & 0xFFFF0000u);
      }
    float dot = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) dot += dp[j][r] * pv[j][r];
    dot += __shfl_xor(dot, 32, 64);   // the other half of the row
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        ds[j][e] = pack_bf16(pv[j][2 * e] * (dp[j][2 * e] - dot) * scale, pv[j][2 * e + 1] * (dp[j][2 * e + 1] - dot) * scale);
  }
  __syncthreads();  // all waves have read dctx_r and v_r: their space becomes the KRow dS tile
  // dS as KRow tiles (k = query, rows = keys) for dK = dS^T Q: two k tiles of 64 queries, 128 key rows of 2 bytes per
  // k-row, the 16-byte chunks of k-row kk rotated by 2 (kk % 8), which keeps these 8-byte writes (32 k-rows at once)
  // and the transposing reads below (4 k-rows at once) off each other's banks.
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int key = 32 * j + 8 * g + 4 * hh, kk = q & 63;
      const int pc = ((key >> 3) + dsk_rot(kk)) & (kSeqMax / 8 - 1);
      *reinterpret_cast<uint2*>(ds_k + (q >> 6) * (kSeqMax * kRowBytes) + kk * (kSeqMax * 2) + pc * 16 + (key & 7) * 2) = uint2{ds[j][2 * g], ds[j][2 * g + 1]};
    }
  __syncthreads();

  // phase 2: three [32 x 64] outputs per wave, multiplied with the operands exchanged so that four consecutive
  // accumulators are four consecutive features of one row: a result parks in the wave's staging rows with 16-byte
  // writes (the 16 chunks of a 256-byte row permuted by row % 16, which keeps both the writes, 32 rows at once, and
  // the row-wise reads off each other's banks) and leaves as whole 128-byte rows.
  float* stage = reinterpret_cast<float*>(out_stage);
  constexpr int kPitch = kHeadDim;
  auto write_out = [&](f32x16 (&o)[2], int col_block) {
    asm volatile("" ::: "memory");
    const int prow = lane & 31;
#pragma unroll
    for (int n = 0; n < 2; ++n)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int chunk = (8 * n + 2 * g + hh) ^ (prow & 15);
        *reinterpret_cast<f32x4*>(stage + prow * kPitch + chunk * 4) = f32x4{o[n][4 * g], o[n][4 * g + 1], o[n][4 * g + 2], o[n][4 * g + 3]};
      }
    asm volatile("" ::: "memory");
    bf16_t* out = dqkv + (size_t)b * seq * ld_qkv + col_block * hidden + h * kHeadDim;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = it * 8 + (lane >> 3), c = (lane & 7) * 2;
      if (q0 + row < seq) {
        float v[8];
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(stage + row * kPitch + (c ^ (row & 15)) * 4);
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(stage + row * kPitch + ((c + 1) ^ (row & 15)) * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = v0[e]; v[4 + e] = v1[e]; }
        *reinterpret_cast<u32x4*>(out + (size_t)(q0 + row) * ld_qkv + c * 4) = pack_bf16x8(v);
      }
    }
    asm volatile("" ::: "memory");
  };
  auto zero = [](f32x16 (&o)[2]) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[j][r] = 0.f;
  };
  f32x16 acc[2];
  // dQ[q, d] = sum_key dS[q, key] K[key, d]: the A fragment of k-group g of key tile kt is ds[2 kt + g / 2][4 (g % 2) ..],
  // whose two half-waves hold keys 16 g + 4 hh + (0..3) and 16 g + 8 + 4 hh + (0..3); K's fragments are fetched in the
  // same order of k.
  zero(acc);
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x4 a[1], bb[2];
      const int j = 2 * kt + (g >> 1), e0 = 4 * (g & 1);
      a[0] = u32x4{ds[j][e0], ds[j][e0 + 1], ds[j][e0 + 2], ds[j][e0 + 3]};
      bb[0] = read_krow<kHeadDim, false, true>(k_k + kt * (kHeadDim * kRowBytes), 0, g, lane);
      bb[1] = read_krow<kHeadDim, false, true>(k_k + kt * (kHeadDim * kRowBytes), 32, g, lane);
      fragments_ready(a, bb);
#pragma unroll
      for (int n = 0; n < 2; ++n)
        acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bb[n]), __builtin_bit_cast(bf16x8, a[0]), acc[n], 0, 0, 0);
    }
  write_out(acc, 0);
  // dK[key, d] = sum_q dS[q, key] Q[q, d]   and   dV[key, d] = sum_q P[q, key] dctx[q, d]: rows = this wave's 32 keys
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const char* a_tile = which == 0 ? ds_k : p_k;
    const char* b_tile = which == 0 ? q_k : dctx_k;
    zero(acc);
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x4 a[1], bb[2];
        a[0] = which == 0 ? read_krow<kSeqMax, true, false>(a_tile + kt * (kSeqMax * kRowBytes), q0, g, lane)
                          : read_fragment<kSeqMax, Layout::KRow>(a_tile + kt * (kSeqMax * kRowBytes), q0, g, lane);
        bb[0] = read_fragment<kHeadDim, Layout::KRow>(b_tile + kt * (kHeadDim * kRowBytes), 0, g, lane);
        bb[1] = read_fragment<kHeadDim, Layout::KRow>(b_tile + kt * (kHeadDim * kRowBytes), 32, g, lane);
        fragments_ready(a, bb);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bb[j]), __builtin_bit_cast(bf16x8, a[0]), acc[j], 0, 0, 0);
      }
    write_out(acc, 1 + which);
  }
}

}  // namespace

bool attention_fused_accepts(int seq, int head_dim, int ld_qkv, int ld_ctx) {
  return head_dim == kHeadDim && seq >= 1 && seq <= kSeqMax && seq % 8 == 0 && ld_qkv % 8 == 0 && ld_ctx % 8 == 0;
}

hipError_t launch_attention_fwd(const void* qkv, int ld_qkv, void* prob, void* ctx, int ld_ctx, int batch, int heads, int seq,
                                int head_dim, float scale, hipStream_t stream) {
  if (!qkv || !ctx || batch <= 0 || heads <= 0 || !attention_fused_accepts(seq, head_dim, ld_qkv, ld_ctx)) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(ctx) | reinterpret_cast<uintptr_t>(prob)) & 15) return hipErrorInvalidValue;
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(attention_fwd_kernel), (size_t)kAttnLds); e != hipSuccess) return e;
  hipLaunchKernelGGL(attention_fwd_kernel, dim3(batch * heads), dim3(256), kAttnLds, stream, static_cast<const bf16_t*>(qkv), ld_qkv,
                     static_cast<bf16_t*>(prob), static_cast<bf16_t*>(ctx), ld_ctx, heads, seq, scale);
  return hipGetLastError();
}

hipError_t launch_attention_bwd(const void* qkv, int ld_qkv, const void* prob, const void* dctx, int ld_ctx, void* dqkv, int batch,
                                int heads, int seq, int head_dim, float scale, hipStream_t stream) {
  if (!qkv || !prob || !dctx || !dqkv || batch <= 0 || heads <= 0 || !attention_fused_accepts(seq, head_dim, ld_qkv, ld_ctx)) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(prob) | reinterpret_cast<uintptr_t>(dctx) | reinterpret_cast<uintptr_t>(dqkv)) & 15)
    return hipErrorInvalidValue;
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(attention_bwd_kernel), (size_t)kBwdLds); e != hipSuccess) return e;
  hipLaunchKernelGGL(attention_bwd_kernel, dim3(batch * heads), dim3(256), kBwdLds, stream, static_cast<const bf16_t*>(qkv), ld_qkv,
                     static_cast<const bf16_t*>(prob), static_cast<const bf16_t*>(dctx), ld_ctx, static_cast<bf16_t*>(dqkv), heads, seq, scale);
  return hipGetLastError();
}

}  // namespace spb
