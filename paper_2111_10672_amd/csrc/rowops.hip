// Row-wise, memory-bound kernels of the Transformer-encoder units: LayerNorm forward and backward, the
// softmax of attention and its backward, embedding lookup and its gradient.  Each row is handled by one
// wavefront (64 lanes), values move as 16-byte chunks of 8 bfloat16, reductions use wavefront shuffles.
// Reductions over rows (LayerNorm scale/shift gradients) are done in two fixed-order stages so that a
// step gives the same bits on every run.
#include "kernels.h"

namespace spb {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxChunks = 4;  // 16-byte chunks per lane: rows of up to 64 * 4 * 8 = 2048 elements
constexpr float kLnEps = 1e-5f;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ void unpack8(const u32x4& w, float (&f)[8]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) { f[2 * d] = __uint_as_float(w[d] << 16); f[2 * d + 1] = __uint_as_float(w[d] & 0xFFFF0000u); }
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) { return bf16_pack2(lo, hi); }
__device__ __forceinline__ u32x4 pack8(const float (&f)[8]) {
  u32x4 o;
#pragma unroll
  for (int d = 0; d < 4; ++d) o[d] = pack2(f[2 * d], f[2 * d + 1]);
  return o;
}
__device__ __forceinline__ uint16_t to_bf16(float v) { return bf16_round(v); }

// y[r] = gamma * (x[src(r)] - mean) * rstd + beta;  stats[r] = (mean, rstd).  src(r) = rows ? rows[r] : r.
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const uint16_t* __restrict__ x, int ldx, const int32_t* __restrict__ rows,
                                                            int n_rows, int width, const uint16_t* __restrict__ gamma,
                                                            const uint16_t* __restrict__ beta, uint16_t* __restrict__ y, int ldy,
                                                            float* __restrict__ stats) {
  const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  const int chunks = width >> 3;
  const uint16_t* src = x + (size_t)(rows ? rows[r] : r) * ldx;
  float v[kMaxChunks][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxChunks; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
      unpack8(*reinterpret_cast<const u32x4*>(src + c * 8), v[i]);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += v[i][e];
    }
  }
  const float mean = wave_sum(sum) / (float)width;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxChunks; ++i)
    if (lane + 64 * i < chunks) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; sq += d * d; }
    }
  const float rstd = rsqrtf(wave_sum(sq) / (float)width + kLnEps);
#pragma unroll
  for (int i = 0; i < kMaxChunks; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
      float g[8], b[8], o[8];
      unpack8(*reinterpret_cast<const u32x4*>(gamma + c * 8), g);
      unpack8(*reinterpret_cast<const u32x4*>(beta + c * 8), b);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = g[e] * ((v[i][e] - mean) * rstd) + b[e];
      *reinterpret_cast<u32x4*>(y + (size_t)r * ldy + c * 8) = pack8(o);
    }
  }
  if (lane == 0) { stats[2 * r] = mean; stats[2 * r + 1] = rstd; }
}

// The same forward pass for the widths that split evenly over lanes (LPR lanes per row, CPL 16-byte chunks per
// lane): a wavefront takes 64 / LPR rows at once, every lane is busy, and scale and shift are requested together
// with the row, not after the two reductions.
template <int LPR, int CPL>
__global__ __launch_bounds__(256) void layernorm_fwd_even_kernel(const uint16_t* __restrict__ x, int ldx, const int32_t* __restrict__ rows,
                                                                 int n_rows, const uint16_t* __restrict__ gamma,
                                                                 const uint16_t* __restrict__ beta, uint16_t* __restrict__ y, int ldy,
                                                                 float* __restrict__ stats) {
  constexpr int RPW = 64 / LPR, kWidth = LPR * CPL * 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPR, l = lane % LPR;
  const int r = (blockIdx.x * 4 + wave) * RPW + sub;
  const bool live = r < n_rows;
  const int rc = live ? r : n_rows - 1;
  const uint16_t* src = x + (size_t)(rows ? rows[rc] : rc) * ldx;
  u32x4 xraw[CPL], graw[CPL], braw[CPL];
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int c = (l + LPR * i) * 8;
    xraw[i] = *reinterpret_cast<const u32x4*>(src + c);
    graw[i] = *reinterpret_cast<const u32x4*>(gamma + c);
    braw[i] = *reinterpret_cast<const u32x4*>(beta + c);
  }
  float v[CPL][8];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    unpack8(xraw[i], v[i]);
#pragma unroll
    for (int e = 0; e < 8; ++e) sum += v[i][e];
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
  const float mean = sum / (float)kWidth;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < CPL; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; sq += d * d; }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
  const float rstd = rsqrtf(sq / (float)kWidth + kLnEps);
  if (!live) return;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    float g[8], b[8], o[8];
    unpack8(graw[i], g);
    unpack8(braw[i], b);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = g[e] * ((v[i][e] - mean) * rstd) + b[e];
    *reinterpret_cast<u32x4*>(y + (size_t)r * ldy + (l + LPR * i) * 8) = pack8(o);
  }
  if (l == 0) { stats[2 * r] = mean; stats[2 * r + 1] = rstd; }
}

// LayerNorm backward for rows r0 .. r0+7 of this workgroup (2 per wavefront, so that the row loop is short and
// a matrix of a few thousand rows still fills the chip):
//   g = dy * gamma;  dx = (g - mean(g) - xhat * mean(g * xhat)) * rstd (+ res);  partial sums of dy * xhat and dy per column.
constexpr int kLnRowsPerBlock = 8;
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const uint16_t* __restrict__ dy, int lddy, const uint16_t* __restrict__ x,
                                                            int ldx, const int32_t* __restrict__ rows, const float* __restrict__ stats,
                                                            const uint16_t* __restrict__ gamma, const uint16_t* __restrict__ res, int ldres,
                                                            uint16_t* __restrict__ dx, int lddx, float* __restrict__ partial,
                                                            int n_rows, int width) {
  extern __shared__ float sh[];  // [4 wavefronts][2][width]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunks = width >> 3;
  float dgam[kMaxChunks][8], dbet[kMaxChunks][8], gam[kMaxChunks][8];
#pragma unroll
  for (int i = 0; i < kMaxChunks; ++i) {
#pragma unroll
    for (int e = 0; e < 8; ++e) { dgam[i][e] = 0.f; dbet[i][e] = 0.f; gam[i][e] = 0.f; }
    if (lane + 64 * i < chunks) unpack8(*reinterpret_cast<const u32x4*>(gamma + (lane + 64 * i) * 8), gam[i]);
  }
  for (int j = 0; j < kLnRowsPerBlock / 4; ++j) {
    const int r = blockIdx.x * kLnRowsPerBlock + wave * (kLnRowsPerBlock / 4) + j;
    if (r >= n_rows) break;
    const size_t xr = rows ? rows[r] : r;
    const float mean = stats[2 * r], rstd = stats[2 * r + 1];
    float g[kMaxChunks][8], xh[kMaxChunks][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxChunks; ++i) {
      const int c = lane + 64 * i;
      if (c < chunks) {
        float d[8], xv[8];
        unpack8(*reinterpret_cast<const u32x4*>(dy + (size_t)r * lddy + c * 8), d);
        unpack8(*reinterpret_cast<const u32x4*>(x + xr * ldx + c * 8), xv);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          xh[i][e] = (xv[e] - mean) * rstd;
          g[i][e] = d[e] * gam[i][e];
          s1 += g[i][e];
          s2 += g[i][e] * xh[i][e];
          dgam[i][e] += d[e] * xh[i][e];
          dbet[i][e] += d[e];
        }
      }
    }
    if (dx) {
      const float m1 = wave_sum(s1) / (float)width, m2 = wave_sum(s2) / (float)width;
#pragma unroll
      for (int i = 0; i < kMaxChunks; ++i) {
        const int c = lane + 64 * i;
        if (c < chunks) {
          float o[8], rv[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) rv[e] = 0.f;
          if (res) unpack8(*reinterpret_cast<const u32x4*>(res + (size_t)r * ldres + c * 8), rv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (g[i][e] - m1 - xh[i][e] * m2) * rstd + rv[e];
          *reinterpret_cast<u32x4*>(dx + xr * lddx + c * 8) = pack8(o);
        }
      }
    }
  }
  // add the four wavefronts' column sums in wavefront order
  float* mine = sh + (size_t)wave * 2 * width;
#pragma unroll
  for (int i = 0; i < kMaxChunks; ++i) {
    const int c = lane + 64 * i;
    if (c < chunks) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { mine[c * 8 + e] = dgam[i][e]; mine[width + c * 8 + e] = dbet[i][e]; }
    }
  }
  __syncthreads();
  for (int col = threadIdx.x; col < 2 * width; col += 256)
    partial[(size_t)blockIdx.x * 2 * width + col] = ((sh[col] + sh[2 * width + col]) + sh[4 * width + col]) + sh[6 * width + col];
}

// The same backward pass for the widths that split evenly over lanes: a row is held by LPR lanes with CPL
// 16-byte chunks each (width = LPR * CPL * 8), a wavefront works on 64 / LPR rows at a time and takes ITERS such
// groups.  Everything the wavefront will read (scale, statistics, all its rows) is requested before the first
// value is used, so the kernel pays one memory latency, not one per row.  Workgroup b handles rows
// b * kRows .. b * kRows + kRows - 1 and writes one partial column sum (the same layout as above).
template <int LPR, int CPL, int ITERS>
__global__ __launch_bounds__(256) void layernorm_bwd_even_kernel(const uint16_t* __restrict__ dy, int lddy, const uint16_t* __restrict__ x,
                                                                 int ldx, const int32_t* __restrict__ rows, const float* __restrict__ stats,
                                                                 const uint16_t* __restrict__ gamma, const uint16_t* __restrict__ res, int ldres,
                                                                 uint16_t* __restrict__ dx, int lddx, float* __restrict__ partial, int n_rows) {
  constexpr int RPW = 64 / LPR, kRows = 4 * RPW * ITERS, kWidth = LPR * CPL * 8;
  extern __shared__ float sh[];  // [4 * RPW row groups][2][kWidth]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane / LPR, l = lane % LPR;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  u32x4 graw[CPL], dyraw[ITERS][CPL], xraw[ITERS][CPL], rraw[ITERS][CPL];
  float mean[ITERS], rstd[ITERS];
  size_t xrow[ITERS];
  bool live[ITERS];
#pragma unroll
  for (int i = 0; i < CPL; ++i) graw[i] = *reinterpret_cast<const u32x4*>(gamma + (l + LPR * i) * 8);
#pragma unroll
  for (int j = 0; j < ITERS; ++j) {
    const int r = blockIdx.x * kRows + (j * 4 + wave) * RPW + sub;
    live[j] = r < n_rows;
    const int rc = live[j] ? r : n_rows - 1;
    xrow[j] = rows ? rows[rc] : rc;
    mean[j] = stats[2 * rc];
    rstd[j] = stats[2 * rc + 1];
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = (l + LPR * i) * 8;
      dyraw[j][i] = live[j] ? *reinterpret_cast<const u32x4*>(dy + (size_t)rc * lddy + c) : zero;
      xraw[j][i] = *reinterpret_cast<const u32x4*>(x + xrow[j] * ldx + c);
      rraw[j][i] = res && live[j] ? *reinterpret_cast<const u32x4*>(res + (size_t)rc * ldres + c) : zero;
    }
  }
  float dgam[CPL][8], dbet[CPL][8];
#pragma unroll
  for (int i = 0; i < CPL; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) { dgam[i][e] = 0.f; dbet[i][e] = 0.f; }
#pragma unroll
  for (int j = 0; j < ITERS; ++j) {
    float g[CPL][8], xh[CPL][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      float d[8], xv[8], gm[8];
      unpack8(dyraw[j][i], d);
      unpack8(xraw[j][i], xv);
      unpack8(graw[i], gm);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        xh[i][e] = (xv[e] - mean[j]) * rstd[j];
        g[i][e] = d[e] * gm[e];
        s1 += g[i][e];
        s2 += g[i][e] * xh[i][e];
        dgam[i][e] += d[e] * xh[i][e];   // a row past the end has d = 0
        dbet[i][e] += d[e];
      }
    }
    if (dx) {
#pragma unroll
      for (int o = LPR / 2; o > 0; o >>= 1) { s1 += __shfl_xor(s1, o, 64); s2 += __shfl_xor(s2, o, 64); }
      const float m1 = s1 / (float)kWidth, m2 = s2 / (float)kWidth;
      if (live[j]) {
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
          float o[8], rv[8];
          unpack8(rraw[j][i], rv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (g[i][e] - m1 - xh[i][e] * m2) * rstd[j] + rv[e];
          *reinterpret_cast<u32x4*>(dx + xrow[j] * lddx + (l + LPR * i) * 8) = pack8(o);
        }
      }
    }
  }
  // add the 4 * RPW row groups' column sums in group order
  float* mine = sh + (size_t)(wave * RPW + sub) * 2 * kWidth;
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int c = (l + LPR * i) * 8;
    *reinterpret_cast<f32x4*>(mine + c) = f32x4{dgam[i][0], dgam[i][1], dgam[i][2], dgam[i][3]};
    *reinterpret_cast<f32x4*>(mine + c + 4) = f32x4{dgam[i][4], dgam[i][5], dgam[i][6], dgam[i][7]};
    *reinterpret_cast<f32x4*>(mine + kWidth + c) = f32x4{dbet[i][0], dbet[i][1], dbet[i][2], dbet[i][3]};
    *reinterpret_cast<f32x4*>(mine + kWidth + c + 4) = f32x4{dbet[i][4], dbet[i][5], dbet[i][6], dbet[i][7]};
  }
  __syncthreads();
  for (int col = threadIdx.x; col < 2 * kWidth; col += 256) {
    float t = sh[col];
#pragma unroll
    for (int q = 1; q < 4 * RPW; ++q) t += sh[(size_t)q * 2 * kWidth + col];
    partial[(size_t)blockIdx.x * 2 * kWidth + col] = t;
  }
}

// out_a[c] = sum_b partial[b][0][c];  out_b[c] = sum_b partial[b][1][c].  A workgroup takes 16 columns: thread
// (g, c) adds blocks g, g + 16, ... of column c in order (16 neighbouring threads read 64 contiguous bytes), then
// the 16 group sums of a column are added in group order: the same bits on every run.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int n_blocks, int width,
                                                              float* __restrict__ out_a, float* __restrict__ out_b) {
  __shared__ float sh[16][17];
  const int c = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int col = blockIdx.x * 16 + c;
  float s = 0.f;
  if (col < 2 * width) {
#pragma unroll 8
    for (int b = g; b < n_blocks; b += 16) s += partial[(size_t)b * 2 * width + col];
  }
  sh[g][c] = s;
  __syncthreads();
  if (threadIdx.x < 16 && col < 2 * width) {
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) t += sh[q][c];
    if (col < width) out_a[col] = t;
    else out_b[col - width] = t;
  }
}

// p[r, :] = softmax(s[r, :]) in bfloat16; one wavefront per row.  A row of up to 64 * kSoftmaxRegs scores is read
// once and kept in registers (attention rows are a few hundred long); longer rows are re-read from cache.
constexpr int kSoftmaxRegs = 8;
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const float* __restrict__ s, uint16_t* __restrict__ p, long long n_rows, int len) {
  const int lane = threadIdx.x & 63;
  const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  const float* in = s + r * len;
  if (len <= 64 * kSoftmaxRegs) {
    float v[kSoftmaxRegs];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < kSoftmaxRegs; ++i) {
      const int c = lane + 64 * i;
      v[i] = c < len ? in[c] : -INFINITY;
      m = fmaxf(m, v[i]);
    }
    m = wave_max(m);
    float z = 0.f;
#pragma unroll
    for (int i = 0; i < kSoftmaxRegs; ++i) { v[i] = lane + 64 * i < len ? expf(v[i] - m) : 0.f; z += v[i]; }
    const float inv = 1.f / wave_sum(z);
#pragma unroll
    for (int i = 0; i < kSoftmaxRegs; ++i)
      if (lane + 64 * i < len) p[r * len + lane + 64 * i] = to_bf16(v[i] * inv);
    return;
  }
  float m = -INFINITY;
  for (int c = lane; c < len; c += 64) m = fmaxf(m, in[c]);
  m = wave_max(m);
  float z = 0.f;
  for (int c = lane; c < len; c += 64) z += expf(in[c] - m);
  const float inv = 1.f / wave_sum(z);
  for (int c = lane; c < len; c += 64) p[r * len + c] = to_bf16(expf(in[c] - m) * inv);
}

// ds[r, :] = p * (dp - sum(dp * p)) * scale in bfloat16; one wavefront per row, same register scheme.
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const float* __restrict__ dp, const uint16_t* __restrict__ p,
                                                          uint16_t* __restrict__ ds, long long n_rows, int len, float scale) {
  const int lane = threadIdx.x & 63;
  const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  if (len <= 64 * kSoftmaxRegs) {
    float d[kSoftmaxRegs], pv[kSoftmaxRegs];
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < kSoftmaxRegs; ++i) {
      const int c = lane + 64 * i;
      d[i] = c < len ? dp[r * len + c] : 0.f;
      pv[i] = c < len ? __uint_as_float(((uint32_t)p[r * len + c]) << 16) : 0.f;
      dot += d[i] * pv[i];
    }
    dot = wave_sum(dot);
#pragma unroll
    for (int i = 0; i < kSoftmaxRegs; ++i)
      if (lane + 64 * i < len) ds[r * len + lane + 64 * i] = to_bf16(pv[i] * (d[i] - dot) * scale);
    return;
  }
  float dot = 0.f;
  for (int c = lane; c < len; c += 64) dot += dp[r * len + c] * __uint_as_float(((uint32_t)p[r * len + c]) << 16);
  dot = wave_sum(dot);
  for (int c = lane; c < len; c += 64) {
    const float pv = __uint_as_float(((uint32_t)p[r * len + c]) << 16);
    ds[r * len + c] = to_bf16(pv * (dp[r * len + c] - dot) * scale);
  }
}
// x0[m, :] = tok[ids[m], :] + pos[m % seq, :].  An id outside [0, vocab) is clamped into range.
__global__ __launch_bounds__(256) void embedding_fwd_kernel(const int32_t* __restrict__ ids, const uint16_t* __restrict__ tok,
                                                            const uint16_t* __restrict__ pos, uint16_t* __restrict__ out, int ldo,
                                                            int n_rows, int seq, int vocab, int width) {
  const int lane = threadIdx.x & 63, m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= n_rows) return;
  const int id = min(max(ids[m], 0), vocab - 1);
  const uint16_t* t = tok + (size_t)id * width;
  const uint16_t* q = pos + (size_t)(m % seq) * width;
  for (int c = lane; c < (width >> 3); c += 64) {
    float a[8], b[8];
    unpack8(*reinterpret_cast<const u32x4*>(t + c * 8), a);
    unpack8(*reinterpret_cast<const u32x4*>(q + c * 8), b);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] += b[e];
    *reinterpret_cast<u32x4*>(out + (size_t)m * ldo + c * 8) = pack8(a);
  }
}

// Token-table gradient without atomics: the workgroup of position m does nothing unless m is the first
// position with its token id; then it adds the rows of every position with that id, in position order.
__global__ __launch_bounds__(256) void embedding_bwd_tok_kernel(const int32_t* __restrict__ ids, const uint16_t* __restrict__ dx, int lddx,
                                                                float* __restrict__ dtok, int n_rows, int vocab, int width) {
  __shared__ int flags[256];
  __shared__ int earlier;
  const int m = blockIdx.x, tid = threadIdx.x;
  const int id = min(max(ids[m], 0), vocab - 1);
  if (tid == 0) earlier = 0;
  __syncthreads();
  int found = 0;
  for (int j = tid; j < m; j += 256) found |= (min(max(ids[j], 0), vocab - 1) == id);
  if (found) earlier = 1;  // benign race: every writer stores 1
  __syncthreads();
  if (earlier) return;
  constexpr int kCols = 8;  // columns per thread: width <= 2048
  float acc[kCols];
#pragma unroll
  for (int i = 0; i < kCols; ++i) acc[i] = 0.f;
  for (int base = m - (m % 256); base < n_rows; base += 256) {
    const int j = base + tid;
    flags[tid] = j >= m && j < n_rows && min(max(ids[j], 0), vocab - 1) == id;
    __syncthreads();
    for (int t = 0; t < 256; ++t) {
      if (!flags[t]) continue;  // uniform across the workgroup
#pragma unroll
      for (int i = 0; i < kCols; ++i) {
        const int c = tid + 256 * i;
        if (c < width) acc[i] += __uint_as_float(((uint32_t)dx[(size_t)(base + t) * lddx + c]) << 16);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < kCols; ++i) {
    const int c = tid + 256 * i;
    if (c < width) dtok[(size_t)id * width + c] = acc[i];
  }
}

// dpos[s, :] = sum over the batch of dx[b * seq + s, :], batch entries added in order.
__global__ __launch_bounds__(256) void embedding_bwd_pos_kernel(const uint16_t* __restrict__ dx, int lddx, float* __restrict__ dpos,
                                                                int batch, int seq, int width) {
  const int s = blockIdx.x;
  for (int c = threadIdx.x; c < width; c += 256) {
    float acc = 0.f;
    for (int b = 0; b < batch; ++b) acc += __uint_as_float(((uint32_t)dx[(size_t)(b * seq + s) * lddx + c]) << 16);
    dpos[(size_t)s * width + c] = acc;
  }
}

bool row_ok(int width, int ld) { return width > 0 && width % 8 == 0 && width <= 64 * kMaxChunks * 8 && ld >= width && ld % 8 == 0; }
bool a16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

size_t layernorm_partial_floats(int n_rows, int width) {
  return (size_t)((n_rows + kLnRowsPerBlock - 1) / kLnRowsPerBlock) * 2 * width;
}

hipError_t launch_layernorm_fwd(const void* x, int ldx, const int32_t* rows, int n_rows, int width, const void* gamma, const void* beta,
                                void* y, int ldy, float* stats, hipStream_t s) {
  if (!x || !gamma || !beta || !y || !stats || n_rows <= 0 || !row_ok(width, ldx) || !row_ok(width, ldy)) return hipErrorInvalidValue;
  if (!a16(x) || !a16(y) || !a16(gamma) || !a16(beta)) return hipErrorInvalidValue;
  auto even = [&](auto kernel, int lpr) {
    const int rows_per_block = 4 * (64 / lpr);
    hipLaunchKernelGGL(kernel, dim3((n_rows + rows_per_block - 1) / rows_per_block), dim3(256), 0, s, (const uint16_t*)x, ldx, rows, n_rows,
                       (const uint16_t*)gamma, (const uint16_t*)beta, (uint16_t*)y, ldy, stats);
  };
  const int chunks = width / 8;
  if (chunks == 96) even(layernorm_fwd_even_kernel<32, 3>, 32);
  else if (chunks == 64) even(layernorm_fwd_even_kernel<64, 1>, 64);
  else if (chunks == 128) even(layernorm_fwd_even_kernel<64, 2>, 64);
  else if (chunks == 16) even(layernorm_fwd_even_kernel<16, 1>, 16);
  else if (chunks == 8) even(layernorm_fwd_even_kernel<8, 1>, 8);
  else
    hipLaunchKernelGGL(layernorm_fwd_kernel, dim3((n_rows + 3) / 4), dim3(256), 0, s, (const uint16_t*)x, ldx, rows, n_rows, width,
                       (const uint16_t*)gamma, (const uint16_t*)beta, (uint16_t*)y, ldy, stats);
  return hipGetLastError();
}

hipError_t launch_layernorm_bwd(const void* dy, int lddy, const void* x, int ldx, const int32_t* rows, const float* stats,
                                const void* gamma, const void* res, int ldres, void* dx, int lddx, float* partial,
                                float* dgamma, float* dbeta, int n_rows, int width, hipStream_t s, ReduceTask* deferred) {
  if (!dy || !x || !stats || !gamma || !partial || !dgamma || !dbeta || n_rows <= 0) return hipErrorInvalidValue;
  if (!row_ok(width, lddy) || !row_ok(width, ldx) || (dx && !row_ok(width, lddx)) || (res && !row_ok(width, ldres))) return hipErrorInvalidValue;
  if (!a16(dy) || !a16(x) || !a16(gamma) || !a16(dx) || !a16(res)) return hipErrorInvalidValue;
  int blocks = 0;
  auto even = [&](auto kernel, int lpr, int iters) {
    const int rows_per_block = 4 * (64 / lpr) * iters;
    blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), (size_t)4 * (64 / lpr) * 2 * width * sizeof(float), s, (const uint16_t*)dy, lddy,
                       (const uint16_t*)x, ldx, rows, stats, (const uint16_t*)gamma, (const uint16_t*)res, ldres, (uint16_t*)dx, lddx,
                       partial, n_rows);
  };
  // every variant gives a workgroup at least kLnRowsPerBlock rows, so the partial sums fit the buffer sized above
  const int chunks = width / 8;
  if (chunks == 96) even(layernorm_bwd_even_kernel<32, 3, 2>, 32, 2);
  else if (chunks == 64) even(layernorm_bwd_even_kernel<64, 1, 4>, 64, 4);
  else if (chunks == 128) even(layernorm_bwd_even_kernel<64, 2, 4>, 64, 4);
  else if (chunks == 16) even(layernorm_bwd_even_kernel<16, 1, 1>, 16, 1);
  else if (chunks == 8) even(layernorm_bwd_even_kernel<8, 1, 1>, 8, 1);
  else {
    blocks = (n_rows + kLnRowsPerBlock - 1) / kLnRowsPerBlock;
    hipLaunchKernelGGL(layernorm_bwd_kernel, dim3(blocks), dim3(256), (size_t)8 * width * sizeof(float), s, (const uint16_t*)dy, lddy,
                       (const uint16_t*)x, ldx, rows, stats, (const uint16_t*)gamma, (const uint16_t*)res, ldres, (uint16_t*)dx, lddx,
                       partial, n_rows, width);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (deferred) {   // the caller adds the column sums up later, several layers' in one launch
    deferred->kind = ReduceTask::kPairs; deferred->partial = partial; deferred->count = blocks; deferred->width = width;
    deferred->out = dgamma; deferred->out_b = dbeta; deferred->blocks = reduce_pairs_blocks(width);
    return hipSuccess;
  }
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((2 * width + 15) / 16), dim3(256), 0, s, partial, blocks, width, dgamma, dbeta);
  return hipGetLastError();
}

hipError_t launch_softmax_fwd(const float* scores, void* prob, long long n_rows, int len, hipStream_t s) {
  if (!scores || !prob || n_rows <= 0 || len <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(softmax_fwd_kernel, dim3((unsigned)((n_rows + 3) / 4)), dim3(256), 0, s, scores, (uint16_t*)prob, n_rows, len);
  return hipGetLastError();
}

hipError_t launch_softmax_bwd(const float* dprob, const void* prob, void* dscore, long long n_rows, int len, float scale, hipStream_t s) {
  if (!dprob || !prob || !dscore || n_rows <= 0 || len <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(softmax_bwd_kernel, dim3((unsigned)((n_rows + 3) / 4)), dim3(256), 0, s, dprob, (const uint16_t*)prob, (uint16_t*)dscore,
                     n_rows, len, scale);
  return hipGetLastError();
}

hipError_t launch_embedding_fwd(const int32_t* ids, const void* tok, const void* pos, void* out, int ldo, int n_rows, int seq, int vocab,
                                int width, hipStream_t s) {
  if (!ids || !tok || !pos || !out || n_rows <= 0 || seq <= 0 || vocab <= 0 || !row_ok(width, ldo) || !a16(tok) || !a16(pos) || !a16(out))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(embedding_fwd_kernel, dim3((n_rows + 3) / 4), dim3(256), 0, s, ids, (const uint16_t*)tok, (const uint16_t*)pos,
                     (uint16_t*)out, ldo, n_rows, seq, vocab, width);
  return hipGetLastError();
}

hipError_t launch_embedding_bwd(const int32_t* ids, const void* dx, int lddx, float* dtok, float* dpos, int batch, int seq, int vocab,
                                int width, hipStream_t s) {
  if (!ids || !dx || !dtok || !dpos || batch <= 0 || seq <= 0 || vocab <= 0 || width <= 0 || width > 2048 || lddx < width) return hipErrorInvalidValue;
  hipError_t e = launch_fill_zero(dtok, (size_t)vocab * width * 4, s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(embedding_bwd_tok_kernel, dim3(batch * seq), dim3(256), 0, s, ids, (const uint16_t*)dx, lddx, dtok, batch * seq, vocab, width);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(embedding_bwd_pos_kernel, dim3(seq), dim3(256), 0, s, (const uint16_t*)dx, lddx, dpos, batch, seq, width);
  return hipGetLastError();
}

}  // namespace spb
