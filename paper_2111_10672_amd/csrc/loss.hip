// Softmax cross-entropy, forward and gradient in one pass over the logits (the loss that ends the
// forward pass and starts the backward pass, Sec. 1-2 of the paper).  Memory-bound: every logit is
// read from HBM once (the row stays in registers or L2 for the second sweep) and every gradient
// entry is written once.
#include "kernels.h"

namespace spb {
namespace {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ void store_dz(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_dz(uint16_t* p, float v) { *p = bf16_round(v); }

// One workgroup of WAVES wavefronts per row when classes is large, one wavefront per row otherwise.
template <typename DZ, int WAVES_PER_ROW>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ logits, int ldz,
                                                           const int32_t* __restrict__ labels, int rows, int classes,
                                                           DZ* __restrict__ dz, int lddz, float* __restrict__ row_loss) {
  constexpr int ROWS_PER_BLOCK = 4 / WAVES_PER_ROW;
  constexpr int STRIDE = 64 * WAVES_PER_ROW;
  __shared__ float red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * ROWS_PER_BLOCK + (WAVES_PER_ROW == 1 ? wave : 0);
  const bool live = row < rows;                      // uniform per wavefront (per workgroup when WAVES_PER_ROW == 4)
  const int first = WAVES_PER_ROW == 1 ? lane : (int)threadIdx.x;
  const float* z = logits + (size_t)(live ? row : 0) * ldz;

  float m = -INFINITY;
  if (live) for (int c = first; c < classes; c += STRIDE) m = fmaxf(m, z[c]);
  m = wave_max(m);
  if (WAVES_PER_ROW > 1) {
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
  }
  float s = 0.f;
  if (live) for (int c = first; c < classes; c += STRIDE) s += expf(z[c] - m);
  s = wave_sum(s);
  if (WAVES_PER_ROW > 1) {
    if (lane == 0) red[wave] = s;
    __syncthreads();
    s = (red[0] + red[1]) + (red[2] + red[3]);
  }
  if (!live) return;
  const float lse = m + logf(s);
  const int y = labels[row];
  const float inv_rows = 1.f / (float)rows;
  DZ* out = dz + (size_t)row * lddz;
  for (int c = first; c < classes; c += STRIDE) {
    const float p = expf(z[c] - lse);
    store_dz(out + c, (p - (c == y ? 1.f : 0.f)) * inv_rows);
  }
  // a label outside [0, classes) contributes no target term instead of reading out of bounds
  for (int c = classes + first; c < lddz; c += STRIDE) store_dz(out + c, 0.f);  // keep the pitch padding zero
  if (first == 0) row_loss[row] = lse - ((unsigned)y < (unsigned)classes ? z[y] : 0.f);
}

// Long rows (a vocabulary of tens of thousands): one workgroup of 512 threads per row holds the whole row in
// registers as 16-byte vectors, so the logits are read from memory exactly once, with every load of the row in
// flight together; the exponentials are kept and only scaled for the gradient.  Columns between `classes` and
// the pitch count as minus infinity on the way in and come out as zero.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kXentThreads = 512, kXentVecs = 16;   // rows of up to 512 * 16 * 4 = 32768 columns, pitch included
__device__ __forceinline__ void store_dz4(float* p, const f32x4& v) { *reinterpret_cast<f32x4*>(p) = v; }
__device__ __forceinline__ void store_dz4(uint16_t* p, const f32x4& v) {
  *reinterpret_cast<uint2*>(p) = make_uint2(bf16_pack2(v[0], v[1]), bf16_pack2(v[2], v[3]));
}
template <typename DZ>
__global__ __launch_bounds__(kXentThreads) void softmax_xent_long_kernel(const float* __restrict__ logits, int ldz,
                                                                        const int32_t* __restrict__ labels, int rows, int classes,
                                                                        DZ* __restrict__ dz, int lddz, float* __restrict__ row_loss) {
  __shared__ float red[kXentThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x;
  const float* z = logits + (size_t)row * ldz;
  f32x4 v[kXentVecs];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < kXentVecs; ++i) {
    const int c = 4 * ((int)threadIdx.x + kXentThreads * i);
    v[i] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (c + 4 <= ldz) v[i] = *reinterpret_cast<const f32x4*>(z + c);
  }
#pragma unroll
  for (int i = 0; i < kXentVecs; ++i) {
    const int c = 4 * ((int)threadIdx.x + kXentThreads * i);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (c + e >= classes) v[i][e] = -INFINITY;
      m = fmaxf(m, v[i][e]);
    }
  }
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = red[0];
#pragma unroll
  for (int w = 1; w < kXentThreads / 64; ++w) m = fmaxf(m, red[w]);
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kXentVecs; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[i][e] = expf(v[i][e] - m); s += v[i][e]; }
  s = wave_sum(s);
  if (lane == 0) red[wave] = s;
  __syncthreads();
  s = red[0];
#pragma unroll
  for (int w = 1; w < kXentThreads / 64; ++w) s += red[w];
  const int y = labels[row];
  const float scale = 1.f / (s * (float)rows), inv_rows = 1.f / (float)rows;
  DZ* out = dz + (size_t)row * lddz;
#pragma unroll
  for (int i = 0; i < kXentVecs; ++i) {
    const int c = 4 * ((int)threadIdx.x + kXentThreads * i);
    if (c + 4 <= lddz) {
      f32x4 g = v[i] * scale;
      // a label outside [0, classes) contributes no target term
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (c + e == y && y < classes) g[e] -= inv_rows;
      store_dz4(out + c, g);
    }
  }
  if (threadIdx.x == 0) row_loss[row] = m + logf(s) - ((unsigned)y < (unsigned)classes ? z[y] : 0.f);
}

// Adds the per-row losses in a fixed order (same result on every run) and stores the mean.
__global__ __launch_bounds__(256) void mean_kernel(const float* __restrict__ row_loss, int rows, float* __restrict__ out) {
  __shared__ float red[4];
  float s = 0.f;
  for (int i = threadIdx.x; i < rows; i += 256) s += row_loss[i];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) out[0] = ((red[0] + red[1]) + (red[2] + red[3])) / (float)rows;
}

// Few classes and few rows (a perceptron's 10-way head): everything in ONE workgroup and one launch.  A row takes
// lpr lanes (the power of two that holds its classes), so a wave works on 64 / lpr rows at a time; the mean adds
// each wave's rows in order and then the four waves in a fixed order.
template <typename DZ>
__global__ __launch_bounds__(256) void softmax_xent_one_block_kernel(const float* __restrict__ logits, int ldz,
                                                                     const int32_t* __restrict__ labels, int rows, int classes, int lpr,
                                                                     DZ* __restrict__ dz, int lddz, float* __restrict__ row_loss,
                                                                     float* __restrict__ loss_out) {
  __shared__ float red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sub = lane % lpr, rows_per_wave = 64 / lpr;
  const float inv_rows = 1.f / (float)rows;
  float acc = 0.f;
  for (int base = 0; base < rows; base += 4 * rows_per_wave) {
    const int row = base + wave * rows_per_wave + lane / lpr;
    const bool live = row < rows, mine = live && sub < classes;
    const float z = mine ? logits[(size_t)row * ldz + sub] : -INFINITY;
    float m = z;
    for (int o = lpr >> 1; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    float s = mine ? expf(z - m) : 0.f;
    for (int o = lpr >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (!live) continue;                       // no shuffles below
    const float lse = m + logf(s);
    const int y = labels[row];
    DZ* out = dz + (size_t)row * lddz;
    if (mine) store_dz(out + sub, (expf(z - lse) - (sub == y ? 1.f : 0.f)) * inv_rows);
    for (int c = classes + sub; c < lddz; c += lpr) store_dz(out + c, 0.f);  // keep the pitch padding zero
    if (sub == 0) {
      // a label outside [0, classes) contributes no target term instead of reading out of bounds
      const float l = lse - ((unsigned)y < (unsigned)classes ? logits[(size_t)row * ldz + y] : 0.f);
      row_loss[row] = l;
      acc += l;
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) red[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) loss_out[0] = ((red[0] + red[1]) + (red[2] + red[3])) * inv_rows;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, size_t words) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

}  // namespace

hipError_t launch_softmax_xent(const float* logits, int ldz, const int32_t* labels, int rows, int classes,
                               void* dz, int lddz, DType dz_dtype, float* row_loss, float* loss_out,
                               hipStream_t stream) {
  if (!logits || !labels || !dz || !row_loss || !loss_out || rows <= 0 || classes <= 0 || ldz < classes || lddz < classes)
    return hipErrorInvalidValue;
  if (classes <= 64 && rows <= 4096) {
    int lpr = 1;
    while (lpr < classes) lpr <<= 1;
    if (dz_dtype == DType::F32)
      hipLaunchKernelGGL((softmax_xent_one_block_kernel<float>), dim3(1), dim3(256), 0, stream, logits, ldz, labels, rows, classes, lpr, (float*)dz, lddz, row_loss, loss_out);
    else
      hipLaunchKernelGGL((softmax_xent_one_block_kernel<uint16_t>), dim3(1), dim3(256), 0, stream, logits, ldz, labels, rows, classes, lpr, (uint16_t*)dz, lddz, row_loss, loss_out);
    return hipGetLastError();
  }
  const bool vec_ok = ldz % 4 == 0 && lddz % 4 == 0 && (reinterpret_cast<uintptr_t>(logits) & 15u) == 0 && (reinterpret_cast<uintptr_t>(dz) & 15u) == 0;
  if (classes > 2048 && vec_ok && (ldz > lddz ? ldz : lddz) <= kXentThreads * kXentVecs * 4) {
    if (dz_dtype == DType::F32)
      hipLaunchKernelGGL((softmax_xent_long_kernel<float>), dim3(rows), dim3(kXentThreads), 0, stream, logits, ldz, labels, rows, classes, (float*)dz, lddz, row_loss);
    else
      hipLaunchKernelGGL((softmax_xent_long_kernel<uint16_t>), dim3(rows), dim3(kXentThreads), 0, stream, logits, ldz, labels, rows, classes, (uint16_t*)dz, lddz, row_loss);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, stream, row_loss, rows, loss_out);
    return hipGetLastError();
  }
  const bool wide = classes > 2048;
  const int grid = wide ? rows : (rows + 3) / 4;
  if (dz_dtype == DType::F32) {
    if (wide) hipLaunchKernelGGL((softmax_xent_kernel<float, 4>), dim3(grid), dim3(256), 0, stream, logits, ldz, labels, rows, classes, (float*)dz, lddz, row_loss);
    else hipLaunchKernelGGL((softmax_xent_kernel<float, 1>), dim3(grid), dim3(256), 0, stream, logits, ldz, labels, rows, classes, (float*)dz, lddz, row_loss);
  } else {
    if (wide) hipLaunchKernelGGL((softmax_xent_kernel<uint16_t, 4>), dim3(grid), dim3(256), 0, stream, logits, ldz, labels, rows, classes, (uint16_t*)dz, lddz, row_loss);
    else hipLaunchKernelGGL((softmax_xent_kernel<uint16_t, 1>), dim3(grid), dim3(256), 0, stream, logits, ldz, labels, rows, classes, (uint16_t*)dz, lddz, row_loss);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, stream, row_loss, rows, loss_out);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t stream) {
  if (!ptr || bytes % 4) return hipErrorInvalidValue;
  if (bytes == 0) return hipSuccess;
  const size_t words = bytes / 4;
  const int grid = (int)((words + 255) / 256 < 2048 ? (words + 255) / 256 : 2048);
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, stream, (uint32_t*)ptr, words);
  return hipGetLastError();
}

}  // namespace spb
