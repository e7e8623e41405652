// Memory-bound kernels of the residual-CNN units (activations NHWC bfloat16, channel counts multiples of 8):
// the backward of "per-channel affine -> ReLU" with its per-channel reductions, the pools, channel padding of
// the 3-channel input, and the fixed-order sum of split-k partial products.  Each moves every tensor through
// HBM once, in 16-byte pieces along the channel index.
#include <algorithm>

#include "kernels.h"

namespace spb {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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
__device__ __forceinline__ float bf(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t to_bf16(float v) { return bf16_round(v); }

// Backward of z = scale * y + shift followed by an optional ReLU whose output is `act`:
//   dz = dout * [act > 0]   (dz = dout without act);   dy = scale * dz;   dsum = dz (optional)
//   partial[block][0][c] = sum over the block's rows of dz * y;   partial[block][1][c] = sum of dz
// A workgroup takes a range of rows (blockIdx.x) of a slab of at most 256 channels (blockIdx.y), so that wide
// tensors still give many workgroups while the partial sums stay small next to the tensor.  Thread t owns chunk
// t % slab_chunks of the slab, rows (t / slab_chunks), (t / slab_chunks) + rows_per_pass, ...
constexpr int kAffineSlabChunks = 32;
__global__ __launch_bounds__(256) void affine_relu_bwd_kernel(const uint16_t* __restrict__ dout, const uint16_t* __restrict__ act,
                                                              const uint16_t* __restrict__ y, const uint16_t* __restrict__ scale,
                                                              uint16_t* __restrict__ dy, uint16_t* __restrict__ dsum,
                                                              float* __restrict__ partial, long long rows, int channels, int rows_per_block) {
  extern __shared__ float sh[];  // [rows_per_pass][slab_chunks][16]
  const int chunks = channels >> 3;
  const int slab_chunks = min(chunks, kAffineSlabChunks);
  const int rows_per_pass = 256 / slab_chunks;
  const int local_chunk = threadIdx.x % slab_chunks, lane_row = threadIdx.x / slab_chunks;
  const int chunk = blockIdx.y * slab_chunks + local_chunk;
  const bool active = lane_row < rows_per_pass && chunk < chunks;
  float s1[8], s0[8], sc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { s1[e] = 0.f; s0[e] = 0.f; sc[e] = 0.f; }
  if (active) unpack8(*reinterpret_cast<const u32x4*>(scale + chunk * 8), sc);
  const long long first = (long long)blockIdx.x * rows_per_block;
  const long long last = min(rows, first + rows_per_block);
  if (active) {
    // two rows per trip, all their loads requested before the first is used
    auto finish = [&](size_t off, const u32x4& dw, const u32x4& yw, const u32x4& aw) {
      float d[8], yv[8], o[8];
      unpack8(dw, d);
      unpack8(yw, yv);
      if (act) {
        float a[8];
        unpack8(aw, a);
#pragma unroll
        for (int e = 0; e < 8; ++e) if (!(a[e] > 0.f)) d[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) { s1[e] += d[e] * yv[e]; s0[e] += d[e]; o[e] = sc[e] * d[e]; }
      *reinterpret_cast<u32x4*>(dy + off) = pack8(o);
      if (dsum) *reinterpret_cast<u32x4*>(dsum + off) = pack8(d);
    };
    // The three inputs are read here for the last time in the step (the gradient, the kept pre-affine output, the
    // kept activation): streaming loads, so they do not push the freshly written dy, which the next product reads,
    // out of the caches.  Four rows per trip, all their loads requested before the first is used.
    const u32x4 zero = {0u, 0u, 0u, 0u};
    auto fetch = [&](const uint16_t* base, size_t off) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off)); };
    long long r = first + lane_row;
    const size_t pass = (size_t)rows_per_pass * channels;
    for (; r + 3 * rows_per_pass < last; r += 4 * rows_per_pass) {
      const size_t off0 = (size_t)r * channels + chunk * 8;
      u32x4 d[4], yv[4], a[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        d[u] = fetch(dout, off0 + u * pass);
        yv[u] = fetch(y, off0 + u * pass);
        a[u] = act ? fetch(act, off0 + u * pass) : zero;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) finish(off0 + u * pass, d[u], yv[u], a[u]);
    }
    for (; r < last; r += rows_per_pass) {
      const size_t off = (size_t)r * channels + chunk * 8;
      finish(off, fetch(dout, off), fetch(y, off), act ? fetch(act, off) : zero);
    }
  }
  if (lane_row < rows_per_pass) {  // lanes past the tensor's last chunk park zeros
    float* mine = sh + ((size_t)lane_row * slab_chunks + local_chunk) * 16;
#pragma unroll
    for (int e = 0; e < 8; ++e) { mine[e] = s1[e]; mine[8 + e] = s0[e]; }
  }
  __syncthreads();
  // column sums over the block's row lanes, in lane order
  const int slab_cols = slab_chunks * 8;
  for (int col = threadIdx.x; col < 2 * slab_cols; col += 256) {
    const int which = col / slab_cols, c = col % slab_cols;
    const int channel = blockIdx.y * slab_cols + c;
    if (channel >= channels) continue;
    float acc = 0.f;
    for (int l = 0; l < rows_per_pass; ++l) acc += sh[((size_t)l * slab_chunks + (c >> 3)) * 16 + which * 8 + (c & 7)];
    partial[((size_t)blockIdx.x * 2 + which) * channels + channel] = acc;
  }
}

// out_a[c] = sum_b partial[b][0][c], out_b[c] = sum_b partial[b][1][c].  A workgroup takes 16 neighbouring columns
// (reduce_pairs_blocks workgroups in all): thread (g, c) adds blocks g, g + 16, ... of column c in order - the 16
// threads of a group read 64 contiguous bytes, where one wavefront per column touched a cache line per lane - and
// the 16 group sums of a column are added in group order: the same bits on every run.
__device__ __forceinline__ void reduce_pairs_block(unsigned block, const float* __restrict__ partial, int n_blocks, int width,
                                                   float* __restrict__ out_a, float* __restrict__ out_b) {
  __shared__ float sh[16][17];
  const int c = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int col = block * 16 + c;
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
__global__ __launch_bounds__(256) void reduce_pairs_kernel(const float* __restrict__ partial, int n_blocks, int width,
                                                           float* __restrict__ out_a, float* __restrict__ out_b) {
  reduce_pairs_block(blockIdx.x, partial, n_blocks, width, out_a, out_b);
}

// out[j] = sum over slices of partial[slice][map(j)], slices added in index order; map drops padded input channels.
__device__ __forceinline__ void splitk_reduce_block(unsigned block, const float* __restrict__ partial, int slices, long long slice_stride,
                                                    float* __restrict__ out, long long numel, int cin, int cin_padded) {
  const long long j = (long long)block * 256 + threadIdx.x;
  if (j >= numel) return;
  const long long src = cin == cin_padded ? j : (j / cin) * cin_padded + (j % cin);
  float s = 0.f;
  for (int z = 0; z < slices; ++z) s += partial[(size_t)z * slice_stride + src];
  out[j] = s;
}
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int slices, long long slice_stride,
                                                            float* __restrict__ out, long long numel, int cin, int cin_padded) {
  splitk_reduce_block(blockIdx.x, partial, slices, slice_stride, out, numel, cin, cin_padded);
}

// The same for tensors without channel padding, four neighbouring elements per thread and four slices requested
// at a time (the additions still run in slice order).
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void splitk_reduce4_block(unsigned block, const f32x4* __restrict__ partial, int slices, long long slice_stride4,
                                                     f32x4* __restrict__ out, long long numel4) {
  const long long j = (long long)block * 256 + threadIdx.x;
  if (j >= numel4) return;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  int z = 0;
  for (; z + 4 <= slices; z += 4) {
    const f32x4 a = partial[(size_t)z * slice_stride4 + j], b = partial[(size_t)(z + 1) * slice_stride4 + j];
    const f32x4 c = partial[(size_t)(z + 2) * slice_stride4 + j], d = partial[(size_t)(z + 3) * slice_stride4 + j];
    s += a; s += b; s += c; s += d;
  }
  for (; z < slices; ++z) s += partial[(size_t)z * slice_stride4 + j];
  out[j] = s;
}
__global__ __launch_bounds__(256) void splitk_reduce4_kernel(const f32x4* __restrict__ partial, int slices, long long slice_stride4,
                                                             f32x4* __restrict__ out, long long numel4) {
  splitk_reduce4_block(blockIdx.x, partial, slices, slice_stride4, out, numel4);
}

// Several of the reductions above in one launch: the column sums of a unit's affine backward passes and the k-slice
// sums of its weight gradients are a handful of tiny kernels each bound by its launch; a table in the kernel
// arguments says which range of workgroups does which, with the arithmetic (and so the bits) of the kernels above.
__global__ __launch_bounds__(256) void unit_reduce_kernel(ReduceTable t) {
  int i = 0;
  while (i + 1 < t.n && blockIdx.x >= t.end_block[i]) ++i;
  const unsigned block = blockIdx.x - (i ? t.end_block[i - 1] : 0u);
  const ReduceTask& k = t.task[i];
  if (k.kind == ReduceTask::kPairs) reduce_pairs_block(block, k.partial, k.count, k.width, k.out, k.out_b);
  else if (k.kind == ReduceTask::kSlices4)
    splitk_reduce4_block(block, reinterpret_cast<const f32x4*>(k.partial), k.count, k.stride, reinterpret_cast<f32x4*>(k.out), k.numel);
  else splitk_reduce_block(block, k.partial, k.count, k.stride, k.out, k.numel, k.cin, k.cin_padded);
}

// The same with a bfloat16 result (the input gradient of a product whose k range was cut into slices): eight
// neighbouring elements per thread, slices added in index order, one rounding at the end.
__global__ __launch_bounds__(256) void splitk_reduce_bf16_kernel(const f32x4* __restrict__ partial, int slices, long long slice_stride4,
                                                                 uint4* __restrict__ out, long long numel8) {
  const long long j = (long long)blockIdx.x * 256 + threadIdx.x;
  if (j >= numel8) return;
  f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = lo;
#pragma unroll 4
  for (int z = 0; z < slices; ++z) {
    lo += partial[(size_t)z * slice_stride4 + 2 * j];
    hi += partial[(size_t)z * slice_stride4 + 2 * j + 1];
  }
  out[j] = make_uint4(bf16_pack2(lo[0], lo[1]), bf16_pack2(lo[2], lo[3]), bf16_pack2(hi[0], hi[1]), bf16_pack2(hi[2], hi[3]));
}

// 3x3 window, stride 2, padding 1 (acting as -inf); the first maximum in row-major window order wins.
// which[n, oh, ow, c] (optional) = index 0..8 of the winning window position.
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ out, uint8_t* __restrict__ which,
                                                          int n, int h, int w, int c, int oh, int ow) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)n * oh * ow * c) return;
  const int ch = idx % c;
  long long t = idx / c;
  const int j = t % ow; t /= ow;
  const int i = t % oh;
  const int b = t / oh;
  float best = -INFINITY;
  int arg = 0;
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      const int hi = 2 * i + r - 1, wi = 2 * j + s - 1;
      if ((unsigned)hi < (unsigned)h && (unsigned)wi < (unsigned)w) {
        const float v = bf(x[((size_t)(b * h + hi) * w + wi) * c + ch]);
        if (v > best) { best = v; arg = r * 3 + s; }
      }
    }
  out[idx] = to_bf16(best);
  if (which) which[idx] = (uint8_t)arg;
}

// The same, eight channels (16 bytes) per thread, for channel counts that are multiples of 8.
__global__ __launch_bounds__(256) void maxpool_fwd8_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ out, uint8_t* __restrict__ which,
                                                           int n, int h, int w, int c, int oh, int ow) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const int c8 = c >> 3;
  if (idx >= (long long)n * oh * ow * c8) return;
  const int chunk = idx % c8;
  long long t = idx / c8;
  const int j = t % ow; t /= ow;
  const int i = t % oh;
  const int b = t / oh;
  float best[8];
  int arg[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { best[e] = -INFINITY; arg[e] = 0; }
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      const int hi = 2 * i + r - 1, wi = 2 * j + s - 1;
      if ((unsigned)hi < (unsigned)h && (unsigned)wi < (unsigned)w) {
        float v[8];
        unpack8(*reinterpret_cast<const u32x4*>(x + ((size_t)(b * h + hi) * w + wi) * c + chunk * 8), v);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (v[e] > best[e]) { best[e] = v[e]; arg[e] = r * 3 + s; }
      }
    }
  const size_t o = (size_t)idx * 8;
  *reinterpret_cast<u32x4*>(out + o) = pack8(best);
  if (which) {
    uint2 wbits;
    wbits.x = arg[0] | (arg[1] << 8) | (arg[2] << 16) | (arg[3] << 24);
    wbits.y = arg[4] | (arg[5] << 8) | (arg[6] << 16) | (arg[7] << 24);
    *reinterpret_cast<uint2*>(which + o) = wbits;
  }
}

// da[n, h, w, c] = sum of dout over the (at most 4) windows whose maximum sat at (h, w).
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(const uint16_t* __restrict__ dout, const uint8_t* __restrict__ which,
                                                          uint16_t* __restrict__ da, int n, int h, int w, int c, int oh, int ow) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)n * h * w * c) return;
  const int ch = idx % c;
  long long t = idx / c;
  const int wi = t % w; t /= w;
  const int hi = t % h;
  const int b = t / h;
  float acc = 0.f;
  for (int i = (hi + 1) / 2 - (hi & 1); i <= (hi + 1) / 2; ++i) {     // windows with 2i-1 <= hi <= 2i+1: one for even hi, two for odd
    if (i < 0 || i >= oh) continue;
    for (int j = (wi + 1) / 2 - (wi & 1); j <= (wi + 1) / 2; ++j) {
      if (j < 0 || j >= ow) continue;
      const size_t o = ((size_t)(b * oh + i) * ow + j) * c + ch;
      if (which[o] == (hi - 2 * i + 1) * 3 + (wi - 2 * j + 1)) acc += bf(dout[o]);
    }
  }
  da[idx] = to_bf16(acc);
}

// pooled[n, c] = mean over the hw pixels of x[n, :, c]
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ pooled, int n, int hw, int c) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= n * c) return;
  const int b = idx / c, ch = idx % c;
  float acc = 0.f;
  for (int p = 0; p < hw; ++p) acc += bf(x[((size_t)b * hw + p) * c + ch]);
  pooled[idx] = to_bf16(acc / (float)hw);
}

// dx[n, p, c] = dpooled[n, c] / hw
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(const uint16_t* __restrict__ dpooled, uint16_t* __restrict__ dx, int n, int hw, int c) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)n * hw * c) return;
  const int ch = idx % c;
  const int b = idx / ((long long)hw * c);
  dx[idx] = to_bf16(bf(dpooled[b * c + ch]) / (float)hw);
}

// out[row, 0..c_out) = in[row, 0..c_in) followed by zeros
__global__ __launch_bounds__(256) void pad_channels_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out, long long rows, int c_in, int c_out) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * c_out) return;
  const int ch = idx % c_out;
  out[idx] = ch < c_in ? in[(idx / c_out) * c_in + ch] : (uint16_t)0;
}

unsigned blocks_for(long long n) { return (unsigned)((n + 255) / 256); }

}  // namespace

// rows handled by one workgroup of the affine backward kernel, and the size of its partial buffer
static int affine_slab_chunks(int channels) { return std::min(channels >> 3, kAffineSlabChunks); }
static int affine_slabs(int channels) { return ((channels >> 3) + affine_slab_chunks(channels) - 1) / affine_slab_chunks(channels); }
static int affine_rows_per_block(long long rows, int channels) {
  const int per_pass = 256 / affine_slab_chunks(channels);
  const long long row_blocks = std::max(1, 1024 / affine_slabs(channels));  // about a thousand workgroups in all
  long long want = (rows + row_blocks - 1) / row_blocks;
  want = (want + per_pass - 1) / per_pass * per_pass;
  return (int)std::max<long long>(want, 4LL * per_pass);
}
size_t affine_partial_floats(long long rows, int channels) {
  const int rpb = affine_rows_per_block(rows, channels);
  return (size_t)((rows + rpb - 1) / rpb) * 2 * channels;
}

hipError_t launch_affine_relu_bwd(const void* dout, const void* act, const void* y, const void* scale, void* dy, void* dsum,
                                  float* partial, float* dscale, float* dshift, long long rows, int channels, hipStream_t s, ReduceTask* deferred) {
  if (!dout || !y || !scale || !dy || !partial || !dscale || !dshift || rows <= 0 || channels <= 0 || channels % 8 || channels > 2048)
    return hipErrorInvalidValue;
  const int rpb = affine_rows_per_block(rows, channels);
  const int blocks = (int)((rows + rpb - 1) / rpb);
  const int slab_chunks = affine_slab_chunks(channels);
  const size_t lds = (size_t)(256 / slab_chunks) * slab_chunks * 16 * sizeof(float);
  hipLaunchKernelGGL(affine_relu_bwd_kernel, dim3(blocks, affine_slabs(channels)), dim3(256), lds, s, (const uint16_t*)dout, (const uint16_t*)act,
                     (const uint16_t*)y, (const uint16_t*)scale, (uint16_t*)dy, (uint16_t*)dsum, partial, rows, channels, rpb);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (deferred) {   // the caller adds the column sums up later (launch_unit_reduce)
    deferred->kind = ReduceTask::kPairs; deferred->partial = partial; deferred->count = blocks; deferred->width = channels;
    deferred->out = dscale; deferred->out_b = dshift; deferred->blocks = reduce_pairs_blocks(channels);
    return hipSuccess;
  }
  hipLaunchKernelGGL(reduce_pairs_kernel, dim3(reduce_pairs_blocks(channels)), dim3(256), 0, s, partial, blocks, channels, dscale, dshift);
  return hipGetLastError();
}

bool make_splitk_reduce_task(const float* partial, int slices, long long slice_stride, float* out, long long numel, int cin, int cin_padded,
                             ReduceTask* task) {
  if (!partial || !out || !task || slices < 1 || numel <= 0 || cin <= 0 || cin_padded < cin) return false;
  task->partial = partial; task->count = slices; task->out = out; task->out_b = nullptr; task->width = 0;
  task->cin = cin; task->cin_padded = cin_padded;
  if (cin == cin_padded && numel % 4 == 0 && slice_stride % 4 == 0 && (reinterpret_cast<uintptr_t>(partial) & 15) == 0 &&
      (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
    task->kind = ReduceTask::kSlices4; task->stride = slice_stride / 4; task->numel = numel / 4;
  } else {
    task->kind = ReduceTask::kSlices; task->stride = slice_stride; task->numel = numel;
  }
  task->blocks = blocks_for(task->numel);
  return true;
}

hipError_t launch_unit_reduce(const ReduceTask* tasks, int n, hipStream_t s) {
  if (!tasks || n < 1) return hipErrorInvalidValue;
  for (int first = 0; first < n; first += ReduceTable::kMax) {   // more than a table holds: several launches
    ReduceTable t;
    t.n = std::min(n - first, (int)ReduceTable::kMax);
    unsigned end = 0;
    for (int i = 0; i < t.n; ++i) {
      t.task[i] = tasks[first + i];
      if (t.task[i].blocks == 0) return hipErrorInvalidValue;
      end += t.task[i].blocks;
      t.end_block[i] = end;
    }
    hipLaunchKernelGGL(unit_reduce_kernel, dim3(end), dim3(256), 0, s, t);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_splitk_reduce(const float* partial, int slices, long long slice_stride, float* out, long long numel, int cin, int cin_padded,
                                hipStream_t s) {
  if (!partial || !out || slices < 1 || numel <= 0 || cin <= 0 || cin_padded < cin) return hipErrorInvalidValue;
  if (cin == cin_padded && numel % 4 == 0 && slice_stride % 4 == 0 && (reinterpret_cast<uintptr_t>(partial) & 15) == 0 &&
      (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
    hipLaunchKernelGGL(splitk_reduce4_kernel, dim3(blocks_for(numel / 4)), dim3(256), 0, s, reinterpret_cast<const f32x4*>(partial), slices,
                       slice_stride / 4, reinterpret_cast<f32x4*>(out), numel / 4);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks_for(numel)), dim3(256), 0, s, partial, slices, slice_stride, out, numel, cin, cin_padded);
  return hipGetLastError();
}

hipError_t launch_splitk_reduce_bf16(const float* partial, int slices, long long slice_stride, void* out, long long numel, hipStream_t s) {
  if (!partial || !out || slices < 1 || numel <= 0 || numel % 8 || slice_stride % 4 || slice_stride < numel ||
      (reinterpret_cast<uintptr_t>(partial) & 15) || (reinterpret_cast<uintptr_t>(out) & 15))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(splitk_reduce_bf16_kernel, dim3(blocks_for(numel / 8)), dim3(256), 0, s, reinterpret_cast<const f32x4*>(partial), slices,
                     slice_stride / 4, reinterpret_cast<uint4*>(out), numel / 8);
  return hipGetLastError();
}

hipError_t launch_maxpool_fwd(const void* x, void* out, uint8_t* which, int n, int h, int w, int c, hipStream_t s) {
  if (!x || !out || n <= 0 || h <= 0 || w <= 0 || c <= 0) return hipErrorInvalidValue;
  const int oh = (h - 1) / 2 + 1, ow = (w - 1) / 2 + 1;
  const bool aligned = ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(out)) & 15) == 0 && (reinterpret_cast<uintptr_t>(which) & 7) == 0;
  if (c % 8 == 0 && aligned) {
    hipLaunchKernelGGL(maxpool_fwd8_kernel, dim3(blocks_for((long long)n * oh * ow * (c / 8))), dim3(256), 0, s, (const uint16_t*)x, (uint16_t*)out, which, n, h, w, c, oh, ow);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(blocks_for((long long)n * oh * ow * c)), dim3(256), 0, s, (const uint16_t*)x, (uint16_t*)out, which, n, h, w, c, oh, ow);
  return hipGetLastError();
}

hipError_t launch_maxpool_bwd(const void* dout, const uint8_t* which, void* da, int n, int h, int w, int c, hipStream_t s) {
  if (!dout || !which || !da || n <= 0 || h <= 0 || w <= 0 || c <= 0) return hipErrorInvalidValue;
  const int oh = (h - 1) / 2 + 1, ow = (w - 1) / 2 + 1;
  hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(blocks_for((long long)n * h * w * c)), dim3(256), 0, s, (const uint16_t*)dout, which, (uint16_t*)da, n, h, w, c, oh, ow);
  return hipGetLastError();
}

hipError_t launch_avgpool_fwd(const void* x, void* pooled, int n, int hw, int c, hipStream_t s) {
  if (!x || !pooled || n <= 0 || hw <= 0 || c <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(avgpool_fwd_kernel, dim3(blocks_for((long long)n * c)), dim3(256), 0, s, (const uint16_t*)x, (uint16_t*)pooled, n, hw, c);
  return hipGetLastError();
}

hipError_t launch_avgpool_bwd(const void* dpooled, void* dx, int n, int hw, int c, hipStream_t s) {
  if (!dpooled || !dx || n <= 0 || hw <= 0 || c <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(blocks_for((long long)n * hw * c)), dim3(256), 0, s, (const uint16_t*)dpooled, (uint16_t*)dx, n, hw, c);
  return hipGetLastError();
}

hipError_t launch_pad_channels(const void* in, void* out, long long rows, int c_in, int c_out, hipStream_t s) {
  if (!in || !out || rows <= 0 || c_in <= 0 || c_out < c_in) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pad_channels_kernel, dim3(blocks_for(rows * c_out)), dim3(256), 0, s, (const uint16_t*)in, (uint16_t*)out, rows, c_in, c_out);
  return hipGetLastError();
}

}  // namespace spb
