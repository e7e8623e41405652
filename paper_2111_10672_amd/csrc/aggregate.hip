// Server side of one SPB iteration (Sec. 2 of the paper): each parameter's gradient is the average over the
// workers whose backpropagated suffix reached it, its learning rate is scaled with their number, and the
// parameter takes one step of SGD with momentum and weight decay (Sec. 4.1).
//
// Memory-bound: per element c float32 gradient reads, one velocity read and write, one parameter read and
// write, nothing else.  A model has up to a few hundred parameter tensors, most of them tiny, so one launch
// takes a table of up to kMaxTensors tensors in its kernel arguments (no device-side table, nothing allocated)
// and a workgroup looks up which tensor its 16-byte-chunk range belongs to.
#include "kernels.h"

namespace spb {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxTensors = 24;
constexpr int kChunkElems = 2048;  // elements per workgroup: 256 threads x 2 x 4

struct AggTensor {
  void* w;                         // parameter, model dtype
  float* v;                        // velocity
  const float* g[kMaxAggWorkers];  // contributing workers' gradients, first `count` entries
  long long numel;
  int first_block;                 // first workgroup of this tensor in the launch
  int count;                       // contributors
  float rate;                      // learning rate of this tensor
};
struct AggTable {
  AggTensor t[kMaxTensors];
  int n;
  int bf16;
  float momentum, weight_decay;
};

__device__ __forceinline__ float bf(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t to_bf16(float v) { return bf16_round(v); }

__global__ __launch_bounds__(256) void aggregate_update_kernel(AggTable tab) {
  // which tensor: the last one whose first_block is not past this workgroup (uniform, a handful of compares)
  int ti = 0;
  for (int i = 1; i < tab.n; ++i)
    if ((int)blockIdx.x >= tab.t[i].first_block) ti = i;
  const AggTensor& t = tab.t[ti];
  const long long base = (long long)((int)blockIdx.x - t.first_block) * kChunkElems;
  const float inv = 1.f / (float)t.count;
  const bool vec = (t.numel & 3) == 0;
#pragma unroll
  for (int part = 0; part < 2; ++part) {
    const long long e0 = base + (long long)(part * 256 + threadIdx.x) * 4;
    if (e0 >= t.numel) continue;
    float g[4] = {0.f, 0.f, 0.f, 0.f}, w[4], v[4];
    const int live = (int)(t.numel - e0 < 4 ? t.numel - e0 : 4);
    if (vec) {
      for (int j = 0; j < t.count; ++j) {   // workers added in index order
        const f32x4 x = *reinterpret_cast<const f32x4*>(t.g[j] + e0);
        g[0] += x[0]; g[1] += x[1]; g[2] += x[2]; g[3] += x[3];
      }
      const f32x4 vv = *reinterpret_cast<const f32x4*>(t.v + e0);
      v[0] = vv[0]; v[1] = vv[1]; v[2] = vv[2]; v[3] = vv[3];
    } else {
      for (int j = 0; j < t.count; ++j)
        for (int e = 0; e < live; ++e) g[e] += t.g[j][e0 + e];
      for (int e = 0; e < live; ++e) v[e] = t.v[e0 + e];
    }
    for (int e = 0; e < live; ++e)
      w[e] = tab.bf16 ? bf(static_cast<const uint16_t*>(t.w)[e0 + e]) : static_cast<const float*>(t.w)[e0 + e];
    for (int e = 0; e < live; ++e) {
      v[e] = tab.momentum * v[e] + (g[e] * inv + tab.weight_decay * w[e]);
      w[e] = w[e] - t.rate * v[e];
    }
    if (vec) *reinterpret_cast<f32x4*>(t.v + e0) = f32x4{v[0], v[1], v[2], v[3]};
    else for (int e = 0; e < live; ++e) t.v[e0 + e] = v[e];
    for (int e = 0; e < live; ++e) {
      if (tab.bf16) static_cast<uint16_t*>(t.w)[e0 + e] = to_bf16(w[e]);
      else static_cast<float*>(t.w)[e0 + e] = w[e];
    }
  }
}

}  // namespace

hipError_t launch_aggregate_update(const AggregateTensor* tensors, int n_tensors, DType param_dtype, float momentum,
                                   float weight_decay, hipStream_t stream) {
  if (!tensors || n_tensors < 0) return hipErrorInvalidValue;
  int i = 0;
  while (i < n_tensors) {
    AggTable tab;
    tab.n = 0; tab.bf16 = param_dtype == DType::BF16; tab.momentum = momentum; tab.weight_decay = weight_decay;
    int blocks = 0;
    for (; i < n_tensors && tab.n < kMaxTensors; ++i) {
      const AggregateTensor& s = tensors[i];
      if (!s.w || !s.v || s.numel <= 0 || s.count < 1 || s.count > kMaxAggWorkers) return hipErrorInvalidValue;
      AggTensor& d = tab.t[tab.n++];
      d.w = s.w; d.v = s.v; d.numel = s.numel; d.count = s.count; d.rate = s.rate; d.first_block = blocks;
      for (int j = 0; j < s.count; ++j) {
        if (!s.g[j]) return hipErrorInvalidValue;
        d.g[j] = s.g[j];
      }
      blocks += (int)((s.numel + kChunkElems - 1) / kChunkElems);
    }
    hipLaunchKernelGGL(aggregate_update_kernel, dim3(blocks), dim3(256), 0, stream, tab);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace spb
