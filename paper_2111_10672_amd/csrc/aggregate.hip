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
constexpr int kParts = 2;                        // 4-element pieces per thread
constexpr int kChunkElems = 256 * kParts * 4;    // elements per workgroup

struct AggTensor {
  void* w;                         // parameter, model dtype
  float* v;                        // velocity
  const float* g[kMaxAggWorkers];  // contributing workers' gradients, first `count` entries
  long long numel;
  int first_block;                 // first workgroup of this tensor in the launch
  int count;                       // contributors
  float rate;                      // learning rate of this tensor
  int aligned;                     // numel % 4 == 0 and every buffer 16-byte aligned: the vector path
};
struct AggTable {
  AggTensor t[kMaxTensors];
  int n;
  int bf16;
  float momentum, weight_decay;
};

__device__ __forceinline__ float bf(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t to_bf16(float v) { return bf16_round(v); }

// The common case (element count a multiple of 4, every buffer 16-byte aligned): a thread's kParts 4-element pieces, all
// of their C + 2 loads requested before the first is used, parameters as one 8- or 16-byte access per piece.  The
// additions run in worker order, as in the general path below: same bits.
template <int C>
__device__ __forceinline__ void update_aligned(const AggTensor& t, const AggTable& tab, long long base) {
  f32x4 x[kParts][C], vv[kParts], ww[kParts];
  uint2 wb[kParts];
  long long e0[kParts];
  bool live[kParts];
#pragma unroll
  for (int part = 0; part < kParts; ++part) {
    e0[part] = base + (long long)(part * 256 + threadIdx.x) * 4;
    live[part] = e0[part] < t.numel;
    if (!live[part]) continue;
#pragma unroll
    for (int j = 0; j < C; ++j) x[part][j] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(t.g[j] + e0[part]));   // read once
    vv[part] = *reinterpret_cast<const f32x4*>(t.v + e0[part]);
    if (tab.bf16) wb[part] = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(t.w) + e0[part]);
    else ww[part] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(t.w) + e0[part]);
  }
  const float inv = 1.f / (float)C;
#pragma unroll
  for (int part = 0; part < kParts; ++part) {
    if (!live[part]) continue;
    f32x4 g = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < C; ++j) g += x[part][j];   // workers added in index order
    f32x4 w = ww[part];
    if (tab.bf16) w = f32x4{__uint_as_float(wb[part].x << 16), __uint_as_float(wb[part].x & 0xFFFF0000u),
                            __uint_as_float(wb[part].y << 16), __uint_as_float(wb[part].y & 0xFFFF0000u)};
    f32x4 v = vv[part];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = tab.momentum * v[e] + (g[e] * inv + tab.weight_decay * w[e]);
      w[e] = w[e] - t.rate * v[e];
    }
    *reinterpret_cast<f32x4*>(t.v + e0[part]) = v;
    if (tab.bf16)
      *reinterpret_cast<uint2*>(static_cast<uint16_t*>(t.w) + e0[part]) =
          uint2{(uint32_t)to_bf16(w[0]) | ((uint32_t)to_bf16(w[1]) << 16), (uint32_t)to_bf16(w[2]) | ((uint32_t)to_bf16(w[3]) << 16)};
    else *reinterpret_cast<f32x4*>(static_cast<float*>(t.w) + e0[part]) = w;
  }
}

__global__ __launch_bounds__(256) void aggregate_update_kernel(AggTable tab) {
  // which tensor: the last one whose first_block is not past this workgroup (uniform, a handful of compares)
  int ti = 0;
  for (int i = 1; i < tab.n; ++i)
    if ((int)blockIdx.x >= tab.t[i].first_block) ti = i;
  const AggTensor& t = tab.t[ti];
  const long long base = (long long)((int)blockIdx.x - t.first_block) * kChunkElems;
  if (t.aligned) {   // uniform over the workgroup
    switch (t.count) {
      case 1: update_aligned<1>(t, tab, base); return;
      case 2: update_aligned<2>(t, tab, base); return;
      case 3: update_aligned<3>(t, tab, base); return;
      case 4: update_aligned<4>(t, tab, base); return;
      case 5: update_aligned<5>(t, tab, base); return;
      case 6: update_aligned<6>(t, tab, base); return;
      case 7: update_aligned<7>(t, tab, base); return;
      case 8: update_aligned<8>(t, tab, base); return;
      default: break;
    }
  }
  const float inv = 1.f / (float)t.count;
#pragma unroll
  for (int part = 0; part < kParts; ++part) {
    const long long e0 = base + (long long)(part * 256 + threadIdx.x) * 4;
    if (e0 >= t.numel) continue;
    float g[4] = {0.f, 0.f, 0.f, 0.f}, w[4], v[4];
    const int live = (int)(t.numel - e0 < 4 ? t.numel - e0 : 4);
    for (int j = 0; j < t.count; ++j)   // workers added in index order
      for (int e = 0; e < live; ++e) g[e] += t.g[j][e0 + e];
    for (int e = 0; e < live; ++e) v[e] = t.v[e0 + e];
    for (int e = 0; e < live; ++e)
      w[e] = tab.bf16 ? bf(static_cast<const uint16_t*>(t.w)[e0 + e]) : static_cast<const float*>(t.w)[e0 + e];
    for (int e = 0; e < live; ++e) {
      v[e] = tab.momentum * v[e] + (g[e] * inv + tab.weight_decay * w[e]);
      w[e] = w[e] - t.rate * v[e];
    }
    for (int e = 0; e < live; ++e) t.v[e0 + e] = v[e];
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
      uintptr_t bits = reinterpret_cast<uintptr_t>(s.w) | reinterpret_cast<uintptr_t>(s.v) | (uintptr_t)(s.numel & 3);
      for (int j = 0; j < s.count; ++j) {
        if (!s.g[j]) return hipErrorInvalidValue;
        d.g[j] = s.g[j];
        bits |= reinterpret_cast<uintptr_t>(s.g[j]);
      }
      d.aligned = (bits & 15) == 0;
      blocks += (int)((s.numel + kChunkElems - 1) / kChunkElems);
    }
    hipLaunchKernelGGL(aggregate_update_kernel, dim3(blocks), dim3(256), 0, stream, tab);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace spb
