// Host-side model object behind the C ABI: unit list, parameter list, buffer plan, step drivers.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <functional>
#include <map>
#include <memory>
#include <string>
#include <vector>

#include "../../include/spb.h"
#include "kernels.h"

namespace spb {

void set_error(const char* fmt, ...);

struct ParamInfo {
  std::string name;
  int unit = 0;
  DType dtype = DType::BF16;
  std::vector<int64_t> shape;
  int64_t numel() const {
    int64_t n = 1;
    for (auto d : shape) n *= d;
    return n;
  }
};

// Optional HIP-event bracket around every launch, summed per kernel class.
class KernelTimer {
 public:
  ~KernelTimer();
  void enable(bool on);
  bool enabled() const { return enabled_; }
  hipError_t run(const char* name, double flops, double bytes, hipStream_t stream, const std::function<hipError_t()>& launch);
  int read(spb_kernel_time* out, int cap, int* n_out);

 private:
  struct Rec { std::string name; hipEvent_t start, stop; double flops, bytes; };
  void get_events(hipEvent_t* a, hipEvent_t* b);
  bool enabled_ = false;
  std::vector<Rec> recs_;
  std::vector<hipEvent_t> pool_;
};

class Model {
 public:
  virtual ~Model();
  virtual size_t workspace_size(int k) const = 0;
  virtual int forward(const void* x, const int32_t* labels, const int32_t* loss_rows, int k, void* ws, float* loss_out, hipStream_t s) = 0;
  virtual int backward(int k, hipStream_t s) = 0;
  // Where a forward pass that stashed for depth k keeps the input of unit `unit` (>= L - k), and where the gradient
  // with respect to that unit's output lies once a backward pass of depth exactly L - unit has run (the unit being
  // the lowest visited one, nothing has overwritten it).  Host-only.
  virtual void unit_io(int k, int unit, spb_buffer_view* input, spb_buffer_view* output_grad) const = 0;

  int num_units = 0;
  DType dtype = DType::BF16;
  std::vector<ParamInfo> params;
  std::vector<void*> param_ptrs, grad_ptrs;
  bool params_bound = false, grads_bound = false;
  bool needs_loss_rows = false;
  int stashed_k = -1;  // depth the last forward pass stashed for; -1 = no forward yet
  void* ws = nullptr;
  KernelTimer timer;
  struct Product { GemmProblem first, second; bool pair = false; };
  std::map<std::string, Product> last_product;  // per kernel class, the most recent product or pair (kept while timing is on)
  int replay(const char* name, int count, hipStream_t s);

  // Creates the side stream (see fork) unless s is being captured into a graph right now; called by the C ABI
  // before a forward pass, so a model built on a machine without a GPU never touches the runtime.
  void ensure_side_stream(hipStream_t s);
  int finish(hipStream_t s) { return join(s); }   // after a backward pass: s waits for whatever is still on the side stream

 protected:
  // Work that does not feed the main chain of a backward pass (a layer's weight gradient, beside its input
  // gradient) goes to a second stream so that both kinds of kernel share the chip: fork(s) makes the side
  // stream wait for everything enqueued on s so far and returns it; join(s) makes s wait for everything enqueued
  // on the side stream.  While kernels are being timed, while s is being captured into a graph, or before the
  // side stream exists, fork returns s itself and everything stays in one order.
  hipStream_t fork(hipStream_t s);
  int join(hipStream_t s);
  // Finer than join: mark() stands for everything enqueued on the side stream so far (-1 when nothing is forked),
  // wait_mark(s, m) makes s wait for just that.  At most kMarks marks are live at a time.
  static constexpr int kMarks = 16;
  int mark();
  int wait_mark(hipStream_t s, int m);
  int gemm(const GemmProblem& p, hipStream_t s);
  int gemm_pair(const GemmProblem& d, const GemmProblem& w, hipStream_t s);  // see launch_gemm_pair
  int run(const char* name, double bytes, hipStream_t s, const std::function<hipError_t()>& launch);
  int check(hipError_t e, const char* what);

 private:
  hipStream_t side_ = nullptr;
  hipEvent_t fork_ev_ = nullptr, join_ev_ = nullptr, mark_ev_[kMarks] = {};
  int next_mark_ = 0;
  bool forked_ = false;
};

std::unique_ptr<Model> make_mlp(const spb_model_desc& d);
std::unique_ptr<Model> make_encoder(const spb_model_desc& d);
std::unique_ptr<Model> make_resnet(const spb_model_desc& d);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline spb_buffer_view make_view(long long offset, long long rows, long long cols, long long pitch, DType t, int relu_applied = 0) {
  spb_buffer_view v;
  v.offset = offset; v.rows = rows; v.cols = cols; v.pitch = pitch;
  v.dtype = t == DType::F32 ? SPB_DTYPE_F32 : SPB_DTYPE_BF16; v.relu_applied = relu_applied;
  return v;
}
inline spb_buffer_view no_view() { spb_buffer_view v; v.offset = SPB_VIEW_NONE; v.rows = v.cols = v.pitch = 0; v.dtype = SPB_DTYPE_BF16; v.relu_applied = 0; return v; }


}  // namespace spb

struct spb_model {
  std::unique_ptr<spb::Model> impl;
};
