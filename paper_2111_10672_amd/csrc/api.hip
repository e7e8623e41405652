// The C ABI (include/spb.h): argument checks on the host, then the family's step driver.
#include <cstdlib>
#include "model.h"

#include <cstring>
#include <map>
#include <mutex>

namespace spb {

static thread_local std::string g_last_error;

void set_error(const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
}

int Model::check(hipError_t e, const char* what) {
  if (e == hipSuccess) return SPB_OK;
  if (e == hipErrorInvalidValue) { set_error("%s: shapes or alignment not accepted by the kernel", what); return SPB_ERR_INVALID_ARG; }
  set_error("%s: %s", what, hipGetErrorString(e));
  return SPB_ERR_HIP;
}

int Model::replay(const char* name, int count, hipStream_t s) {
  auto it = last_product.find(name);
  if (it == last_product.end()) { set_error("spb_replay_kernel: no product of class %s has run with timing enabled", name); return SPB_ERR_STATE; }
  const Product& pr = it->second;
  for (int i = 0; i < count; ++i)
    if (int rc = check(pr.pair ? launch_gemm_pair(pr.first, pr.second, s) : launch_gemm(pr.first, s), name)) return rc;
  return SPB_OK;
}

Model::~Model() {
  if (side_) (void)hipStreamDestroy(side_);
  if (fork_ev_) (void)hipEventDestroy(fork_ev_);
  if (join_ev_) (void)hipEventDestroy(join_ev_);
  for (auto e : mark_ev_) if (e) (void)hipEventDestroy(e);
}

void Model::ensure_side_stream(hipStream_t s) {
  if (side_) return;
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess || st != hipStreamCaptureStatusNone) { (void)hipGetLastError(); return; }
  hipStream_t q = nullptr;
  hipEvent_t ev[2 + kMarks] = {};
  bool ok = hipStreamCreateWithFlags(&q, hipStreamNonBlocking) == hipSuccess;
  for (int i = 0; ok && i < 2 + kMarks; ++i) ok = hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) == hipSuccess;
  if (ok) {
    side_ = q; fork_ev_ = ev[0]; join_ev_ = ev[1];
    for (int i = 0; i < kMarks; ++i) mark_ev_[i] = ev[2 + i];
    return;
  }
  (void)hipGetLastError();
  if (q) (void)hipStreamDestroy(q);
  for (auto e : ev) if (e) (void)hipEventDestroy(e);
}

int Model::mark() {
  if (!forked_) return -1;
  const int m = next_mark_;
  if (hipEventRecord(mark_ev_[m], side_) != hipSuccess) { (void)hipGetLastError(); return -2; }  // -2: wait for everything instead
  next_mark_ = (next_mark_ + 1) % kMarks;
  return m;
}

int Model::wait_mark(hipStream_t s, int m) {
  if (m == -2) return join(s);
  if (m < 0 || !side_) return SPB_OK;
  return check(hipStreamWaitEvent(s, mark_ev_[m], 0), "wait_mark");
}

hipStream_t Model::fork(hipStream_t s) {
  if (!side_ || timer.enabled()) return s;
  // A graph replays its parallel branches no faster than a single chain here, and every fork and join adds an
  // edge to it: while s is being captured everything stays on s.
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess || st != hipStreamCaptureStatusNone) { (void)hipGetLastError(); return s; }
  if (hipEventRecord(fork_ev_, s) != hipSuccess || hipStreamWaitEvent(side_, fork_ev_, 0) != hipSuccess) { (void)hipGetLastError(); return s; }
  forked_ = true;
  return side_;
}

int Model::join(hipStream_t s) {
  if (!forked_) return SPB_OK;
  forked_ = false;
  if (int rc = check(hipEventRecord(join_ev_, side_), "join")) return rc;
  return check(hipStreamWaitEvent(s, join_ev_, 0), "join");
}

int Model::gemm(const GemmProblem& p, hipStream_t s) {
  if (!timer.enabled()) return check(launch_gemm(p, s), p.name);
  // while timing, products are told apart by shape as well: "conv_fwd 200704x256x64"
  char key[SPB_NAME_LEN];
  if (p.batch > 1) std::snprintf(key, sizeof key, "%s %dx%dx%d b%d", p.name, p.M, p.N, p.K, p.batch);
  else std::snprintf(key, sizeof key, "%s %dx%dx%d", p.name, p.M, p.N, p.K);
  Product pr;
  pr.first = p;
  last_product[key] = pr;
  hipError_t e = timer.run(key, gemm_flops(p), gemm_bytes(p), s, [&] { return launch_gemm(p, s); });
  return check(e, p.name);
}

int Model::gemm_pair(const GemmProblem& d, const GemmProblem& w, hipStream_t s) {
  if (!gemm_pair_shares_launch(d, w)) {
    if (int rc = gemm(w, s)) return rc;
    return gemm(d, s);
  }
  if (!timer.enabled()) return check(launch_gemm_pair(d, w, s), d.name);
  char key[SPB_NAME_LEN];
  std::snprintf(key, sizeof key, "%s+w %dx%dx%d+%dx%dx%d", d.name, d.M, d.N, d.K, w.M, w.N, w.K);
  Product pr;
  pr.first = d; pr.second = w; pr.pair = true;
  last_product[key] = pr;
  hipError_t e = timer.run(key, gemm_flops(d) + gemm_flops(w), gemm_bytes(d) + gemm_bytes(w), s, [&] { return launch_gemm_pair(d, w, s); });
  return check(e, d.name);
}

int Model::run(const char* name, double bytes, hipStream_t s, const std::function<hipError_t()>& launch) {
  return check(timer.run(name, 0.0, bytes, s, launch), name);
}

KernelTimer::~KernelTimer() {
  for (auto& r : recs_) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  for (auto e : pool_) (void)hipEventDestroy(e);
}

void KernelTimer::enable(bool on) { enabled_ = on; }

void KernelTimer::get_events(hipEvent_t* a, hipEvent_t* b) {
  hipEvent_t* out[2] = {a, b};
  for (auto* o : out) {
    *o = nullptr;
    if (!pool_.empty()) { *o = pool_.back(); pool_.pop_back(); }
    else if (hipEventCreate(o) != hipSuccess) { *o = nullptr; (void)hipGetLastError(); }
  }
}

hipError_t KernelTimer::run(const char* name, double flops, double bytes, hipStream_t stream, const std::function<hipError_t()>& launch) {
  if (!enabled_) return launch();
  Rec r;
  r.name = name; r.flops = flops; r.bytes = bytes;
  get_events(&r.start, &r.stop);
  if (!r.start || !r.stop) {                          // no events to be had: launch untimed rather than record garbage
    if (r.start) pool_.push_back(r.start);
    if (r.stop) pool_.push_back(r.stop);
    return launch();
  }
  const hipError_t e0 = hipEventRecord(r.start, stream);
  const hipError_t e = launch();
  const hipError_t e1 = hipEventRecord(r.stop, stream);
  if (e0 != hipSuccess || e1 != hipSuccess) {         // a bracket that was not recorded must not be read back later
    pool_.push_back(r.start); pool_.push_back(r.stop);
    (void)hipGetLastError();
    return e != hipSuccess ? e : (e0 != hipSuccess ? e0 : e1);
  }
  recs_.push_back(r);
  return e;
}

int KernelTimer::read(spb_kernel_time* out, int cap, int* n_out) {
  std::map<std::string, spb_kernel_time> acc;
  std::vector<std::string> order;
  for (auto& r : recs_) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
      set_error("kernel timing: event query failed");
      return SPB_ERR_HIP;
    }
    auto it = acc.find(r.name);
    if (it == acc.end()) {
      spb_kernel_time t;
      std::memset(&t, 0, sizeof t);
      std::snprintf(t.name, sizeof t.name, "%s", r.name.c_str());
      it = acc.emplace(r.name, t).first;
      order.push_back(r.name);
    }
    it->second.launches += 1;
    it->second.total_ms += ms;
    it->second.flops += r.flops;
    it->second.bytes += r.bytes;
  }
  if ((int)order.size() > cap) { set_error("kernel timing: %zu records, room for %d", order.size(), cap); return SPB_ERR_INVALID_ARG; }
  for (size_t i = 0; i < order.size(); ++i) out[i] = acc[order[i]];
  *n_out = (int)order.size();
  for (auto& r : recs_) { pool_.push_back(r.start); pool_.push_back(r.stop); }
  recs_.clear();
  return SPB_OK;
}

}  // namespace spb

using spb::set_error;

#define SPB_REQUIRE(cond, code, ...) \
  do { if (!(cond)) { set_error(__VA_ARGS__); return (code); } } while (0)

static int depth_ok(const spb_model* m, int k, const char* who) {
  if (k < 0 || k > m->impl->num_units) { set_error("%s: depth %d outside 0..%d", who, k, m->impl->num_units); return SPB_ERR_DEPTH_RANGE; }
  return SPB_OK;
}

extern "C" {

const char* spb_last_error(void) { return spb::g_last_error.c_str(); }

int spb_model_create(const spb_model_desc* desc, spb_model** out) {
  SPB_REQUIRE(desc && out, SPB_ERR_INVALID_ARG, "spb_model_create: null argument");
  *out = nullptr;
  SPB_REQUIRE(desc->dtype == SPB_DTYPE_F32 || desc->dtype == SPB_DTYPE_BF16, SPB_ERR_INVALID_ARG, "spb_model_create: dtype %d", desc->dtype);
  SPB_REQUIRE(desc->batch > 0, SPB_ERR_INVALID_ARG, "spb_model_create: batch %d", desc->batch);
  std::unique_ptr<spb::Model> impl;
  switch (desc->family) {
    case SPB_FAMILY_MLP: impl = spb::make_mlp(*desc); break;
    case SPB_FAMILY_ENCODER: impl = spb::make_encoder(*desc); break;
    case SPB_FAMILY_RESNET_BASIC:
    case SPB_FAMILY_RESNET_BOTTLENECK: impl = spb::make_resnet(*desc); break;
    default:
      set_error("spb_model_create: unknown family %d", desc->family);
      return SPB_ERR_INVALID_ARG;
  }
  if (!impl) return SPB_ERR_INVALID_ARG;
  *out = new spb_model{std::move(impl)};
  return SPB_OK;
}

int spb_model_destroy(spb_model* m) {
  SPB_REQUIRE(m, SPB_ERR_INVALID_ARG, "spb_model_destroy: null model");
  delete m;
  return SPB_OK;
}

int spb_num_units(const spb_model* m, int32_t* n_units) {
  SPB_REQUIRE(m && n_units, SPB_ERR_INVALID_ARG, "spb_num_units: null argument");
  *n_units = m->impl->num_units;
  return SPB_OK;
}

int spb_param_count(const spb_model* m, int32_t* n_params) {
  SPB_REQUIRE(m && n_params, SPB_ERR_INVALID_ARG, "spb_param_count: null argument");
  *n_params = (int32_t)m->impl->params.size();
  return SPB_OK;
}

int spb_param_info(const spb_model* m, int32_t index, spb_tensor_info* out) {
  SPB_REQUIRE(m && out, SPB_ERR_INVALID_ARG, "spb_param_info: null argument");
  SPB_REQUIRE(index >= 0 && index < (int)m->impl->params.size(), SPB_ERR_INVALID_ARG, "spb_param_info: index %d outside 0..%zu", index, m->impl->params.size() - 1);
  const spb::ParamInfo& p = m->impl->params[index];
  std::memset(out, 0, sizeof *out);
  std::snprintf(out->name, sizeof out->name, "%s", p.name.c_str());
  out->unit = p.unit;
  out->dtype = p.dtype == spb::DType::F32 ? SPB_DTYPE_F32 : SPB_DTYPE_BF16;
  out->ndim = (int32_t)p.shape.size();
  for (size_t i = 0; i < p.shape.size() && i < 4; ++i) out->shape[i] = p.shape[i];
  out->numel = p.numel();
  return SPB_OK;
}

static int bind(spb_model* m, void* const* ptrs, int32_t n, bool grads) {
  const char* who = grads ? "spb_bind_grads" : "spb_bind_params";
  SPB_REQUIRE(m && ptrs, SPB_ERR_INVALID_ARG, "%s: null argument", who);
  SPB_REQUIRE(n == (int)m->impl->params.size(), SPB_ERR_INVALID_ARG, "%s: %d pointers for %zu parameters", who, n, m->impl->params.size());
  for (int i = 0; i < n; ++i) {
    SPB_REQUIRE(grads || ptrs[i], SPB_ERR_INVALID_ARG, "%s: pointer %d (%s) is null", who, i, m->impl->params[i].name.c_str());
    SPB_REQUIRE((reinterpret_cast<uintptr_t>(ptrs[i]) & 15u) == 0, SPB_ERR_INVALID_ARG, "%s: pointer %d (%s) is not 16-byte aligned", who, i, m->impl->params[i].name.c_str());
  }
  auto& dst = grads ? m->impl->grad_ptrs : m->impl->param_ptrs;
  dst.assign(ptrs, ptrs + n);
  (grads ? m->impl->grads_bound : m->impl->params_bound) = true;
  return SPB_OK;
}

int spb_bind_params(spb_model* m, void* const* ptrs, int32_t n) { return bind(m, ptrs, n, false); }
int spb_bind_grads(spb_model* m, void* const* ptrs, int32_t n) { return bind(m, ptrs, n, true); }

int spb_workspace_size(const spb_model* m, int32_t k, size_t* bytes) {
  SPB_REQUIRE(m && bytes, SPB_ERR_INVALID_ARG, "spb_workspace_size: null argument");
  if (int rc = depth_ok(m, k, "spb_workspace_size")) return rc;
  *bytes = m->impl->workspace_size(k);
  return SPB_OK;
}

int spb_forward(spb_model* m, const void* x, const int32_t* labels, const int32_t* loss_rows, int32_t k,
                void* workspace, size_t workspace_bytes, float* loss_out, void* stream) {
  SPB_REQUIRE(m, SPB_ERR_INVALID_ARG, "spb_forward: null model");
  m->impl->stashed_k = -1;
  SPB_REQUIRE(x && labels && loss_out, SPB_ERR_INVALID_ARG, "spb_forward: null input, labels or loss pointer");
  SPB_REQUIRE(!m->impl->needs_loss_rows || loss_rows, SPB_ERR_INVALID_ARG, "spb_forward: this model needs the loss_rows index array");
  SPB_REQUIRE((reinterpret_cast<uintptr_t>(x) & 15u) == 0, SPB_ERR_INVALID_ARG, "spb_forward: input is not 16-byte aligned");
  if (int rc = depth_ok(m, k, "spb_forward")) return rc;
  SPB_REQUIRE(m->impl->params_bound, SPB_ERR_STATE, "spb_forward: parameters are not bound");
  const size_t need = m->impl->workspace_size(k);
  SPB_REQUIRE(workspace && workspace_bytes >= need, SPB_ERR_WORKSPACE, "spb_forward: workspace of %zu bytes, depth %d needs %zu", workspace_bytes, k, need);
  SPB_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, SPB_ERR_WORKSPACE, "spb_forward: workspace is not 256-byte aligned");
  m->impl->ensure_side_stream(static_cast<hipStream_t>(stream));
  int rc = m->impl->forward(x, labels, loss_rows, k, workspace, loss_out, static_cast<hipStream_t>(stream));
  if (rc != SPB_OK) return rc;
  m->impl->stashed_k = k;
  m->impl->ws = workspace;
  return SPB_OK;
}

// ---- forward pass on a workspace the library holds itself ---------------------------------------------------
// For callers that may not allocate (code under stream capture, tight serving loops): the workspace is a
// file-scope device array of fixed size instead of a caller buffer, and nothing on this path allocates (no
// stream, no event, no device memory).  Every device the library runs on has its own copy of the array; its
// address on a device is looked up once, with that device current.
static __device__ __align__(256) unsigned char scratch[SPB_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of `scratch` (never the array's name: in host code that is a stand-in).
int static_workspace(void** out) {
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) {
    (void)hipGetLastError();
    set_error("spb_forward_static: cannot tell the current device");
    return SPB_ERR_HIP;
  }
  std::lock_guard<std::mutex> guard(g_scratch_lock);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      set_error("spb_forward_static: address of the static workspace on device %d: %s", device, hipGetErrorString(e));
      return SPB_ERR_HIP;
    }
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return SPB_OK;
}
}  // namespace

int spb_forward_static(spb_model* m, const void* x, const int32_t* labels, const int32_t* loss_rows, int32_t k,
                       float* loss_out, void* stream) {
  SPB_REQUIRE(m, SPB_ERR_INVALID_ARG, "spb_forward_static: null model");
  m->impl->stashed_k = -1;
  SPB_REQUIRE(x && labels && loss_out, SPB_ERR_INVALID_ARG, "spb_forward_static: null input, labels or loss pointer");
  SPB_REQUIRE(!m->impl->needs_loss_rows || loss_rows, SPB_ERR_INVALID_ARG, "spb_forward_static: this model needs the loss_rows index array");
  SPB_REQUIRE((reinterpret_cast<uintptr_t>(x) & 15u) == 0, SPB_ERR_INVALID_ARG, "spb_forward_static: input is not 16-byte aligned");
  if (int rc = depth_ok(m, k, "spb_forward_static")) return rc;
  SPB_REQUIRE(m->impl->params_bound, SPB_ERR_STATE, "spb_forward_static: parameters are not bound");
  const size_t need = m->impl->workspace_size(k);
  SPB_REQUIRE(need <= (size_t)SPB_STATIC_WORKSPACE_BYTES, SPB_ERR_WORKSPACE,
              "spb_forward_static: depth %d needs a workspace of %zu bytes, the static one holds %zu", k, need, (size_t)SPB_STATIC_WORKSPACE_BYTES);
  void* workspace = nullptr;
  if (int rc = static_workspace(&workspace)) return rc;
  // no ensure_side_stream here: creating a stream and events would allocate.  Without one (or while `stream` is
  // being captured) the backward pass keeps everything on the caller's stream.
  int rc = m->impl->forward(x, labels, loss_rows, k, workspace, loss_out, static_cast<hipStream_t>(stream));
  if (rc != SPB_OK) return rc;
  m->impl->stashed_k = k;
  m->impl->ws = workspace;
  return SPB_OK;
}

static int grads_ok(const spb_model* m, int k, const char* who) {
  const auto& im = *m->impl;
  if (k > 0 && !im.grads_bound) { set_error("%s: gradient buffers are not bound", who); return SPB_ERR_STATE; }
  for (size_t i = 0; i < im.params.size(); ++i)
    if (im.params[i].unit >= im.num_units - k && !im.grad_ptrs[i]) {
      set_error("%s: gradient buffer of %s (unit %d, above the cut at depth %d) is null", who, im.params[i].name.c_str(), im.params[i].unit, k);
      return SPB_ERR_STATE;
    }
  return SPB_OK;
}

int spb_backward_truncated(spb_model* m, int32_t k, void* stream) {
  SPB_REQUIRE(m, SPB_ERR_INVALID_ARG, "spb_backward_truncated: null model");
  if (int rc = depth_ok(m, k, "spb_backward_truncated")) return rc;
  SPB_REQUIRE(m->impl->stashed_k >= 0, SPB_ERR_STATE, "spb_backward_truncated: no forward pass has run");
  SPB_REQUIRE(k <= m->impl->stashed_k, SPB_ERR_STATE, "spb_backward_truncated: depth %d, but the forward pass stashed for depth %d", k, m->impl->stashed_k);
  if (k == 0) return SPB_OK;
  if (int rc = grads_ok(m, k, "spb_backward_truncated")) return rc;
  const int rc = m->impl->backward(k, static_cast<hipStream_t>(stream));
  const int rj = m->impl->finish(static_cast<hipStream_t>(stream));  // the caller's stream waits for the side stream's kernels
  return rc != SPB_OK ? rc : rj;
}

int spb_grad_buffers(const spb_model* m, int32_t k, spb_grad_view* out, int32_t cap, int32_t* n_out) {
  SPB_REQUIRE(m && n_out, SPB_ERR_INVALID_ARG, "spb_grad_buffers: null argument");
  if (int rc = depth_ok(m, k, "spb_grad_buffers")) return rc;
  *n_out = 0;
  if (k == 0) return SPB_OK;
  if (int rc = grads_ok(m, k, "spb_grad_buffers")) return rc;
  const auto& im = *m->impl;
  int n = 0;
  for (int u = im.num_units - 1; u >= im.num_units - k; --u)
    for (size_t i = 0; i < im.params.size(); ++i)
      if (im.params[i].unit == u) {
        SPB_REQUIRE(out && n < cap, SPB_ERR_INVALID_ARG, "spb_grad_buffers: room for %d views is not enough at depth %d", cap, k);
        out[n].param_index = (int32_t)i;
        out[n].unit = u;
        out[n].data = im.grad_ptrs[i];
        out[n].numel = im.params[i].numel();
        ++n;
      }
  *n_out = n;
  return SPB_OK;
}

int spb_unit_io(const spb_model* m, int32_t k, int32_t unit, spb_buffer_view* input, spb_buffer_view* output_grad) {
  SPB_REQUIRE(m && input && output_grad, SPB_ERR_INVALID_ARG, "spb_unit_io: null argument");
  if (int rc = depth_ok(m, k, "spb_unit_io")) return rc;
  const int L = m->impl->num_units;
  SPB_REQUIRE(unit >= L - k && unit < L, SPB_ERR_INVALID_ARG, "spb_unit_io: unit %d is not among the top %d of %d units", unit, k, L);
  m->impl->unit_io(k, unit, input, output_grad);
  return SPB_OK;
}

int spb_zero_absent_grads(spb_model* m, int32_t k, void* stream) {
  SPB_REQUIRE(m, SPB_ERR_INVALID_ARG, "spb_zero_absent_grads: null model");
  if (int rc = depth_ok(m, k, "spb_zero_absent_grads")) return rc;
  auto& im = *m->impl;
  for (size_t i = 0; i < im.params.size(); ++i)
    if (im.params[i].unit < im.num_units - k && im.grad_ptrs[i]) {
      hipError_t e = spb::launch_fill_zero(im.grad_ptrs[i], (size_t)im.params[i].numel() * 4, static_cast<hipStream_t>(stream));
      if (e != hipSuccess) { set_error("spb_zero_absent_grads: %s", hipGetErrorString(e)); return SPB_ERR_HIP; }
    }
  return SPB_OK;
}

int spb_worker_depth(const spb_model* m, int32_t j, int32_t n_workers, int32_t* k) {
  SPB_REQUIRE(m && k, SPB_ERR_INVALID_ARG, "spb_worker_depth: null argument");
  SPB_REQUIRE(n_workers >= 1 && j >= 1 && j <= n_workers, SPB_ERR_INVALID_ARG, "spb_worker_depth: worker %d outside 1..%d", j, n_workers);
  const long long L = m->impl->num_units;
  *k = (int32_t)((j * L + n_workers - 1) / n_workers);
  return SPB_OK;
}

int spb_aggregate_update(spb_model* m, int32_t n_workers, const int32_t* depths, void* const* worker_grads,
                         void* const* velocity, float lr, float momentum, float weight_decay, int32_t scale_lr,
                         void* stream) {
  SPB_REQUIRE(m && depths && worker_grads && velocity, SPB_ERR_INVALID_ARG, "spb_aggregate_update: null argument");
  SPB_REQUIRE(n_workers >= 1 && n_workers <= SPB_MAX_WORKERS, SPB_ERR_INVALID_ARG, "spb_aggregate_update: %d workers outside 1..%d", n_workers, SPB_MAX_WORKERS);
  static_assert(SPB_MAX_WORKERS == spb::kMaxAggWorkers, "worker limit");
  auto& im = *m->impl;
  for (int j = 0; j < n_workers; ++j)
    if (int rc = depth_ok(m, depths[j], "spb_aggregate_update")) return rc;
  SPB_REQUIRE(im.params_bound, SPB_ERR_STATE, "spb_aggregate_update: parameters not bound");
  const int n_params = (int)im.params.size();
  std::vector<spb::AggregateTensor> tensors;
  for (int i = 0; i < n_params; ++i) {
    spb::AggregateTensor t;
    for (int j = 0; j < n_workers; ++j) {
      if (im.params[i].unit < im.num_units - depths[j]) continue;  // worker j's suffix does not reach this unit
      const void* g = worker_grads[(size_t)j * n_params + i];
      SPB_REQUIRE(g && (reinterpret_cast<uintptr_t>(g) & 15) == 0, SPB_ERR_INVALID_ARG,
                  "spb_aggregate_update: worker %d contributes to %s but its gradient pointer is null or not 16-byte aligned", j, im.params[i].name.c_str());
      t.g[t.count++] = static_cast<const float*>(g);
    }
    if (t.count == 0) continue;  // nobody reached it: parameter and velocity stay as they are
    SPB_REQUIRE(velocity[i] && (reinterpret_cast<uintptr_t>(velocity[i]) & 15) == 0 && im.param_ptrs[i], SPB_ERR_INVALID_ARG,
                "spb_aggregate_update: velocity of %s null or not 16-byte aligned", im.params[i].name.c_str());
    t.w = im.param_ptrs[i];
    t.v = static_cast<float*>(velocity[i]);
    t.numel = im.params[i].numel();
    t.rate = scale_lr ? lr * (float)t.count / (float)n_workers : lr;
    tensors.push_back(t);
  }
  hipError_t e = spb::launch_aggregate_update(tensors.data(), (int)tensors.size(), im.dtype, momentum, weight_decay, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) { set_error("spb_aggregate_update: %s", hipGetErrorString(e)); return SPB_ERR_HIP; }
  return SPB_OK;
}

int spb_set_kernel_timing(spb_model* m, int32_t enable) {
  SPB_REQUIRE(m, SPB_ERR_INVALID_ARG, "spb_set_kernel_timing: null model");
  m->impl->timer.enable(enable != 0);
  return SPB_OK;
}

int spb_replay_kernel(spb_model* m, const char* name, int32_t count, void* stream) {
  SPB_REQUIRE(m && name && count > 0, SPB_ERR_INVALID_ARG, "spb_replay_kernel: null argument or non-positive count");
  return m->impl->replay(name, count, static_cast<hipStream_t>(stream));
}

int spb_read_kernel_timing(spb_model* m, spb_kernel_time* out, int32_t cap, int32_t* n_out) {
  SPB_REQUIRE(m && out && n_out && cap > 0, SPB_ERR_INVALID_ARG, "spb_read_kernel_timing: null argument");
  return m->impl->timer.read(out, cap, n_out);
}

}  // extern "C"
