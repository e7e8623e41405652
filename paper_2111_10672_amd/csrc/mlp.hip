// Perceptron family: unit u is Linear dims[u] -> dims[u+1] (+ReLU, except the last, which carries the
// softmax cross-entropy).  Forward pass, stash plan and truncated backward pass (Sec. 1-2 of the paper).
//
// Activation a_0 is the caller's input; a_{u+1} = relu(a_u W_u^T + b_u).  The backward pass of unit u
// reads a_u (weight gradient) and the sign of a_{u+1} (ReLU mask, applied in the epilogue of unit
// u+1's input-gradient product), so a depth-k step keeps a_{L-k} .. a_{L-1} and nothing below.
#include "model.h"

namespace spb {
namespace {

class MlpModel : public Model {
 public:
  explicit MlpModel(const spb_model_desc& d) {
    dtype = d.dtype == SPB_DTYPE_F32 ? DType::F32 : DType::BF16;
    batch_ = d.batch;
    dims_.assign(d.dims, d.dims + d.n_dims);
    num_units = d.n_dims - 1;
    per_ = dtype == DType::F32 ? 4 : 8;
    for (int u = 0; u < num_units; ++u) {
      ParamInfo w, b;
      w.name = "fc" + std::to_string(u) + ".weight"; w.unit = u; w.dtype = dtype; w.shape = {dims_[u + 1], dims_[u]};
      b.name = "fc" + std::to_string(u) + ".bias"; b.unit = u; b.dtype = dtype; b.shape = {dims_[u + 1]};
      params.push_back(w);
      params.push_back(b);
    }
    param_ptrs.assign(params.size(), nullptr);
    grad_ptrs.assign(params.size(), nullptr);
  }

  // pitch (elements) of activation l, l >= 1: whole 16-byte chunks
  int ld(int l) const { return (int)align_up((size_t)dims_[l], (size_t)per_); }
  size_t act_bytes(int l) const { return align_up((size_t)batch_ * ld(l) * dtype_size(dtype), 256); }
  size_t max_hidden_bytes() const {
    size_t m = 0;
    for (int l = 1; l < num_units; ++l) m = std::max(m, act_bytes(l));
    return m;
  }
  int classes() const { return (int)dims_[num_units]; }
  int ldz() const { return (int)align_up((size_t)classes(), 4); }

  struct Plan {
    std::vector<size_t> act;     // offset of a_l, l = 1..L-1 (index l); SIZE_MAX = ping-pong
    size_t pingpong[2], logits, row_loss, dlogits, dz[2], total;
  };

  Plan plan(int k) const {
    Plan p;
    const int L = num_units;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    const size_t hid = max_hidden_bytes();
    p.pingpong[0] = take(hid);
    p.pingpong[1] = take(hid);
    p.act.assign(L + 1, SIZE_MAX);
    for (int l = std::max(1, L - k); l <= L - 1; ++l) p.act[l] = take(act_bytes(l));
    p.logits = take((size_t)batch_ * ldz() * 4);
    p.row_loss = take((size_t)batch_ * 4);
    p.dlogits = take((size_t)batch_ * ld(L) * dtype_size(dtype));
    p.dz[0] = p.dz[1] = 0;
    if (k >= 2) { p.dz[0] = take(hid); p.dz[1] = take(hid); }
    p.total = off;
    return p;
  }

  size_t workspace_size(int k) const override { return plan(k).total; }

  int forward(const void* x, const int32_t* labels, const int32_t*, int k, void* wsp, float* loss_out, hipStream_t s) override {
    const int L = num_units;
    const Plan p = plan(k);
    char* base = static_cast<char*>(wsp);
    const void* in = x;
    int ld_in = (int)dims_[0];
    for (int u = 0; u < L; ++u) {
      GemmProblem g;
      g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::RowK;
      g.M = batch_; g.N = (int)dims_[u + 1]; g.K = (int)dims_[u];
      g.A = in; g.lda = ld_in;
      g.B = param_ptrs[2 * u]; g.ldb = (int)dims_[u];
      g.bias = param_ptrs[2 * u + 1];
      if (u < L - 1) {
        const size_t o = p.act[u + 1] != SIZE_MAX ? p.act[u + 1] : p.pingpong[u & 1];
        g.C = base + o; g.ldc = ld(u + 1);
        g.epilogue = Epilogue::BiasAct; g.relu = 1;
        g.name = dtype == DType::F32 ? "gemm_f32_fwd" : "gemm_bf16_fwd";
      } else {
        g.C = base + p.logits; g.ldc = ldz();
        g.epilogue = Epilogue::StoreF32;
        g.name = dtype == DType::F32 ? "gemm_f32_fwd_logits" : "gemm_bf16_fwd_logits";
      }
      if (int rc = gemm(g, s)) return rc;
      in = g.C; ld_in = g.ldc;
    }
    const int C = classes();
    const double bytes = (double)batch_ * C * (4.0 + dtype_size(dtype));
    hipError_t e = timer.run("softmax_xent", 0.0, bytes, s, [&] {
      return launch_softmax_xent(reinterpret_cast<const float*>(base + p.logits), ldz(), labels, batch_, C,
                                 base + p.dlogits, ld(L), dtype, reinterpret_cast<float*>(base + p.row_loss), loss_out, s);
    });
    if (int rc = check(e, "softmax cross-entropy")) return rc;
    x_ = x;
    return SPB_OK;
  }

  int backward(int k, hipStream_t s) override {
    const int L = num_units;
    const Plan p = plan(stashed_k);
    char* base = static_cast<char*>(ws);
    const void* dz = base + p.dlogits;
    int ld_dz = ld(L);
    for (int u = L - 1; u >= L - k; --u) {
      const void* a_u = u == 0 ? x_ : base + p.act[u];
      const int ld_a = u == 0 ? (int)dims_[0] : ld(u);
      const int n_out = (int)dims_[u + 1], n_in = (int)dims_[u];
      GemmProblem w;  // dW[n, i] = sum_b dz[b, n] * a_u[b, i];  db[n] = sum_b dz[b, n]
      w.dtype = dtype; w.a_layout = Layout::KRow; w.b_layout = Layout::KRow;
      w.M = n_out; w.N = n_in; w.K = batch_;
      w.A = dz; w.lda = ld_dz; w.B = a_u; w.ldb = ld_a;
      w.C = grad_ptrs[2 * u]; w.ldc = n_in; w.epilogue = Epilogue::StoreF32;
      w.a_row_sum = static_cast<float*>(grad_ptrs[2 * u + 1]);
      w.a_pad_zero = w.b_pad_zero = true;  // dz: padding zeroed by its producer; activations have none
      w.name = dtype == DType::F32 ? "gemm_f32_wgrad" : "gemm_bf16_wgrad";
      if (u == L - k) {  // lowest visited unit: no input gradient (nothing below consumes it)
        if (int rc = gemm(w, s)) return rc;
        break;
      }
      GemmProblem d;  // dz_{u-1}[b, i] = (sum_n dz[b, n] * W_u[n, i]) * [a_u[b, i] > 0]
      d.dtype = dtype; d.a_layout = Layout::RowK; d.b_layout = Layout::KRow;
      d.M = batch_; d.N = n_in; d.K = n_out;
      d.A = dz; d.lda = ld_dz; d.B = param_ptrs[2 * u]; d.ldb = n_in;
      d.C = base + p.dz[u & 1]; d.ldc = ld(u);
      d.epilogue = Epilogue::MaskStore; d.mask = a_u; d.ldmask = ld_a;
      d.a_pad_zero = d.b_pad_zero = true;
      d.name = dtype == DType::F32 ? "gemm_f32_dgrad" : "gemm_bf16_dgrad";
      if (int rc = gemm_pair(d, w, s)) return rc;  // independent of each other: one launch where both are small
      dz = d.C; ld_dz = d.ldc;
    }
    return SPB_OK;
  }

  void unit_io(int k, int unit, spb_buffer_view* input, spb_buffer_view* output_grad) const override {
    const int L = num_units;
    const Plan p = plan(k);
    // a_unit, the unit's input; unit 0 reads the caller's x
    *input = unit == 0 ? make_view(SPB_VIEW_CALLER_INPUT, batch_, dims_[0], dims_[0], dtype)
                       : make_view((long long)p.act[unit], batch_, dims_[unit], ld(unit), dtype);
    // the input gradient of unit + 1 with the ReLU of this unit fused in: the gradient at this unit's pre-activation
    *output_grad = (unit == L - 1 || k < 2) ? no_view() : make_view((long long)p.dz[(unit + 1) & 1], batch_, dims_[unit + 1], ld(unit + 1), dtype, 1);
  }

 private:
  int batch_ = 0, per_ = 8;
  std::vector<int64_t> dims_;
  const void* x_ = nullptr;
};

}  // namespace

std::unique_ptr<Model> make_mlp(const spb_model_desc& d) {
  if (d.n_dims < 2 || d.n_dims > SPB_MAX_DIMS) { set_error("mlp: n_dims %d outside 2..%d", d.n_dims, SPB_MAX_DIMS); return nullptr; }
  const int per = d.dtype == SPB_DTYPE_F32 ? 4 : 8;
  for (int i = 0; i < d.n_dims; ++i) {
    if (d.dims[i] <= 0) { set_error("mlp: dims[%d] = %d is not positive", i, d.dims[i]); return nullptr; }
    if (i < d.n_dims - 1 && d.dims[i] % per) {
      set_error("mlp: dims[%d] = %d is not a whole number of 16-byte chunks (multiple of %d)", i, d.dims[i], per);
      return nullptr;
    }
  }
  return std::make_unique<MlpModel>(d);
}

}  // namespace spb
