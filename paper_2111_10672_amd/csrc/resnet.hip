// Residual-CNN families: units = stem | residual blocks (basic or bottleneck) | pooled classifier.
// Forward pass, stash plan and truncated backward pass (Sec. 1-2 of the paper; ResNets are the paper's own
// workloads, Tables 1-2).
//
// Every convolution is an implicit GEMM on the MFMA kernel of gemm_dma.hip, activations NHWC, weights
// [Cout, R, S, Cin]:
//   forward          out[pixel, co]  = sum_{tap, ci} x[pixel + tap][ci] * w[co][tap][ci]       rows gathered from x
//   input gradient   dx[pixel, ci]   = sum_{tap, co} dy[(pixel - tap) / stride][co] * w[co][tap][ci]
//   weight gradient  dw[co][tap][ci] = sum_pixel dy[pixel][co] * x[pixel + tap][ci]            k cut into slices
// The per-channel affine that follows each convolution (a BatchNorm folded to scale and shift, kept
// trainable), the ReLU and the residual add ride in the forward product's epilogue, which also writes the
// pre-affine output a unit above the cut keeps for the scale gradient.  Backward, one memory-bound kernel per
// convolution turns the incoming gradient into dy and the scale/shift gradients; the shortcut's gradient
// joins in the epilogue of the block's first input-gradient product.
#include <algorithm>
#include <cmath>

#include "model.h"

namespace spb {
namespace {

struct Conv {
  int cin = 0, cout = 0, k = 1, stride = 1, pad = 0;
  int in_h = 0, in_w = 0, out_h = 0, out_w = 0;
  int cin_eff = 0;               // cin rounded up to 8 (only the stem's 3-channel input differs)
  int w = -1, scale = -1, shift = -1;  // parameter indices
  long long in_rows(int batch) const { return (long long)batch * in_h * in_w; }
  long long out_rows(int batch) const { return (long long)batch * out_h * out_w; }
  int k_total() const { return k * k * cin_eff; }
};

struct Block {
  std::vector<Conv> convs;  // main path
  bool has_proj = false;
  Conv proj;
};

// Offsets of one unit's tensors in the workspace.
struct ConvBuf { size_t y = 0, a = 0; };   // pre-affine output (kept only above the cut), post-activation output
struct UnitBuf {
  std::vector<ConvBuf> conv;    // main-path convolutions; the last one's `a` is the unit's output
  ConvBuf proj;                 // projection shortcut: y = pre-affine, a = its affine output
  size_t xpad = 0, wpad = 0, pool_out = 0, which = 0;  // stem only
  size_t out = 0;               // the unit's output tensor
};

class ResnetModel : public Model {
 public:
  explicit ResnetModel(const spb_model_desc& d) {
    dtype = DType::BF16;
    batch_ = d.batch;
    classes_ = d.classes;
    const bool bottleneck = d.family == SPB_FAMILY_RESNET_BOTTLENECK;
    auto add = [&](const std::string& name, int unit, std::vector<int64_t> shape) {
      ParamInfo p; p.name = name; p.unit = unit; p.dtype = dtype; p.shape = std::move(shape); params.push_back(p);
      return (int)params.size() - 1;
    };
    auto make_conv = [&](const std::string& conv_name, const std::string& aff_name, int unit, int cin, int cout, int k, int stride, int pad, int h, int w) {
      Conv c;
      c.cin = cin; c.cout = cout; c.k = k; c.stride = stride; c.pad = pad; c.in_h = h; c.in_w = w;
      c.out_h = (h + 2 * pad - k) / stride + 1; c.out_w = (w + 2 * pad - k) / stride + 1;
      c.cin_eff = (cin + 7) / 8 * 8;
      c.w = add(conv_name + ".weight", unit, {cout, k, k, cin});
      c.scale = add(aff_name + ".scale", unit, {cout});
      c.shift = add(aff_name + ".shift", unit, {cout});
      return c;
    };
    stem_ = make_conv("stem.conv", "stem.aff", 0, d.image_c, d.stem_width, d.stem_kernel, d.stem_stride, d.stem_pad, d.image_h, d.image_w);
    pool_ = d.stem_pool != 0;
    int h = stem_.out_h, w = stem_.out_w, cin = d.stem_width;
    if (pool_) { h = (h - 1) / 2 + 1; w = (w - 1) / 2 + 1; }
    pool_h_ = h; pool_w_ = w;
    for (int stage = 0; stage < d.n_stages; ++stage)
      for (int j = 0; j < d.stage_blocks[stage]; ++j) {
        const int width = d.stage_widths[stage], stride = (stage > 0 && j == 0) ? 2 : 1, unit = (int)blocks_.size() + 1;
        const std::string pre = "block" + std::to_string(blocks_.size()) + ".";
        Block b;
        if (bottleneck) {
          const int mid = width / 4;
          b.convs.push_back(make_conv(pre + "conv1", pre + "aff1", unit, cin, mid, 1, 1, 0, h, w));
          b.convs.push_back(make_conv(pre + "conv2", pre + "aff2", unit, mid, mid, 3, stride, 1, h, w));
          b.convs.push_back(make_conv(pre + "conv3", pre + "aff3", unit, mid, width, 1, 1, 0, b.convs[1].out_h, b.convs[1].out_w));
        } else {
          b.convs.push_back(make_conv(pre + "conv1", pre + "aff1", unit, cin, width, 3, stride, 1, h, w));
          b.convs.push_back(make_conv(pre + "conv2", pre + "aff2", unit, width, width, 3, 1, 1, b.convs[0].out_h, b.convs[0].out_w));
        }
        b.has_proj = stride != 1 || cin != width;
        if (b.has_proj) b.proj = make_conv(pre + "proj", pre + "projaff", unit, cin, width, 1, stride, 0, h, w);
        h = b.convs.back().out_h; w = b.convs.back().out_w; cin = width;
        blocks_.push_back(b);
      }
    final_h_ = h; final_w_ = w; features_ = cin;
    num_units = (int)blocks_.size() + 2;
    fc_w_ = add("head.fc.weight", num_units - 1, {classes_, features_});
    fc_b_ = add("head.fc.bias", num_units - 1, {classes_});
    param_ptrs.assign(params.size(), nullptr);
    grad_ptrs.assign(params.size(), nullptr);
  }

  bool shapes_ok(std::string* why) const {
    auto conv_ok = [&](const Conv& c, bool first) {
      if ((c.cout % 8) || c.cout > 2048) { *why = "channel counts must be multiples of 8 and at most 2048"; return false; }
      if (!first && c.cin % 8) { *why = "channel counts must be multiples of 8"; return false; }
      if (c.out_h <= 0 || c.out_w <= 0 || (long long)c.out_h * c.out_w > 65535 || (long long)c.in_h * c.in_w > 65535) { *why = "feature maps must have 1..65535 pixels"; return false; }
      if (c.k * c.k > 255 || (c.stride != 1 && c.stride != 2)) { *why = "kernel up to 15x15, stride 1 or 2"; return false; }
      return true;
    };
    if (!conv_ok(stem_, true)) return false;
    for (const Block& b : blocks_) {
      for (const Conv& c : b.convs) if (!conv_ok(c, false)) return false;
      if (b.has_proj && !conv_ok(b.proj, false)) return false;
    }
    return true;
  }

  // ---- workspace plan ----------------------------------------------------------------------------
  struct Plan {
    std::vector<UnitBuf> unit;   // stem, blocks
    size_t pooled, logits, row_loss, dlogits, dpooled;
    // backward transients, gradients of activations: 0, 1 the gradient handed from unit to unit where it is stored
    // unmasked (the top unit's, the stem's), 2 a convolution's input gradient on its way to an unfused affine pass,
    // 3 the projection's input gradient; then three sets (units i % 3) of: dy (three in rotation), the projection's
    // dy, and the unit's masked output gradient (what its shortcut carries)
    static constexpr int kSets = 3, kSetBase = 4, kPerSet = 5;
    size_t g[kSetBase + kSets * kPerSet];
    static constexpr int kReduceSlots = 4;   // a unit has at most three convolutions and a projection
    size_t affine_partial[kSets][kReduceSlots], wgrad_partial[kSets][kReduceSlots];   // per set of units
    size_t total;
  };
  static constexpr int kFwdPool = 8;

  size_t act_bytes(long long rows, int c) const { return (size_t)rows * c * 2; }
  size_t max_act_bytes() const {
    size_t m = act_bytes(stem_.in_rows(batch_), stem_.cin_eff);
    auto see = [&](const Conv& c) { m = std::max(m, act_bytes(c.out_rows(batch_), c.cout)); };
    see(stem_);
    for (const Block& b : blocks_) { for (const Conv& c : b.convs) see(c); if (b.has_proj) see(b.proj); }
    return m;
  }
  int wgrad_splits(const Conv& c) const {
    const long tiles = (long)((c.cout + 127) / 128) * ((c.k_total() + 127) / 128);
    const long k_tiles = (long)((c.out_rows(batch_) + 63) / 64);
    // k-slices for about 192 workgroups, not one per CU: the weight gradients run beside the input-gradient chain of the
    // other stream, and a quarter of the CUs left to that chain measured best on the step (128: -0.6 %, 256: -1.1 to
    // -1.8 %, 512: -3.5 to -8 %)
    long s = (192 + tiles - 1) / tiles;
    s = std::min(s, std::max(1L, k_tiles / 4));
    return (int)std::max(1L, std::min(s, 1024L));
  }

  Plan plan(int k) const {
    Plan p;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    const int cut = num_units - k;
    const size_t amax = max_act_bytes();
    size_t pool[kFwdPool];
    for (auto& b : pool) b = take(amax);
    int next = 0;
    auto transient = [&]() { size_t o = pool[next]; next = (next + 1) % kFwdPool; return o; };
    p.unit.resize(blocks_.size() + 1);
    // A unit's tensors are kept when the unit is above the cut; its output also when the next unit is.
    {
      UnitBuf& u = p.unit[0];
      const bool keep = 0 >= cut, keep_out = keep || 1 >= cut;
      u.conv.resize(1);
      u.xpad = stem_.cin_eff != stem_.cin ? (keep ? take(act_bytes(stem_.in_rows(batch_), stem_.cin_eff)) : transient()) : 0;
      u.wpad = take((size_t)stem_.cout * stem_.k * stem_.k * stem_.cin_eff * 2);
      u.conv[0].y = keep ? take(act_bytes(stem_.out_rows(batch_), stem_.cout)) : 0;
      const size_t a_bytes = act_bytes(stem_.out_rows(batch_), stem_.cout);
      if (pool_) {
        u.conv[0].a = keep ? take(a_bytes) : transient();
        u.pool_out = keep_out ? take(act_bytes((long long)batch_ * pool_h_ * pool_w_, stem_.cout)) : transient();
        u.which = keep ? take((size_t)batch_ * pool_h_ * pool_w_ * stem_.cout) : 0;
        u.out = u.pool_out;
      } else {
        u.conv[0].a = keep_out ? take(a_bytes) : transient();
        u.out = u.conv[0].a;
      }
    }
    for (size_t i = 0; i < blocks_.size(); ++i) {
      const Block& b = blocks_[i];
      UnitBuf& u = p.unit[i + 1];
      const int unit = (int)i + 1;
      const bool keep = unit >= cut, keep_out = keep || unit + 1 >= cut;
      u.conv.resize(b.convs.size());
      if (b.has_proj) {
        u.proj.y = keep ? take(act_bytes(b.proj.out_rows(batch_), b.proj.cout)) : 0;
        u.proj.a = transient();   // only the forward pass reads the shortcut's output
      }
      for (size_t j = 0; j < b.convs.size(); ++j) {
        const Conv& c = b.convs[j];
        const size_t bytes = act_bytes(c.out_rows(batch_), c.cout);
        const bool last = j + 1 == b.convs.size();
        u.conv[j].y = keep ? take(bytes) : 0;
        u.conv[j].a = (last ? keep_out : keep) ? take(bytes) : transient();
      }
      u.out = u.conv.back().a;
    }
    p.pooled = take((size_t)batch_ * features_ * 2);
    p.logits = take((size_t)batch_ * align_up((size_t)classes_, 4) * 4);
    p.row_loss = take((size_t)batch_ * 4);
    p.dlogits = take((size_t)batch_ * align_up((size_t)classes_, 8) * 2);
    p.dpooled = take((size_t)batch_ * features_ * 2);
    for (auto& g : p.g) g = 0;
    for (int h = 0; h < Plan::kSets; ++h)
      for (int j = 0; j < Plan::kReduceSlots; ++j) p.affine_partial[h][j] = p.wgrad_partial[h][j] = 0;
    if (k >= 2) {
      for (auto& g : p.g) g = take(amax);
      size_t ap = 0, wp = 0;
      auto see = [&](const Conv& c) {
        ap = std::max(ap, affine_partial_floats(c.out_rows(batch_), c.cout) * 4);
        ap = std::max(ap, (size_t)((c.out_rows(batch_) + 63) / 64) * 2 * c.cout * 4);   // the fused form: one row of sums per tile row
        wp = std::max(wp, (size_t)wgrad_splits(c) * c.cout * c.k_total() * 4);
      };
      see(stem_);
      for (const Block& b : blocks_) { for (const Conv& c : b.convs) see(c); if (b.has_proj) see(b.proj); }
      // one buffer of each kind per convolution of a unit: their reductions wait for the unit's end (see backward)
      for (int h = 0; h < Plan::kSets; ++h)
        for (int j = 0; j < Plan::kReduceSlots; ++j) { p.affine_partial[h][j] = take(ap); p.wgrad_partial[h][j] = take(wp); }
    }
    p.total = off;
    return p;
  }

  size_t workspace_size(int k) const override { return plan(k).total; }

  // ---- products ----------------------------------------------------------------------------------
  ConvGeom geom(const Conv& c) const {
    ConvGeom g;
    g.n = batch_; g.sh = c.in_h; g.sw = c.in_w; g.sc = c.cin_eff; g.rh = c.out_h; g.rw = c.out_w;
    g.r = c.k; g.s = c.k; g.stride = c.stride; g.pad = c.pad; g.transposed = 0;
    return g;
  }

  // A 1x1 convolution with stride 1 is a plain matrix product over the pixel rows: no gather at all.
  static bool pointwise(const Conv& c) { return c.k == 1 && c.stride == 1 && c.pad == 0 && c.cin_eff == c.cin; }

  // out = act(scale * conv(x, w) + shift + residual); y_keep (optional) receives the pre-affine output
  int conv_forward(const Conv& c, const void* x, const void* w, void* y_keep, const void* residual, bool relu, void* out, hipStream_t s) {
    GemmProblem g;
    g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::RowK; g.epilogue = Epilogue::BiasAct;
    if (!pointwise(c)) { g.a_gather = Gather::ConvRows; g.conv = geom(c); }
    g.M = (int)c.out_rows(batch_); g.N = c.cout; g.K = c.k_total();
    g.A = x; g.lda = g.K; g.B = w; g.ldb = g.K; g.C = out; g.ldc = c.cout;
    g.col_scale = param_ptrs[c.scale]; g.bias = param_ptrs[c.shift];
    g.aux_out = y_keep; g.ldaux = c.cout; g.aux_raw = 1;
    g.residual = residual; g.ldres = c.cout;
    g.act = relu ? Act::Relu : Act::None;
    g.name = "conv_fwd";
    return gemm(g, s);
  }
  // dx = conv_transpose(dy, w) + residual
  int conv_dgrad(const Conv& c, const void* dy, const void* w, const void* residual, void* dx, hipStream_t s) {
    GemmProblem g;
    g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::KRow; g.epilogue = Epilogue::BiasAct;
    if (!pointwise(c)) {
      g.a_gather = Gather::ConvRows; g.b_gather = Gather::ConvWeightT;
      g.conv.n = batch_; g.conv.sh = c.out_h; g.conv.sw = c.out_w; g.conv.sc = c.cout; g.conv.rh = c.in_h; g.conv.rw = c.in_w;
      g.conv.r = c.k; g.conv.s = c.k; g.conv.stride = c.stride; g.conv.pad = c.pad; g.conv.transposed = 1;
      g.conv.w_cin = c.cin_eff; g.conv.w_cout = c.cout;
    }
    g.M = (int)c.in_rows(batch_); g.N = c.cin_eff; g.K = c.k * c.k * c.cout;
    g.A = dy; g.lda = g.K; g.B = w; g.ldb = c.cin_eff; g.C = dx; g.ldc = c.cin_eff;
    g.residual = residual; g.ldres = c.cin_eff;
    g.name = "conv_dgrad";
    return gemm(g, s);
  }
  // Whether unit i + 1's (block i's) last input-gradient product also does the affine pass at the output of the unit
  // below: the tensor shapes must chain and the columns must be whole 16-byte pieces.
  bool fuses_into_unit_below(int i) const {
    if (i < 1) return false;   // below the first block lies the stem (and possibly a pooling layer)
    const Conv& c = blocks_[i].convs[0];
    const Conv& below = blocks_[i - 1].convs.back();
    return c.cin_eff == below.cout && c.cin_eff % 8 == 0 && c.in_rows(batch_) == below.out_rows(batch_);
  }
  // The input-gradient product of convolution c with the backward pass of the affine + ReLU below it (`below`, whose
  // output `act` is c's input and whose input is `y`) in its epilogue: dy_below = scale * (dx * [act > 0]) and the
  // column sums for dscale, dshift, without the gradient dx ever being written.  Returns 1 if the product cannot
  // take that epilogue (the caller then runs the two passes), 0 or an error code otherwise.
  // With `residual` (a second gradient of the same tensor: the shortcut's) the sum of the two is what the ReLU masks,
  // and dz_out (optional) receives that masked sum: the form for a unit's LAST input gradient, which then also does
  // the affine pass at the output of the unit below.
  int conv_dgrad_affine(const Conv& c, const void* dy, const void* w, const Conv& below, const void* act, const void* y, void* dy_below,
                        float* partial, hipStream_t s, const void* residual = nullptr, void* dz_out = nullptr) {
    GemmProblem g;
    g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::KRow; g.epilogue = Epilogue::AffineBwdStore;
    if (!pointwise(c)) {
      g.a_gather = Gather::ConvRows; g.b_gather = Gather::ConvWeightT;
      g.conv.n = batch_; g.conv.sh = c.out_h; g.conv.sw = c.out_w; g.conv.sc = c.cout; g.conv.rh = c.in_h; g.conv.rw = c.in_w;
      g.conv.r = c.k; g.conv.s = c.k; g.conv.stride = c.stride; g.conv.pad = c.pad; g.conv.transposed = 1;
      g.conv.w_cin = c.cin_eff; g.conv.w_cout = c.cout;
    }
    g.M = (int)c.in_rows(batch_); g.N = c.cin_eff; g.K = c.k * c.k * c.cout;
    g.A = dy; g.lda = g.K; g.B = w; g.ldb = c.cin_eff; g.C = dy_below; g.ldc = c.cin_eff;
    g.mask = act; g.ldmask = c.cin_eff; g.affine_y = y; g.ldaffine_y = c.cin_eff; g.col_scale = param_ptrs[below.scale];
    g.col_partial = partial;
    g.residual = residual; g.ldres = c.cin_eff; g.aux_out = dz_out; g.ldaux = c.cin_eff;
    g.col_partial_rows = &fused_tile_rows_;   // (a member: the product may be replayed later from its recorded description)
    g.name = "conv_dgrad_affine";
    if (c.cin_eff != below.cout || !gemm_dma_accepts(g)) return 1;
    if (int rc = gemm(g, s)) return rc;
    ReduceTask task;
    const int tile_rows = fused_tile_rows_;
    task.kind = ReduceTask::kPairs; task.partial = partial; task.count = tile_rows; task.width = below.cout;
    task.out = static_cast<float*>(grad_ptrs[below.scale]); task.out_b = static_cast<float*>(grad_ptrs[below.shift]);
    task.blocks = reduce_pairs_blocks(below.cout);
    reduce_bytes_ += (double)tile_rows * 2 * below.cout * 4;
    reduces_.push_back(task);
    return SPB_OK;
  }
  // dw = sum over pixels of dy (x) x-patch, as k-slices added up in a fixed order
  int conv_wgrad(const Conv& c, const void* x, const void* dy, float* partial, float* dw, hipStream_t s) {
    GemmProblem g;
    g.dtype = dtype; g.a_layout = Layout::KRow; g.b_layout = Layout::KRow; g.epilogue = Epilogue::StoreF32;
    if (!pointwise(c)) { g.b_gather = Gather::ConvPatchT; g.conv = geom(c); }
    g.M = c.cout; g.N = c.k_total(); g.K = (int)c.out_rows(batch_);
    g.A = dy; g.lda = c.cout; g.B = x; g.ldb = g.N; g.C = partial; g.ldc = g.N;
    g.k_splits = wgrad_splits(c);
    g.name = "conv_wgrad";
    if (int rc = gemm(g, s)) return rc;
    const long long numel = (long long)c.cout * c.k * c.k * c.cin;
    ReduceTask task;   // the k-slices are added up with the unit's other small reductions
    if (!make_splitk_reduce_task(partial, g.k_splits, (long long)c.cout * g.N, dw, numel, c.cin, c.cin_eff, &task)) return check(hipErrorInvalidValue, "weight-gradient reduction");
    reduce_bytes_ += (double)(g.k_splits + 1) * numel * 4;
    reduces_.push_back(task);
    return SPB_OK;
  }
  // gradient at the affine's output -> dy, dscale, dshift (and the masked gradient itself, if asked for)
  int affine_bwd(const Conv& c, const void* dout, const void* act, const void* y, void* dy, void* dsum, float* partial, hipStream_t s) {
    const long long rows = c.out_rows(batch_);
    ReduceTask task;
    if (int rc = run("affine_relu_bwd", (double)rows * c.cout * 2 * (3 + (act ? 1 : 0) + (dsum ? 1 : 0)), s, [&] {
          return launch_affine_relu_bwd(dout, act, y, param_ptrs[c.scale], dy, dsum, partial, static_cast<float*>(grad_ptrs[c.scale]),
                                        static_cast<float*>(grad_ptrs[c.shift]), rows, c.cout, s, &task); })) return rc;
    reduce_bytes_ += (double)task.count * 2 * c.cout * 4;
    reduces_.push_back(task);
    return SPB_OK;
  }
  // The small reductions a unit's backward pass has collected (column sums of its affine passes, k-slices of its
  // weight gradients), in one launch.  They finish parameter gradients only, so they go where weight gradients go.
  int flush_reduces(hipStream_t to) {
    if (reduces_.empty()) return SPB_OK;
    const int rc = run("unit_reduce", reduce_bytes_, to, [&] { return launch_unit_reduce(reduces_.data(), (int)reduces_.size(), to); });
    reduces_.clear();
    reduce_bytes_ = 0.0;
    return rc;
  }

  int forward(const void* x, const int32_t* labels, const int32_t*, int k, void* wsp, float* loss_out, hipStream_t s) override {
    const Plan p = plan(k);
    char* w = static_cast<char*>(wsp);
    const int cut = num_units - k;
    auto keep_ptr = [&](bool keep, size_t off) -> void* { return keep ? w + off : nullptr; };
    // ---- stem ----
    const UnitBuf& su = p.unit[0];
    const void* stem_in = x;
    const void* stem_w = param_ptrs[stem_.w];
    if (stem_.cin_eff != stem_.cin) {
      if (int rc = run("pad_channels", (double)stem_.in_rows(batch_) * (stem_.cin + stem_.cin_eff) * 2, s, [&] {
            return launch_pad_channels(x, w + su.xpad, stem_.in_rows(batch_), stem_.cin, stem_.cin_eff, s); })) return rc;
      if (int rc = run("pad_channels", 0.0, s, [&] {
            return launch_pad_channels(param_ptrs[stem_.w], w + su.wpad, (long long)stem_.cout * stem_.k * stem_.k, stem_.cin, stem_.cin_eff, s); })) return rc;
      stem_in = w + su.xpad; stem_w = w + su.wpad;
    }
    x_ = stem_in == x ? x : nullptr;
    if (int rc = conv_forward(stem_, stem_in, stem_w, keep_ptr(0 >= cut, su.conv[0].y), nullptr, true, w + su.conv[0].a, s)) return rc;
    if (pool_) {
      if (int rc = run("maxpool_fwd", (double)stem_.out_rows(batch_) * stem_.cout * 2 * 1.25, s, [&] {
            return launch_maxpool_fwd(w + su.conv[0].a, w + su.pool_out, 0 >= cut ? reinterpret_cast<uint8_t*>(w + su.which) : nullptr,
                                      batch_, stem_.out_h, stem_.out_w, stem_.cout, s); })) return rc;
    }
    const void* cur = w + su.out;
    // ---- residual blocks ----
    for (size_t i = 0; i < blocks_.size(); ++i) {
      const Block& b = blocks_[i];
      const UnitBuf& u = p.unit[i + 1];
      const bool keep = (int)i + 1 >= cut;
      const void* shortcut = cur;
      if (b.has_proj) {
        if (int rc = conv_forward(b.proj, cur, param_ptrs[b.proj.w], keep_ptr(keep, u.proj.y), nullptr, false, w + u.proj.a, s)) return rc;
        shortcut = w + u.proj.a;
      }
      const void* h = cur;
      for (size_t j = 0; j < b.convs.size(); ++j) {
        const bool last = j + 1 == b.convs.size();
        if (int rc = conv_forward(b.convs[j], h, param_ptrs[b.convs[j].w], keep_ptr(keep, u.conv[j].y), last ? shortcut : nullptr, true,
                                  w + u.conv[j].a, s)) return rc;
        h = w + u.conv[j].a;
      }
      cur = h;
    }
    // ---- head ----
    const int hw = final_h_ * final_w_;
    if (int rc = run("avgpool_fwd", (double)batch_ * hw * features_ * 2, s, [&] { return launch_avgpool_fwd(cur, w + p.pooled, batch_, hw, features_, s); })) return rc;
    const int ldz = (int)align_up((size_t)classes_, 4), lddz = (int)align_up((size_t)classes_, 8);
    {
      GemmProblem g;
      g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::RowK; g.epilogue = Epilogue::StoreF32;
      g.M = batch_; g.N = classes_; g.K = features_; g.A = w + p.pooled; g.lda = features_; g.B = param_ptrs[fc_w_]; g.ldb = features_;
      g.bias = param_ptrs[fc_b_]; g.C = w + p.logits; g.ldc = ldz; g.name = "gemm_bf16_fwd_logits";
      if (int rc = gemm(g, s)) return rc;
    }
    return run("softmax_xent", (double)batch_ * classes_ * 6, s, [&] {
      return launch_softmax_xent(reinterpret_cast<const float*>(w + p.logits), ldz, labels, batch_, classes_, w + p.dlogits, lddz, dtype,
                                 reinterpret_cast<float*>(w + p.row_loss), loss_out, s); });
  }

  int backward(int k, hipStream_t s) override {
    const Plan p = plan(stashed_k);
    char* w = static_cast<char*>(ws);
    const int cut = num_units - k;
    const int lddz = (int)align_up((size_t)classes_, 8), hw = final_h_ * final_w_;
    // partial-sum buffers of a unit's convolutions: slot j for convolution j, the last slot for the projection
    int set = 0;   // which set of the buffers the second stream reads the unit at hand uses: unit i uses set i % 3
    auto apart_of = [&](int st, int j) { return reinterpret_cast<float*>(w + p.affine_partial[st][j]); };
    auto apart = [&](int j) { return apart_of(set, j); };
    auto wpart = [&](int j) { return reinterpret_cast<float*>(w + p.wgrad_partial[set][j]); };
    auto G = [&](int st, int which) { return w + p.g[Plan::kSetBase + st * Plan::kPerSet + which]; };   // which: 0-2 dy, 3 the projection's dy, 4 the masked output gradient
    std::vector<int> unit_done(blocks_.size(), -1);   // marks on the second stream: a unit's last work there
    constexpr int kProjSlot = Plan::kReduceSlots - 1;
    reduces_.clear();
    reduce_bytes_ = 0.0;
    // ---- head ----
    {
      GemmProblem g;  // dW = dlogits^T pooled; db = column sums
      g.dtype = dtype; g.a_layout = Layout::KRow; g.b_layout = Layout::KRow; g.epilogue = Epilogue::StoreF32;
      g.M = classes_; g.N = features_; g.K = batch_; g.A = w + p.dlogits; g.lda = lddz; g.B = w + p.pooled; g.ldb = features_;
      g.C = grad_ptrs[fc_w_]; g.ldc = features_; g.a_row_sum = static_cast<float*>(grad_ptrs[fc_b_]); g.a_pad_zero = g.b_pad_zero = true;
      g.name = "gemm_bf16_wgrad";
      if (int rc = gemm(g, s)) return rc;
    }
    if (cut >= num_units - 1) return SPB_OK;  // the head was the lowest unit: no input gradient
    {
      GemmProblem g;  // dpooled = dlogits W
      g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::KRow; g.epilogue = Epilogue::BiasAct;
      g.M = batch_; g.N = features_; g.K = classes_; g.A = w + p.dlogits; g.lda = lddz; g.B = param_ptrs[fc_w_]; g.ldb = features_;
      g.C = w + p.dpooled; g.ldc = features_; g.a_pad_zero = g.b_pad_zero = true; g.name = "gemm_bf16_dgrad";
      if (int rc = gemm(g, s)) return rc;
    }
    void* dout = w + p.g[0];
    int dout_slot = 0;
    bool incoming_fused = false;   // the unit above has already done this unit's output affine pass
    if (int rc = run("avgpool_bwd", (double)batch_ * hw * features_ * 2, s, [&] { return launch_avgpool_bwd(w + p.dpooled, dout, batch_, hw, features_, s); })) return rc;
    // ---- residual blocks, top down ----
    for (int i = (int)blocks_.size() - 1; i >= 0 && i + 1 >= cut; --i) {
      const Block& b = blocks_[i];
      const UnitBuf& u = p.unit[i + 1];
      const bool need_dx = i + 1 > cut;
      const void* x_in = w + p.unit[i].out;
      // Weight gradients and the unit's small reductions run on the second stream, beside the chain of input gradients.
      // What they read and this chain writes (the dy buffers, the projection's dy, the partial sums, the masked output
      // gradient) exists three times, unit i uses set i % 3 and the unit above already writes into the set of the
      // unit below (see the end of this loop), so the chain only has to know that the second stream is done with the
      // units three (here) and two (there) above - which it is long since; a join here would stall the chain behind
      // the previous unit's weight gradients at every unit.
      set = i % Plan::kSets;
      if (i + 3 < (int)blocks_.size())
        if (int rc = wait_mark(s, unit_done[i + 3])) return rc;
      void* dsum = G(set, 4);
      void* da = w + p.g[2];
      const int last = (int)b.convs.size() - 1;
      // dy rotates through three buffers: a fused input-gradient product writes the next dy while the weight gradient
      // forked one convolution earlier may still be reading the one before, and with three the buffer it writes was
      // last read two forks ago.
      void* const dy_slots[3] = {G(set, 0), G(set, 1), G(set, 2)};
      void* dy = dy_slots[0];
      int reader[3] = {-1, -1, -1};   // mark of the weight-gradient product that last read each of them
      int dy_slot = 0;                // dy lives in slot kDySlots[dy_slot]
      // the block's output gradient, masked by its ReLU, feeds the last convolution's affine and the shortcut (where
      // the unit above could fuse that pass into its last product, dy and dsum are there already)
      if (!incoming_fused)
        if (int rc = affine_bwd(b.convs[last], dout, w + u.out, w + u.conv[last].y, dy, dsum, apart(last), s)) return rc;
      for (int j = last; j >= 1; --j) {
        const void* in_j = w + u.conv[j - 1].a;
        if (int rc = conv_wgrad(b.convs[j], in_j, dy, wpart(j), static_cast<float*>(grad_ptrs[b.convs[j].w]), fork(s))) return rc;
        reader[dy_slot] = mark();
        const int next_slot = (dy_slot + 1) % 3;
        void* dy_next = dy_slots[next_slot];
        if (int rc = wait_mark(s, reader[next_slot])) return rc;   // whoever read that slot is done with it
        reader[next_slot] = -1;
        // the gradient at convolution j's input only feeds the affine + ReLU below: one pass where the product can take it
        const int fused = conv_dgrad_affine(b.convs[j], dy, param_ptrs[b.convs[j].w], b.convs[j - 1], in_j, w + u.conv[j - 1].y, dy_next, apart(j - 1), s);
        if (fused < 0) return fused;
        if (fused > 0) {
          if (int rc = conv_dgrad(b.convs[j], dy, param_ptrs[b.convs[j].w], nullptr, da, s)) return rc;
          if (int rc = affine_bwd(b.convs[j - 1], da, in_j, w + u.conv[j - 1].y, dy_next, nullptr, apart(j - 1), s)) return rc;
        }
        dy = dy_next;
        dy_slot = next_slot;
      }
      const void* shortcut_grad = dsum;
      void* dys = G(set, 3);
      if (b.has_proj)
        if (int rc = affine_bwd(b.proj, dsum, nullptr, w + u.proj.y, dys, nullptr, apart(kProjSlot), s)) return rc;
      {
        // the unit's last weight gradients and, behind them, all of its small reductions: the fork comes after every
        // affine pass of the unit, and nothing below reads what the reductions write
        hipStream_t side = fork(s);
        if (int rc = conv_wgrad(b.convs[0], x_in, dy, wpart(0), static_cast<float*>(grad_ptrs[b.convs[0].w]), side)) return rc;
        if (b.has_proj)
          if (int rc = conv_wgrad(b.proj, x_in, dys, wpart(kProjSlot), static_cast<float*>(grad_ptrs[b.proj.w]), side)) return rc;
        if (int rc = flush_reduces(side)) return rc;
        unit_done[i] = mark();
      }
      if (b.has_proj) {
        if (need_dx) {
          if (int rc = conv_dgrad(b.proj, dys, param_ptrs[b.proj.w], nullptr, w + p.g[3], s)) return rc;
          shortcut_grad = w + p.g[3];
        }
      }
      if (!need_dx) return SPB_OK;  // lowest unit: no input gradient
      if (fuses_into_unit_below(i)) {
        // The unit's input gradient (this product plus the shortcut's) only feeds the affine + ReLU at the output of the
        // unit below and, masked, that unit's shortcut: the product's epilogue does that pass and writes the unit
        // below's first dy and its masked output gradient straight into that unit's set of buffers.
        const Block& below = blocks_[i - 1];
        const int set_below = (i - 1) % Plan::kSets, last_below = (int)below.convs.size() - 1;
        if (i + 2 < (int)blocks_.size())
          if (int rc = wait_mark(s, unit_done[i + 2])) return rc;   // the unit that last used that set
        const int fused = conv_dgrad_affine(b.convs[0], dy, param_ptrs[b.convs[0].w], below.convs[last_below], x_in, w + p.unit[i].conv[last_below].y,
                                            G(set_below, 0), apart_of(set_below, last_below), s, shortcut_grad, G(set_below, 4));
        if (fused < 0) return fused;
        if (fused > 0) { set_error("resnet: the last input gradient of unit %d cannot carry the affine pass below it", i + 1); return SPB_ERR_INVALID_ARG; }
        incoming_fused = true;
      } else {
        void* dx = w + p.g[dout_slot ^ 1];
        if (int rc = conv_dgrad(b.convs[0], dy, param_ptrs[b.convs[0].w], shortcut_grad, dx, s)) return rc;
        dout = dx;
        dout_slot ^= 1;
        incoming_fused = false;
      }
    }
    // ---- stem (unit 0), reached only at full depth ----
    if (cut == 0) {
      if (int rc = join(s)) return rc;   // the buffers of set 0 are written next
      const UnitBuf& su = p.unit[0];
      const void* d = dout;
      if (pool_) {
        if (int rc = run("maxpool_bwd", (double)stem_.out_rows(batch_) * stem_.cout * 2 * 1.5, s, [&] {
              return launch_maxpool_bwd(dout, reinterpret_cast<const uint8_t*>(w + su.which), w + p.g[2], batch_, stem_.out_h, stem_.out_w, stem_.cout, s); })) return rc;
        d = w + p.g[2];
      }
      set = 0;
      if (int rc = affine_bwd(stem_, d, w + su.conv[0].a, w + su.conv[0].y, G(0, 0), nullptr, apart(0), s)) return rc;
      const void* stem_in = stem_.cin_eff != stem_.cin ? (const void*)(w + su.xpad) : x_;
      if (int rc = conv_wgrad(stem_, stem_in, G(0, 0), wpart(0), static_cast<float*>(grad_ptrs[stem_.w]), s)) return rc;
      if (int rc = flush_reduces(s)) return rc;
    }
    return SPB_OK;
  }

  void unit_io(int k, int unit, spb_buffer_view* input, spb_buffer_view* output_grad) const override {
    const Plan p = plan(k);
    const int nb = (int)blocks_.size();
    // NHWC tensors as [pixels, channels]
    if (unit == 0) {
      *input = make_view(SPB_VIEW_CALLER_INPUT, stem_.in_rows(batch_), stem_.cin, stem_.cin, dtype);
    } else if (unit <= nb) {
      const Conv& c = blocks_[unit - 1].convs[0];
      *input = make_view((long long)p.unit[unit - 1].out, c.in_rows(batch_), c.cin, c.cin, dtype);
    } else {
      *input = make_view((long long)p.unit[nb].out, (long long)batch_ * final_h_ * final_w_, features_, features_, dtype);
    }
    // The gradient entering the top block lies in slot 0.  Below it, a unit whose upper neighbour fuses the output
    // affine pass (the usual case) receives its gradient already masked by its own ReLU, in its set's fifth buffer;
    // otherwise slots 0 and 1 alternate, as they do for the stem.
    if (unit == nb + 1 || k < 2) {
      *output_grad = no_view();
      return;
    }
    int slot = 0;   // where an unfused hand-over lands next
    for (int i = nb - 1; i >= 0; --i) {   // block i = unit i + 1, walked as the backward pass walks them
      const bool fused_in = i < nb - 1 && fuses_into_unit_below(i + 1);
      if (unit == i + 1) {
        const Conv& c = blocks_[i].convs.back();
        if (fused_in) *output_grad = make_view((long long)p.g[Plan::kSetBase + (i % Plan::kSets) * Plan::kPerSet + 4], c.out_rows(batch_), c.cout, c.cout, dtype, 1);
        else *output_grad = make_view((long long)p.g[slot], c.out_rows(batch_), c.cout, c.cout, dtype);
        return;
      }
      if (!fuses_into_unit_below(i)) slot ^= 1;   // this block writes its input gradient into the other slot
    }
    const long long rows = pool_ ? (long long)batch_ * pool_h_ * pool_w_ : stem_.out_rows(batch_);
    *output_grad = make_view((long long)p.g[slot], rows, stem_.cout, stem_.cout, dtype);
  }

 private:
  int batch_ = 0, classes_ = 0, features_ = 0, final_h_ = 0, final_w_ = 0, pool_h_ = 0, pool_w_ = 0;
  bool pool_ = false;
  Conv stem_;
  std::vector<Block> blocks_;
  int fc_w_ = -1, fc_b_ = -1;
  const void* x_ = nullptr;
  std::vector<ReduceTask> reduces_;   // of the unit whose backward pass is being enqueued
  int fused_tile_rows_ = 0;
  double reduce_bytes_ = 0.0;
};

}  // namespace

std::unique_ptr<Model> make_resnet(const spb_model_desc& d) {
  if (d.dtype != SPB_DTYPE_BF16) { set_error("resnet: only bfloat16 storage is built"); return nullptr; }
  if (d.image_h <= 0 || d.image_w <= 0 || d.image_c <= 0 || d.image_c > 8 || d.stem_kernel <= 0 || d.stem_width <= 0 || d.classes <= 0 ||
      d.n_stages <= 0 || d.n_stages > SPB_MAX_STAGES || d.stem_pad < 0) {
    set_error("resnet: image (up to 8 channels), stem, stages and classes must be positive");
    return nullptr;
  }
  for (int i = 0; i < d.n_stages; ++i)
    if (d.stage_blocks[i] <= 0 || d.stage_widths[i] <= 0 || (d.family == SPB_FAMILY_RESNET_BOTTLENECK && d.stage_widths[i] % 32)) {
      set_error("resnet: stage %d needs blocks > 0 and a positive width (a multiple of 32 for bottlenecks)", i);
      return nullptr;
    }
  auto m = std::make_unique<ResnetModel>(d);
  std::string why;
  if (!m->shapes_ok(&why)) { set_error("resnet: %s", why.c_str()); return nullptr; }
  return m;
}

}  // namespace spb
