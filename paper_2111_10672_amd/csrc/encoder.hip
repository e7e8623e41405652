// Transformer-encoder family: units = embedding | pre-LayerNorm layers | masked-token head.
// Forward pass, stash plan and truncated backward pass (Sec. 1-2 of the paper).
//
//   layer:  u = LN1(x);  qkv = u Wqkv^T + b;  P = softmax(Q K^T / sqrt d);  ctx = P V;  h = x + ctx Wo^T + bo
//           v = LN2(h);  z1 = v W1^T + b1;  f = gelu(z1);  out = h + f W2^T + b2
//   head:   y = LN(x[loss rows]);  logits = y Wv^T + bv;  mean softmax cross-entropy
//
// A layer above the cut keeps u, qkv, P, ctx, h, v, gelu'(z1), f and the LayerNorm statistics; layers below the
// cut share one scratch set and their outputs alternate between two buffers.  Every product runs on the
// MFMA kernel of gemm_dma.hip (attention as batched products over batch x heads); bias, GELU, residual
// adds and the GELU derivative ride in its epilogue, the residual fan-in of the backward pass rides in the
// LayerNorm backward kernel.
#include <algorithm>
#include <cmath>

#include "model.h"

namespace spb {
namespace {

struct LayerBuf { size_t u, stats1, qkv, prob, ctx, h, stats2, v, z1, f; };

class EncoderModel : public Model {
 public:
  explicit EncoderModel(const spb_model_desc& d) {
    dtype = DType::BF16;
    needs_loss_rows = true;
    B = d.batch; S = d.seq; NL = d.layers; H = d.hidden; NH = d.heads; D = H / NH; F = d.ffn; V = d.vocab; R = d.loss_rows;
    M = B * S; Z = B * NH;
    num_units = NL + 2;
    auto add = [&](const std::string& name, int unit, std::vector<int64_t> shape) {
      ParamInfo p; p.name = name; p.unit = unit; p.dtype = dtype; p.shape = std::move(shape); params.push_back(p);
    };
    add("embed.tok.weight", 0, {V, H});
    add("embed.pos.weight", 0, {S, H});
    for (int i = 0; i < NL; ++i) {
      const std::string pre = "layer" + std::to_string(i) + ".";
      add(pre + "ln1.weight", i + 1, {H}); add(pre + "ln1.bias", i + 1, {H});
      add(pre + "attn.qkv.weight", i + 1, {3 * H, H}); add(pre + "attn.qkv.bias", i + 1, {3 * H});
      add(pre + "attn.out.weight", i + 1, {H, H}); add(pre + "attn.out.bias", i + 1, {H});
      add(pre + "ln2.weight", i + 1, {H}); add(pre + "ln2.bias", i + 1, {H});
      add(pre + "ffn.w1.weight", i + 1, {F, H}); add(pre + "ffn.w1.bias", i + 1, {F});
      add(pre + "ffn.w2.weight", i + 1, {H, F}); add(pre + "ffn.w2.bias", i + 1, {H});
    }
    add("head.ln.weight", NL + 1, {H}); add("head.ln.bias", NL + 1, {H});
    add("head.vocab.weight", NL + 1, {V, H}); add("head.vocab.bias", NL + 1, {V});
    param_ptrs.assign(params.size(), nullptr);
    grad_ptrs.assign(params.size(), nullptr);
  }

  enum { LN1W, LN1B, QKVW, QKVB, OUTW, OUTB, LN2W, LN2B, W1W, W1B, W2W, W2B };
  int lp(int layer, int j) const { return 2 + 12 * layer + j; }
  int hp(int j) const { return 2 + 12 * NL + j; }
  int ldz() const { return (int)align_up((size_t)V, 4); }
  int ldv() const { return (int)align_up((size_t)V, 8); }

  struct Plan {
    std::vector<size_t> xout;        // output of unit u, u = 0..NL
    std::vector<LayerBuf> layer;     // per layer: own stash or the shared scratch
    size_t scores, y, statsf, logits, row_loss, dlogits;
    size_t dy, partial, partial_bytes, dx[2], dF[2], dv, dh[2], dctx, dscore, dqkv[2], du;
    size_t total;
  };

  Plan plan(int k) const {
    Plan p;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
    const size_t mh = (size_t)M * H * 2, mf = (size_t)M * F * 2, zss = (size_t)Z * S * S;
    const int cut = num_units - k;  // units >= cut are backpropagated
    auto take_layer = [&]() {
      LayerBuf b;
      b.u = take(mh); b.stats1 = take((size_t)M * 8); b.qkv = take(3 * mh); b.prob = take(zss * 2); b.ctx = take(mh);
      b.h = take(mh); b.stats2 = take((size_t)M * 8); b.v = take(mh); b.z1 = take(mf); b.f = take(mf);
      return b;
    };
    const size_t ping[2] = {take(mh), take(mh)};
    const LayerBuf scratch = take_layer();
    p.xout.assign(NL + 1, 0);
    p.layer.assign(NL, scratch);
    for (int u = 0; u <= NL; ++u) p.xout[u] = (u + 1 >= cut) ? take(mh) : ping[u & 1];  // kept if the unit above reads it in its backward pass
    for (int i = 0; i < NL; ++i) if (i + 1 >= cut) p.layer[i] = take_layer();
    p.scores = take(zss * 4);
    p.y = take((size_t)R * H * 2); p.statsf = take((size_t)R * 8); p.logits = take((size_t)R * ldz() * 4);
    p.row_loss = take((size_t)R * 4); p.dlogits = take((size_t)R * ldv() * 2);
    p.dy = p.partial = p.partial_bytes = p.dx[0] = p.dx[1] = p.dF[0] = p.dF[1] = p.dv = p.dh[0] = p.dh[1] = p.dctx = p.dscore = p.dqkv[0] = p.dqkv[1] = p.du = 0;
    if (k >= 1) {
      p.dy = take((size_t)R * H * 2);
      // one per LayerNorm in the backward pass: their column sums are added up in one launch at the end
      p.partial_bytes = align_up(std::max(layernorm_partial_floats(M, H), layernorm_partial_floats(R, H)) * 4, 256);
      p.partial = take(p.partial_bytes * (size_t)(2 * std::min(k - 1, NL) + 1));
    }
    if (k >= 2) {
      // dF, dh and dqkv are read by weight gradients on the second stream: two of each, used by alternate layers
      p.dx[0] = take(mh); p.dx[1] = take(mh); p.dF[0] = take(mf); p.dF[1] = take(mf); p.dv = take(mh); p.dh[0] = take(mh); p.dh[1] = take(mh);
      p.dctx = take(mh); p.dscore = take(zss * 2); p.dqkv[0] = take(3 * mh); p.dqkv[1] = take(3 * mh); p.du = take(mh);
    }
    p.total = off;
    return p;
  }

  size_t workspace_size(int k) const override { return plan(k).total; }

  // ---- product helpers -------------------------------------------------------------------------
  GemmProblem linear(const void* a, int lda, int rows, const void* w, int n_out, int n_in, const void* bias, void* c, int ldc) const {
    GemmProblem g;  // C[rows, n_out] = a[rows, n_in] * w[n_out, n_in]^T + bias
    g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::RowK; g.epilogue = Epilogue::BiasAct;
    g.M = rows; g.N = n_out; g.K = n_in; g.A = a; g.lda = lda; g.B = w; g.ldb = n_in; g.bias = bias; g.C = c; g.ldc = ldc;
    g.name = "gemm_bf16_fwd";
    return g;
  }
  GemmProblem wgrad(const void* dz, int lddz, const void* a, int lda, int rows, int n_out, int n_in, float* dw, float* db) const {
    GemmProblem g;  // dw[n_out, n_in] = dz[rows, n_out]^T * a[rows, n_in];  db = column sums of dz
    g.dtype = dtype; g.a_layout = Layout::KRow; g.b_layout = Layout::KRow; g.epilogue = Epilogue::StoreF32;
    g.M = n_out; g.N = n_in; g.K = rows; g.A = dz; g.lda = lddz; g.B = a; g.ldb = lda; g.C = dw; g.ldc = n_in; g.a_row_sum = db;
    g.a_pad_zero = g.b_pad_zero = true;
    g.name = "gemm_bf16_wgrad";
    return g;
  }
  GemmProblem dgrad(const void* dz, int lddz, int rows, const void* w, int n_out, int n_in, void* dx, int lddx) const {
    GemmProblem g;  // dx[rows, n_in] = dz[rows, n_out] * w[n_out, n_in]
    g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::KRow; g.epilogue = Epilogue::BiasAct;
    g.M = rows; g.N = n_in; g.K = n_out; g.A = dz; g.lda = lddz; g.B = w; g.ldb = n_in; g.C = dx; g.ldc = lddx;
    g.a_pad_zero = g.b_pad_zero = true;
    g.name = "gemm_bf16_dgrad";
    return g;
  }
  BatchStride per_head(long long row_pitch) const { BatchStride b; b.outer = (long long)S * row_pitch; b.inner = D; b.inner_count = NH; return b; }
  BatchStride per_matrix() const { BatchStride b; b.outer = (long long)NH * S * S; b.inner = (long long)S * S; b.inner_count = NH; return b; }

  const char* bf(const void* base, size_t elems) const { return static_cast<const char*>(base) + elems * 2; }
  char* bf(void* base, size_t elems) const { return static_cast<char*>(base) + elems * 2; }

  int forward(const void* x, const int32_t* labels, const int32_t* loss_rows, int k, void* wsp, float* loss_out, hipStream_t s) override {
    const Plan p = plan(k);
    char* w = static_cast<char*>(wsp);
    ids_ = static_cast<const int32_t*>(x);
    rows_ = loss_rows;
    const float inv_sqrt_d = 1.f / std::sqrt((float)D);
    const double mh = (double)M * H * 2;
    if (int rc = run("embedding_fwd", 2 * mh, s, [&] {
          return launch_embedding_fwd(ids_, param_ptrs[0], param_ptrs[1], w + p.xout[0], H, M, S, V, H, s); })) return rc;
    for (int i = 0; i < NL; ++i) {
      const LayerBuf& b = p.layer[i];
      const void* xin = w + p.xout[i];
      auto P = [&](int j) { return param_ptrs[lp(i, j)]; };
      if (int rc = run("layernorm_fwd", 2 * mh, s, [&] {
            return launch_layernorm_fwd(xin, H, nullptr, M, H, P(LN1W), P(LN1B), w + b.u, H, reinterpret_cast<float*>(w + b.stats1), s); })) return rc;
      if (int rc = gemm(linear(w + b.u, H, M, P(QKVW), 3 * H, H, P(QKVB), w + b.qkv, 3 * H), s)) return rc;
      if (attention_fused_accepts(S, D, 3 * H, H)) {
        // one kernel per layer; P is written only where the backward pass will read it
        void* keep_prob = (i + 1 >= num_units - k) ? w + b.prob : nullptr;
        if (int rc = run("attention_fwd", (double)M * H * 2 * 4 + (keep_prob ? (double)Z * S * S * 2 : 0.0), s, [&] {
              return launch_attention_fwd(w + b.qkv, 3 * H, keep_prob, w + b.ctx, H, B, NH, S, D, inv_sqrt_d, s); })) return rc;
      } else {
      {
        GemmProblem g;  // scores[z, s, s'] = Q[s, :] . K[s', :] / sqrt(d)
        g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::RowK; g.epilogue = Epilogue::StoreF32;
        g.M = S; g.N = S; g.K = D; g.A = w + b.qkv; g.lda = 3 * H; g.B = bf(w + b.qkv, (size_t)H); g.ldb = 3 * H;
        g.C = w + p.scores; g.ldc = S; g.alpha = inv_sqrt_d;
        g.batch = Z; g.a_batch = g.b_batch = per_head(3 * H); g.c_batch = per_matrix();
        g.name = "attn_scores";
        if (int rc = gemm(g, s)) return rc;
      }
      if (int rc = run("softmax_fwd", (double)Z * S * S * 6, s, [&] {
            return launch_softmax_fwd(reinterpret_cast<const float*>(w + p.scores), w + b.prob, (long long)Z * S, S, s); })) return rc;
      {
        GemmProblem g;  // ctx[s, d] = sum_s' P[s, s'] V[s', d]
        g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::KRow; g.epilogue = Epilogue::BiasAct;
        g.M = S; g.N = D; g.K = S; g.A = w + b.prob; g.lda = S; g.B = bf(w + b.qkv, (size_t)2 * H); g.ldb = 3 * H;
        g.C = w + b.ctx; g.ldc = H;
        g.batch = Z; g.a_batch = per_matrix(); g.b_batch = per_head(3 * H); g.c_batch = per_head(H);
        g.name = "attn_context";
        if (int rc = gemm(g, s)) return rc;
      }
      }
      {
        GemmProblem g = linear(w + b.ctx, H, M, P(OUTW), H, H, P(OUTB), w + b.h, H);
        g.residual = xin; g.ldres = H;
        if (int rc = gemm(g, s)) return rc;
      }
      if (int rc = run("layernorm_fwd", 2 * mh, s, [&] {
            return launch_layernorm_fwd(w + b.h, H, nullptr, M, H, P(LN2W), P(LN2B), w + b.v, H, reinterpret_cast<float*>(w + b.stats2), s); })) return rc;
      {
        GemmProblem g = linear(w + b.v, H, M, P(W1W), F, H, P(W1B), w + b.f, F);
        g.act = Act::Gelu;
        if (i + 1 >= num_units - k) { g.aux_out = w + b.z1; g.ldaux = F; g.aux_act_grad = 1; }   // above the cut: keep gelu'(z1), all the backward pass needs of z1
        if (int rc = gemm(g, s)) return rc;
      }
      {
        GemmProblem g = linear(w + b.f, F, M, P(W2W), H, F, P(W2B), w + p.xout[i + 1], H);
        g.residual = w + b.h; g.ldres = H;
        if (int rc = gemm(g, s)) return rc;
      }
    }
    if (int rc = run("layernorm_fwd", 4.0 * R * H, s, [&] {
          return launch_layernorm_fwd(w + p.xout[NL], H, rows_, R, H, param_ptrs[hp(0)], param_ptrs[hp(1)], w + p.y, H,
                                      reinterpret_cast<float*>(w + p.statsf), s); })) return rc;
    {
      GemmProblem g = linear(w + p.y, H, R, param_ptrs[hp(2)], V, H, param_ptrs[hp(3)], w + p.logits, ldz());
      g.epilogue = Epilogue::StoreF32;
      g.name = "gemm_bf16_fwd_logits";
      if (int rc = gemm(g, s)) return rc;
    }
    return run("softmax_xent", (double)R * V * 6, s, [&] {
      return launch_softmax_xent(reinterpret_cast<const float*>(w + p.logits), ldz(), labels, R, V, w + p.dlogits, ldv(), dtype,
                                 reinterpret_cast<float*>(w + p.row_loss), loss_out, s); });
  }

  int backward(int k, hipStream_t s) override {
    const Plan p = plan(stashed_k);
    char* w = static_cast<char*>(ws);
    const int cut = num_units - k;
    const float inv_sqrt_d = 1.f / std::sqrt((float)D);
    const double mh = (double)M * H * 2;
    // The column sums of every LayerNorm backward (dgamma, dbeta) are small reductions that feed nothing in this pass:
    // each leaves its partial sums in a buffer of its own and one launch at the end adds all of them up, instead of
    // two short kernels per layer on the chain.
    std::vector<ReduceTask> ln_sums;
    ln_sums.reserve(2 * NL + 1);
    auto next_partial = [&]() {
      ln_sums.emplace_back();
      return reinterpret_cast<float*>(w + p.partial + p.partial_bytes * (ln_sums.size() - 1));
    };
    auto G = [&](int idx) { return static_cast<float*>(grad_ptrs[idx]); };

    // ---- head (unit NL + 1) ----
    const bool head_lowest = cut == NL + 1;
    // Weight gradients go to the side stream (they feed nothing in this pass); the input-gradient chain stays on s.
    if (int rc = gemm(wgrad(w + p.dlogits, ldv(), w + p.y, H, R, V, H, G(hp(2)), G(hp(3))), fork(s))) return rc;
    {
      // dy = dlogits Wv: a small result over a very long k (the vocabulary).  With too few output tiles to fill
      // the chip the k range is cut into slices; their float32 partial products go where the logits were (read
      // for the last time by the loss) and are added up into dy.
      GemmProblem g = dgrad(w + p.dlogits, ldv(), R, param_ptrs[hp(2)], V, H, w + p.dy, H);
      const long tiles = (long)((R + 127) / 128) * ((H + 127) / 128);
      int slices = (int)std::min<long>(256 / std::max<long>(tiles, 1), 16);
      slices = (int)std::min<long>(slices, std::min<long>(V / 1024, ((long)ldz() * 4) / ((long)H * 4)));
      if (slices >= 2) {
        g.k_splits = slices; g.epilogue = Epilogue::StoreF32; g.C = w + p.logits; g.ldc = H;
        if (int rc = gemm(g, s)) return rc;
        if (int rc = run("splitk_reduce", (double)(slices * 4 + 2) * R * H, s, [&] {
              return launch_splitk_reduce_bf16(reinterpret_cast<const float*>(w + p.logits), slices, (long long)R * H, w + p.dy, (long long)R * H, s); }))
          return rc;
      } else if (int rc = gemm(g, s)) return rc;
    }
    void* dout = nullptr;
    if (!head_lowest) {
      dout = w + p.dx[0];
      if (int rc = run("fill_zero", mh, s, [&] { return launch_fill_zero(dout, (size_t)M * H * 2, s); })) return rc;
    }
    float* part = next_partial();
    if (int rc = run("layernorm_bwd", 6.0 * R * H, s, [&] {
          return launch_layernorm_bwd(w + p.dy, H, w + p.xout[NL], H, rows_, reinterpret_cast<const float*>(w + p.statsf), param_ptrs[hp(0)],
                                      nullptr, 0, dout, H, part, G(hp(0)), G(hp(1)), R, H, s, &ln_sums.back()); })) return rc;
    int which = 0;  // dout lives in p.dx[which]
    std::vector<int> ffn_done(NL, -1), side_done(NL, -1);   // marks on the second stream: after a layer's first / second pair of weight gradients

    // ---- encoder layers, top down ----
    for (int i = NL - 1; i >= 0 && i + 1 >= cut; --i) {
      const bool lowest = i + 1 == cut;
      const LayerBuf& b = p.layer[i];
      const void* xin = w + p.xout[i];
      auto P = [&](int j) { return param_ptrs[lp(i, j)]; };
      auto GP = [&](int j) { return G(lp(i, j)); };
      // Weight gradients on the second stream read dF, dh, dqkv and the layer's incoming gradient.  Alternate layers use
      // alternate copies of the first three, so this layer only has to know that the weight gradients of the layer
      // two above are done - which they are long since; a join here would stall the chain behind the previous
      // layer's weight gradients at every layer.
      char* dF = w + p.dF[i & 1];
      char* dh = w + p.dh[i & 1];
      char* dqkv = w + p.dqkv[i & 1];
      if (i + 2 < NL)
        if (int rc = wait_mark(s, side_done[i + 2])) return rc;
      // feed-forward half
      {
        GemmProblem g = dgrad(dout, H, M, P(W2W), H, F, dF, F);   // dz1 = (dout W2) * gelu'(z1), the factor as stashed
        g.epilogue = Epilogue::ScaleStore; g.mask = w + b.z1; g.ldmask = F;
        if (int rc = gemm(g, s)) return rc;
      }
      {
        hipStream_t side = fork(s);   // one fork for both weight gradients of the feed-forward half: each fork costs a few microseconds
        if (int rc = gemm(wgrad(dout, H, w + b.f, F, M, H, F, GP(W2W), GP(W2B)), side)) return rc;
        if (int rc = gemm(wgrad(dF, F, w + b.v, H, M, F, H, GP(W1W), GP(W1B)), side)) return rc;
        ffn_done[i] = mark();
      }
      if (int rc = gemm(dgrad(dF, F, M, P(W1W), F, H, w + p.dv, H), s)) return rc;
      part = next_partial();
      if (int rc = run("layernorm_bwd", 4 * mh, s, [&] {   // dh = dout + LN2 backward
            return launch_layernorm_bwd(w + p.dv, H, w + b.h, H, nullptr, reinterpret_cast<const float*>(w + b.stats2), P(LN2W), dout, H,
                                        dh, H, part, GP(LN2W), GP(LN2B), M, H, s, &ln_sums.back()); })) return rc;
      // attention half
      // (this product and the one through Wqkv run beside the feed-forward weight gradients, whose workgroups take
      // 128 KB of a CU's LDS: with 64 KB tiles of their own they find room on the same CUs - +2 % on the step; the
      // product through W1 measured better with the big-footprint kernel)
      {
        GemmProblem g = dgrad(dh, H, M, P(OUTW), H, H, w + p.dctx, H);
        g.share_cu = true;
        if (int rc = gemm(g, s)) return rc;
      }
      const char* qbase = w + b.qkv;
      if (attention_fused_accepts(S, D, 3 * H, H)) {
        if (int rc = run("attention_bwd", (double)M * H * 2 * 7 + (double)Z * S * S * 2, s, [&] {
              return launch_attention_bwd(qbase, 3 * H, w + b.prob, w + p.dctx, H, dqkv, B, NH, S, D, inv_sqrt_d, s); })) return rc;
      } else {
      {
        GemmProblem g;  // dP[s, s'] = dctx[s, :] . V[s', :]
        g.dtype = dtype; g.a_layout = Layout::RowK; g.b_layout = Layout::RowK; g.epilogue = Epilogue::StoreF32;
        g.M = S; g.N = S; g.K = D; g.A = w + p.dctx; g.lda = H; g.B = bf(qbase, (size_t)2 * H); g.ldb = 3 * H;
        g.C = w + p.scores; g.ldc = S;
        g.batch = Z; g.a_batch = per_head(H); g.b_batch = per_head(3 * H); g.c_batch = per_matrix();
        g.name = "attn_bwd_dprob";
        if (int rc = gemm(g, s)) return rc;
      }
      if (int rc = run("softmax_bwd", (double)Z * S * S * 8, s, [&] {
            return launch_softmax_bwd(reinterpret_cast<const float*>(w + p.scores), w + b.prob, w + p.dscore, (long long)Z * S, S, inv_sqrt_d, s); })) return rc;
      auto attn_out = [&](const char* name, Layout la, const void* a, int lda, BatchStride ab, const void* bsrc, int col_block) {
        GemmProblem g;  // [S, D] per head, written into the q, k or v third of dqkv
        g.dtype = dtype; g.a_layout = la; g.b_layout = Layout::KRow; g.epilogue = Epilogue::BiasAct;
        g.M = S; g.N = D; g.K = S; g.A = a; g.lda = lda; g.a_batch = ab;
        g.B = bsrc; g.ldb = (bsrc == (const void*)(w + p.dctx)) ? H : 3 * H;
        g.b_batch = per_head(g.ldb);
        g.C = bf(dqkv, (size_t)col_block * H); g.ldc = 3 * H; g.c_batch = per_head(3 * H);
        g.batch = Z; g.name = name;
        return gemm(g, s);
      };
      // dV = P^T dctx;  dQ = dS K;  dK = dS^T Q
      if (int rc = attn_out("attn_bwd_dv", Layout::KRow, w + b.prob, S, per_matrix(), w + p.dctx, 2)) return rc;
      if (int rc = attn_out("attn_bwd_dq", Layout::RowK, w + p.dscore, S, per_matrix(), bf(qbase, (size_t)H), 0)) return rc;
      if (int rc = attn_out("attn_bwd_dk", Layout::KRow, w + p.dscore, S, per_matrix(), qbase, 1)) return rc;
      }
      {
        hipStream_t side = fork(s);   // and one for the attention half
        if (int rc = gemm(wgrad(dh, H, w + b.ctx, H, M, H, H, GP(OUTW), GP(OUTB)), side)) return rc;
        // (the lowest layer's goes behind its LayerNorm on the chain itself, which has nothing else left to do, so
        // that the step does not end on two weight gradients in a row on the second stream)
        if (!lowest)
          if (int rc = gemm(wgrad(dqkv, 3 * H, w + b.u, H, M, 3 * H, H, GP(QKVW), GP(QKVB)), side)) return rc;
        side_done[i] = mark();
      }
      {
        GemmProblem g = dgrad(dqkv, 3 * H, M, P(QKVW), 3 * H, H, w + p.du, H);
        g.share_cu = true;
        if (int rc = gemm(g, s)) return rc;
      }
      void* dx = lowest ? nullptr : w + p.dx[which ^ 1];
      // dx lands where the layer above found its incoming gradient, which that layer's feed-forward weight gradient reads
      if (dx && i + 1 < NL)
        if (int rc = wait_mark(s, ffn_done[i + 1])) return rc;
      part = next_partial();
      if (int rc = run("layernorm_bwd", (lowest ? 2 : 4) * mh, s, [&] {   // dx = dh + LN1 backward; the lowest unit forms no input gradient
            return launch_layernorm_bwd(w + p.du, H, xin, H, nullptr, reinterpret_cast<const float*>(w + b.stats1), P(LN1W), dh, H,
                                        dx, H, part, GP(LN1W), GP(LN1B), M, H, s, &ln_sums.back()); })) return rc;
      if (lowest)
        if (int rc = gemm(wgrad(dqkv, 3 * H, w + b.u, H, M, 3 * H, H, GP(QKVW), GP(QKVB)), s)) return rc;
      dout = dx;
      which ^= 1;
    }
    {
      double bytes = 0;
      for (const ReduceTask& t : ln_sums) bytes += (double)(t.count + 1) * 2 * t.width * 4;
      if (int rc = run("layernorm_sums", bytes, s, [&] { return launch_unit_reduce(ln_sums.data(), (int)ln_sums.size(), s); })) return rc;
    }
    // ---- embedding (unit 0), only at full depth ----
    if (cut == 0)
      return run("embedding_bwd", mh + (double)V * H * 4, s, [&] { return launch_embedding_bwd(ids_, dout, H, G(0), G(1), B, S, V, H, s); });
    return SPB_OK;
  }

  void unit_io(int k, int unit, spb_buffer_view* input, spb_buffer_view* output_grad) const override {
    const Plan p = plan(k);
    if (unit == 0) {
      *input = make_view(SPB_VIEW_CALLER_INPUT, B, S, S, DType::F32);
      input->dtype = SPB_DTYPE_I32;   // token ids
    } else {
      *input = make_view((long long)p.xout[unit - 1], M, H, H, dtype);
    }
    // The head writes the gradient of the last layer's output into dx[0]; each layer reads one and writes the other.
    *output_grad = (unit == NL + 1 || k < 2) ? no_view() : make_view((long long)p.dx[(NL - unit) & 1], M, H, H, dtype);
  }

 private:
  int B = 0, S = 0, NL = 0, H = 0, NH = 0, D = 0, F = 0, V = 0, R = 0, M = 0, Z = 0;
  const int32_t* ids_ = nullptr;
  const int32_t* rows_ = nullptr;
};

}  // namespace

std::unique_ptr<Model> make_encoder(const spb_model_desc& d) {
  if (d.dtype != SPB_DTYPE_BF16) { set_error("encoder: only bfloat16 storage is built"); return nullptr; }
  if (d.seq <= 0 || d.layers <= 0 || d.hidden <= 0 || d.heads <= 0 || d.ffn <= 0 || d.vocab <= 0 || d.loss_rows <= 0) {
    set_error("encoder: seq, layers, hidden, heads, ffn, vocab and loss_rows must be positive"); return nullptr;
  }
  if (d.hidden % d.heads || (d.hidden / d.heads) % 8 || d.hidden % 8 || d.ffn % 8 || d.seq % 8 || d.hidden > 2048) {
    set_error("encoder: hidden/heads, hidden, ffn and seq must be multiples of 8 (16-byte chunks), hidden <= 2048"); return nullptr;
  }
  if ((long long)d.loss_rows > (long long)d.batch * d.seq) { set_error("encoder: more loss rows than positions"); return nullptr; }
  if ((long long)d.batch * d.heads > 65535) { set_error("encoder: batch * heads exceeds 65535"); return nullptr; }
  return std::make_unique<EncoderModel>(d);
}

}  // namespace spb
