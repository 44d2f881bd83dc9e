// Post-LN transformer encoder classifier in bf16 with fp32 accumulation: the explicit forward / backward kernel
// sequence (no autograd).  x0 = LN(tok[ids] + pos); per layer x <- LN1(x + Attn(x)), x <- LN2(x + FFN(x));
// logits = x_L[:, 0] Wc^T + bc.  Residual sums and every LayerNorm input stay fp32; GEMM operands are bf16.
#include "kernels.h"
#include "model.h"

namespace sama {
static bool g_side_stream = true, g_side_sink = true;
void encoder_side_stream(bool on) { g_side_stream = on; }
void encoder_side_sink(bool on) { g_side_sink = on; }
namespace {
inline bool side_enabled() { return g_side_stream; }

struct LayerOff { int64_t Wqkv, Wo, W1, W2, bqkv, bo, ln1g, ln1b, b1, b2, ln2g, ln2b; };

class EncoderModel : public Model {
 public:
  EncoderModel(const sama_config& c, const std::vector<TensorInfo>& lay) {
    L_ = c.dims[0]; d_ = c.dims[1]; heads_ = c.dims[2]; ffn_ = c.dims[3]; S_ = c.dims[4]; V_ = c.dims[5]; C_ = c.dims[6];
    auto find = [&](const std::string& nm) { for (auto& t : lay) if (t.name == nm) return t.offset; return (int64_t)-1; };
    for (int l = 0; l < L_; ++l) {
      const std::string p = "l" + std::to_string(l) + ".";
      off_.push_back({find(p + "Wqkv"), find(p + "Wo"), find(p + "W1"), find(p + "W2"), find(p + "bqkv"), find(p + "bo"),
                      find(p + "ln1_g"), find(p + "ln1_b"), find(p + "b1"), find(p + "b2"), find(p + "ln2_g"), find(p + "ln2_b")});
    }
    tok_ = find("tok_emb"); pos_ = find("pos_emb"); eg_ = find("emb_ln_g"); eb_ = find("emb_ln_b"); wc_ = find("Wc"); bc_ = find("bc");
    wm_ = find("Wmlm"); bm_ = find("bmlm");
    P_ = wm_ >= 0 ? (c.max_aux_masked + 63) / 64 * 64 : 0;
  }
  int n_classes() const override { return C_; }
  bool has_mlm() const override { return wm_ >= 0; }
  int mlm_stride() const override { return P_; }

  void plan(BumpAlloc& ws, int max_b) override {
    const size_t M = (size_t)max_b * S_;
    X_.resize(L_ + 1); qkv_.resize(L_); lse_.resize(L_); ao_.resize(L_); pre1_.resize(L_); mean1_.resize(L_); rstd1_.resize(L_);
    x1_.resize(L_); fpre_.resize(L_); fact_.resize(L_); pre2_.resize(L_); mean2_.resize(L_); rstd2_.resize(L_);
    // Forward-only passes run in activation slot 0 and ping-pong between X_[0] / X_[1]; the + and the - pass of
    // Eq. 5 run stacked (2M rows), so those buffers are twice as tall.
    for (int l = 0; l <= L_; ++l) X_[l] = ws.take<bf16_t>((l < 2 ? 2 : 1) * M * d_);
    for (int l = 0; l < L_; ++l) {
      const size_t R = (l == 0 ? 2 : 1) * M;
      qkv_[l] = ws.take<bf16_t>(R * 3 * d_); lse_[l] = ws.take<float>((size_t)max_b * heads_ * S_);
      ao_[l] = ws.take<bf16_t>(R * d_); pre1_[l] = ws.take<float>(R * d_); mean1_[l] = ws.take<float>(M); rstd1_[l] = ws.take<float>(M);
      x1_[l] = ws.take<bf16_t>(R * d_); fpre_[l] = ws.take<bf16_t>(R * ffn_); fact_[l] = ws.take<bf16_t>(R * ffn_);
      pre2_[l] = ws.take<float>(R * d_); mean2_[l] = ws.take<float>(M); rstd2_[l] = ws.take<float>(M);
    }
    pre0_ = ws.take<float>(M * d_); mean0_ = ws.take<float>(M); rstd0_ = ws.take<float>(M);
    dX_[0] = ws.take<float>(M * d_); dX_[1] = ws.take<float>(M * d_);
    res_[0] = ws.take<float>(2 * M * d_); res_[1] = ws.take<float>(2 * M * d_);
    ds32_ = ws.take<float>(M * d_); do_ = ws.take<bf16_t>(M * d_);
    // What a layer's weight-gradient launches read exists twice (layer parity): they run on a second stream while the
    // next layer's backward chain already writes the other set.
    for (int p = 0; p < 2; ++p) {
      ds16_[p][0] = ws.take<bf16_t>(M * d_); ds16_[p][1] = ws.take<bf16_t>(M * d_);
      dpre_[p] = ws.take<bf16_t>(M * ffn_); dqkv_[p] = ws.take<bf16_t>(M * 3 * d_);
    }
    const size_t nblk = (M + LN_BWD_ROWS - 1) / LN_BWD_ROWS, nrb = (M + COLSUM_ROWS - 1) / COLSUM_ROWS;
    const size_t wide = (size_t)(3 * d_ > ffn_ ? 3 * d_ : ffn_);
    for (int p = 0; p < 2; ++p) {
      lnpart_[p][0] = ws.take<float>(nblk * 3 * d_); lnpart_[p][1] = ws.take<float>(nblk * 3 * d_);
      cspart_[p][0] = ws.take<float>(nrb * wide); cspart_[p][1] = ws.take<float>(nrb * wide);
    }
    if (has_mlm()) {   // masked-token head: P_ positions (a multiple of 64, zero rows beyond the batch's), two stacked passes
      hm_ = ws.take<bf16_t>((size_t)2 * P_ * d_); hm_lo_ = ws.take<bf16_t>((size_t)2 * P_ * d_); zt_ = ws.take<float>((size_t)2 * P_ * V_); lse_pos_ = ws.take<float>((size_t)2 * P_);
      dzt_ = ws.take<bf16_t>((size_t)P_ * V_); dhm_ = ws.take<float>((size_t)GEMM_MAX_BATCH * P_ * d_);
      cs_mlm_ = ws.take<float>((size_t)((P_ + COLSUM_ROWS - 1) / COLSUM_ROWS) * V_);
    }
  }

  // One linear layer of `nw` stacked passes (pass k owns rows [k M, (k + 1) M) of every activation): the same
  // epilogue `e` (its pointers are those of pass 0) for each pass, with that pass's weights.
  void fwd_linear(hipStream_t st, const PassWeights* w, int nw, const bf16_t* A, int K, int64_t woff, int N, int64_t boff, int M,
                  const GemmBf16Args& e) const {
    GemmBf16Args g[2];
    for (int k = 0; k < nw; ++k) {
      g[k] = e;
      const int64_t ro = (int64_t)k * M * N;
      g[k].A = A + (int64_t)k * M * K; g[k].lda = K; g[k].a_trans = 0;
      g[k].B = w[k].hi + woff; g[k].B2 = w[k].lo ? w[k].lo + woff : nullptr; g[k].ldb = K; g[k].b_trans = 1;
      g[k].M = M; g[k].N = N; g[k].K = K; g[k].ldc = N;
      g[k].bias = w[k].theta + boff;
      if (w[k].sign != 0.f) { g[k].bias_v = w[k].vdir + boff; g[k].beps = w[k].eps_ptr; g[k].bsign = w[k].sign; }
      if (e.res32) g[k].res32 = e.res32 + ro;
      if (e.C32) g[k].C32 = e.C32 + ro;
      if (e.C16) g[k].C16 = e.C16 + ro;
      if (e.C16_pre) g[k].C16_pre = e.C16_pre + ro;
    }
    launch_gemm_bf16_batch(st, g, nw);
  }

  // nw = 1: one pass with weights w[0].  nw = 2: the theta + eps v and theta - eps v passes of Eq. 5 on the same
  // batch, stacked along the row dimension (forward only, keep must be false); logits [nw B x C].
  void run_forward(hipStream_t st, const PassWeights* w, int nw, const sama_batch& b, bool keep, float* logits) {
    const int B = b.n, M = B * S_, R = nw * M;
    ParamView pv{w[0].theta, w[0].vdir, w[0].eps_ptr, w[0].sign, nw == 2 ? M : 0};
    LnFwdArgs e{};
    e.x = nullptr; e.ids = (const int32_t*)b.x; e.ids_rows = M; e.S = S_; e.V = V_; e.tok_off = tok_; e.pos_off = pos_; e.x_out = keep ? pre0_ : nullptr;
    e.pv = pv; e.g_off = eg_; e.b_off = eb_; e.y = X_[0]; e.y32 = res_[0]; e.mean = keep ? mean0_ : nullptr; e.rstd = keep ? rstd0_ : nullptr;
    e.M = R; e.d = d_;
    launch_ln_fwd(st, e);
    for (int l = 0; l < L_; ++l) {
      const int s = keep ? l : 0;                       // activation slot: forward-only passes reuse slot 0
      const bf16_t* xin = keep ? X_[l] : X_[l & 1];
      bf16_t* xout = keep ? X_[l + 1] : X_[(l + 1) & 1];
      const LayerOff& o = off_[l];
      GemmBf16Args g{};
      g.C16 = qkv_[s];
      fwd_linear(st, w, nw, xin, d_, o.Wqkv, 3 * d_, o.bqkv, M, g);
      launch_attention_fwd(st, qkv_[s], ao_[s], keep ? lse_[s] : nullptr, nw * B, S_, heads_, d_, b.seq_len, B);
      g = GemmBf16Args{};
      g.res32 = res_[0]; g.C32 = pre1_[s];          // the residual stream stays fp32
      fwd_linear(st, w, nw, ao_[s], d_, o.Wo, d_, o.bo, M, g);
      LnFwdArgs n1{};
      n1.x = pre1_[s]; n1.pv = pv; n1.g_off = o.ln1g; n1.b_off = o.ln1b; n1.y = x1_[s]; n1.y32 = res_[1];
      n1.mean = keep ? mean1_[s] : nullptr; n1.rstd = keep ? rstd1_[s] : nullptr; n1.M = R; n1.d = d_;
      launch_ln_fwd(st, n1);
      g = GemmBf16Args{};
      g.act = GEMM_ACT_GELU_FWD; g.C16_pre = keep ? fpre_[s] : nullptr; g.C16 = fact_[s];   // only a backward pass reads the pre-activation
      fwd_linear(st, w, nw, x1_[s], d_, o.W1, ffn_, o.b1, M, g);
      g = GemmBf16Args{};
      g.res32 = res_[1]; g.C32 = pre2_[s];
      fwd_linear(st, w, nw, fact_[s], ffn_, o.W2, d_, o.b2, M, g);
      LnFwdArgs n2{};
      n2.x = pre2_[s]; n2.pv = pv; n2.g_off = o.ln2g; n2.b_off = o.ln2b; n2.y = xout; n2.y32 = res_[0];
      n2.mean = keep ? mean2_[s] : nullptr; n2.rstd = keep ? rstd2_[s] : nullptr; n2.M = R; n2.d = d_;
      launch_ln_fwd(st, n2);
    }
    pv.flip_row = nw == 2 ? B : 0;                  // the head's rows are samples
    launch_head_fwd(st, res_[0], S_, d_, nw * B, C_, pv, wc_, bc_, logits);   // res_[0] = fp32 output of the last LayerNorm
  }

  void forward(hipStream_t st, const PassWeights& w, const sama_batch& b, bool keep, float* logits) override {
    run_forward(st, &w, 1, b, keep, logits);
  }
  void forward_pair(hipStream_t st, const PassWeights& wp, const PassWeights& wm, const sama_batch& b, float* logits) override {
    const PassWeights w[2] = {wp, wm};
    run_forward(st, w, 2, b, false, logits);
  }

  void mlm_forward(hipStream_t st, const PassWeights* w, int nw, int pass_rows, bool kept, const MlmBatch& mb,
                   float* loss_pos) override {
    // A kept pass (base step) contracts the bf16 hidden states like every other layer.  The +- passes of Eq. 5 feed
    // a loss whose difference is the signal: their hidden states enter as the two-term split of the fp32 LayerNorm
    // output, x_hi (W_hi + W_lo) + x_lo W_hi, so that the rounding of x to bf16 does not bury that difference.
    if (kept) launch_gather_rows(st, X_[L_], pass_rows, mb.row_base, mb.rows_in_batch, mb.rows, mb.n_mask, P_, d_, nw, hm_);
    else launch_gather_rows_split(st, res_[0], pass_rows, mb.row_base, mb.rows_in_batch, mb.rows, mb.n_mask, P_, d_, nw, hm_, hm_lo_);
    GemmBf16Args g{};
    g.C32 = zt_;
    fwd_linear(st, w, nw, hm_, d_, wm_, V_, bm_, P_, g);
    if (!kept) {
      GemmBf16Args lo[2];
      for (int k = 0; k < nw; ++k) {
        lo[k] = GemmBf16Args{};
        lo[k].A = hm_lo_ + (int64_t)k * P_ * d_; lo[k].lda = d_; lo[k].a_trans = 0;
        lo[k].B = w[k].hi + wm_; lo[k].ldb = d_; lo[k].b_trans = 1;
        lo[k].M = P_; lo[k].N = V_; lo[k].K = d_; lo[k].ldc = V_;
        lo[k].res32 = zt_ + (int64_t)k * P_ * V_; lo[k].C32 = zt_ + (int64_t)k * P_ * V_;   // in place: an element is read and written by the same thread
      }
      launch_gemm_bf16_batch(st, lo, nw);
    }
    launch_mlm_ce(st, zt_, V_, P_, mb.tgt, mb.n_mask, nw, loss_pos, lse_pos_);
  }

  // dW[N x K] = dY^T . X into `out`
  GemmBf16Args wgrad(const bf16_t* dY, int N, const bf16_t* X, int K, int M, float* out) const {
    GemmBf16Args g{};
    g.A = dY; g.lda = N; g.a_trans = 1;
    g.B = X; g.ldb = K; g.b_trans = 0;
    g.M = N; g.N = K; g.K = M; g.ldc = K; g.C32 = out;
    return g;
  }
  // dX[M x K] = dY[M x N] . W[N x K]
  GemmBf16Args dgrad(const PassWeights& w, const bf16_t* dY, int N, int64_t woff, int K, int M) const {
    GemmBf16Args g{};
    g.A = dY; g.lda = N; g.a_trans = 0;
    g.B = w.hi + woff; g.B2 = w.lo ? w.lo + woff : nullptr; g.ldb = K; g.b_trans = 0;
    g.M = M; g.N = K; g.K = N; g.ldc = K;
    return g;
  }

  void backward(hipStream_t st, const PassWeights& w, const sama_batch& b, const float* dlogits, float* grad) override {
    run_backward(st, w, b, dlogits, grad, nullptr, nullptr);
  }
  void backward_mlm(hipStream_t st, const PassWeights& w, const sama_batch& b, const float* dlogits, float* grad,
                    const MlmBatch& mb, const float* coef_pos) override {
    run_backward(st, w, b, dlogits, grad, &mb, coef_pos);
  }

  // The masked-token head's backward: dZ = coef (softmax - onehot) in bf16; the hidden-state gradient dZ . Wmlm has a
  // small output and a vocabulary-long contraction, so it runs as up to GEMM_MAX_BATCH K-chunks in one launch whose
  // partial results the scatter adds into the token rows of dx; then dWmlm = dZ^T . H and dbmlm = column sums of dZ.
  void mlm_backward(hipStream_t st, const PassWeights& w, const MlmBatch& mb, const float* coef_pos, float* grad, float* dx) {
    launch_mlm_dz(st, zt_, V_, mb.tgt, coef_pos, lse_pos_, mb.n_mask, P_, dzt_);
    const int slabs = V_ / 64, np = slabs < GEMM_MAX_BATCH ? slabs : GEMM_MAX_BATCH;
    GemmBf16Args g[GEMM_MAX_BATCH];
    for (int k = 0; k < np; ++k) {
      const int64_t k0 = (int64_t)(slabs * k / np) * 64, k1 = (int64_t)(slabs * (k + 1) / np) * 64;
      g[k] = GemmBf16Args{};
      g[k].A = dzt_ + k0; g[k].lda = V_; g[k].a_trans = 0;
      g[k].B = w.hi + wm_ + k0 * d_; g[k].B2 = w.lo ? w.lo + wm_ + k0 * d_ : nullptr; g[k].ldb = d_; g[k].b_trans = 0;
      g[k].M = P_; g[k].N = d_; g[k].K = (int)(k1 - k0); g[k].ldc = d_;
      g[k].C32 = dhm_ + (int64_t)k * P_ * d_;
    }
    launch_gemm_bf16_batch(st, g, np);
    launch_scatter_add_rows(st, dhm_, np, (int64_t)P_ * d_, mb.row_base, mb.rows_in_batch, mb.rows, mb.n_mask, d_, dx);
    launch_gemm_bf16(st, wgrad(dzt_, V_, hm_, d_, P_, grad + wm_));
    launch_colsum_bf16(st, dzt_, P_, V_, cs_mlm_, grad + bm_);
  }

  void run_backward(hipStream_t st, const PassWeights& w, const sama_batch& b, const float* dlogits, float* grad,
                    const MlmBatch* mb, const float* coef_pos) {
    const int B = b.n, M = B * S_;
    const int nblk = (M + LN_BWD_ROWS - 1) / LN_BWD_ROWS;
    float* dx = dX_[0];
    float* dx_next = dX_[1];
    launch_fill_f32(st, dx, 0.f, (int64_t)M * d_);
    launch_head_bwd(st, res_[0], S_, d_, B, C_, w.theta, wc_, bc_, dlogits, grad, dx);
    if (mb) mlm_backward(st, w, *mb, coef_pos, grad, dx);
    else if (has_mlm()) {   // a loss without masked-token terms leaves the head's gradient at zero
      launch_fill_f32(st, grad + wm_, 0.f, (int64_t)V_ * d_);
      launch_fill_f32(st, grad + bm_, 0.f, V_);
    }
    // The layer's four weight gradients, its two bias column sums and its four small reductions leave in three
    // launches at the end of the layer, on a second stream of the same priority: nothing in the backward chain
    // depends on them, and the chain's launches (small dgrad tiles, LayerNorm, attention) leave room on the CUs.
    // Their inputs alternate between two buffer sets; the chain waits for the launches of two layers ago before it
    // overwrites a set, and the pass ends with both streams joined.
    const bool two = side_enabled() && ensure_side();
    hipStream_t ss = two ? side_ : st;
    bool sink_used = false;
    for (int l = L_ - 1; l >= 0; --l) {
      const LayerOff& o = off_[l];
      const int p = l & 1;
      if (two && side_busy_[p]) { (void)hipStreamWaitEvent(st, ev_side_[p], 0); side_busy_[p] = false; }
      bf16_t* const ds2 = ds16_[p][0]; bf16_t* const ds1 = ds16_[p][1]; bf16_t* const dpre = dpre_[p]; bf16_t* const dqkv = dqkv_[p];
      GemmBf16Args wg[4];
      // LN2
      LnBwdArgs n2{dx, pre2_[l], mean2_[l], rstd2_[l], w.theta + o.ln2g, ds32_, ds2, lnpart_[p][0], M, d_};
      launch_ln_bwd(st, n2);
      // FFN
      wg[0] = wgrad(ds2, d_, fact_[l], ffn_, M, grad + o.W2);
      GemmBf16Args g = dgrad(w, ds2, d_, o.W2, ffn_, M);
      g.act = GEMM_ACT_GELU_BWD; g.aux16 = fpre_[l]; g.C16 = dpre;
      launch_gemm_bf16(st, g);
      wg[1] = wgrad(dpre, ffn_, x1_[l], d_, M, grad + o.W1);
      g = dgrad(w, dpre, ffn_, o.W1, d_, M);
      g.res32 = ds32_; g.C32 = dx_next;                       // + the residual branch
      launch_gemm_bf16(st, g);
      // LN1
      LnBwdArgs n1{dx_next, pre1_[l], mean1_[l], rstd1_[l], w.theta + o.ln1g, ds32_, ds1, lnpart_[p][1], M, d_};
      launch_ln_bwd(st, n1);
      // attention
      wg[2] = wgrad(ds1, d_, ao_[l], d_, M, grad + o.Wo);
      g = dgrad(w, ds1, d_, o.Wo, d_, M);
      g.C16 = do_;
      launch_gemm_bf16(st, g);
      launch_attention_bwd(st, qkv_[l], ao_[l], do_, lse_[l], dqkv, B, S_, heads_, d_, b.seq_len, B);
      wg[3] = wgrad(dqkv, 3 * d_, X_[l], d_, M, grad + o.Wqkv);
      g = dgrad(w, dqkv, 3 * d_, o.Wqkv, d_, M);
      g.res32 = ds32_; g.C32 = dx;                            // gradient w.r.t. the layer input
      if (two) {   // everything the side launches read is written by now (the last dgrad only reads dqkv)
        (void)hipEventRecord(ev_chain_[p], st);
        (void)hipStreamWaitEvent(side_, ev_chain_[p], 0);
      }
      launch_gemm_bf16(st, g);
      const bool sink_now = two && g_side_sink && sink_ != nullptr;
      if (sink_now) (void)hipEventRecord(ev_last_[p], st);   // behind the layer's last read of its own weights
      launch_gemm_bf16_batch(ss, wg, 4);
      const ColsumJob cj[2] = {{dpre, M, ffn_, cspart_[p][0]}, {dqkv, M, 3 * d_, cspart_[p][1]}};
      launch_colsum_partial_multi(ss, cj, 2);
      const int nrb = (M + COLSUM_ROWS - 1) / COLSUM_ROWS;
      const ReduceRowsJob rj[4] = {
          {lnpart_[p][0], nblk, 3 * d_, d_, d_, {grad + o.ln2g, grad + o.ln2b, grad + o.b2}},
          {lnpart_[p][1], nblk, 3 * d_, d_, d_, {grad + o.ln1g, grad + o.ln1b, grad + o.bo}},
          {cspart_[p][0], nrb, ffn_, 0, ffn_, {grad + o.b1, nullptr, nullptr}},
          {cspart_[p][1], nrb, 3 * d_, 0, 3 * d_, {grad + o.bqkv, nullptr, nullptr}}};
      launch_reduce_rows_multi(ss, rj, 4);
      if (two) { (void)hipEventRecord(ev_side_[p], side_); side_busy_[p] = true; }
      if (sink_now) {   // this layer's gradients are final (matrices and vectors are one range each); a consumer may
        (void)hipStreamWaitEvent(side_, ev_last_[p], 0);   // overwrite the layer's weights once its last dgrad has read them
        sink_->ready(side_, o.Wqkv, (int64_t)4 * d_ * d_ + (int64_t)2 * ffn_ * d_);
        sink_->ready(side_, o.bqkv, (int64_t)9 * d_ + ffn_);
        sink_used = true;
      }
    }
    if (sink_used) { (void)hipEventRecord(ev_side_[0], side_); side_busy_[0] = true; }   // join behind the consumer's work too
    for (int p = 0; p < 2; ++p)
      if (two && side_busy_[p]) { (void)hipStreamWaitEvent(st, ev_side_[p], 0); side_busy_[p] = false; }
    LnBwdArgs n0{dx, pre0_, mean0_, rstd0_, w.theta + eg_, ds32_, nullptr, lnpart_[0][0], M, d_};
    launch_ln_bwd(st, n0);
    launch_reduce_rows(st, lnpart_[0][0], nblk, 3 * d_, d_, d_, grad + eg_, grad + eb_, nullptr);
    launch_fill_f32(st, grad + tok_, 0.f, (int64_t)V_ * d_);
    launch_embedding_bwd(st, ds32_, (const int32_t*)b.x, B, S_, d_, V_, grad + tok_, grad + pos_);
  }

  // second stream (default priority, created at the first backward pass) and the events that order it
  bool ensure_side() {
    if (side_ != nullptr) return true;
    if (side_failed_) return false;
    bool ok = hipStreamCreateWithFlags(&side_, hipStreamNonBlocking) == hipSuccess;
    for (int p = 0; p < 2 && ok; ++p)
      ok = hipEventCreateWithFlags(&ev_chain_[p], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&ev_side_[p], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&ev_last_[p], hipEventDisableTiming) == hipSuccess;
    if (!ok) { release_side(); side_failed_ = true; (void)hipGetLastError(); }
    return ok;
  }
  void release_side() {
    for (int p = 0; p < 2; ++p) {
      if (ev_chain_[p]) (void)hipEventDestroy(ev_chain_[p]);
      if (ev_side_[p]) (void)hipEventDestroy(ev_side_[p]);
      if (ev_last_[p]) (void)hipEventDestroy(ev_last_[p]);
      ev_chain_[p] = ev_side_[p] = ev_last_[p] = nullptr;
    }
    if (side_) (void)hipStreamDestroy(side_);
    side_ = nullptr;
  }
  ~EncoderModel() override { release_side(); }

 private:
  int L_, d_, heads_, ffn_, S_, V_, C_;
  std::vector<LayerOff> off_;
  int64_t tok_, pos_, eg_, eb_, wc_, bc_, wm_, bm_;
  int P_ = 0;   // masked-token head: padded maximum number of positions
  bf16_t* hm_ = nullptr; bf16_t* hm_lo_ = nullptr; float* zt_ = nullptr; float* lse_pos_ = nullptr; bf16_t* dzt_ = nullptr; float* dhm_ = nullptr;
  float* cs_mlm_ = nullptr;
  std::vector<bf16_t*> X_, qkv_, ao_, x1_, fpre_, fact_;
  std::vector<float*> lse_, pre1_, mean1_, rstd1_, pre2_, mean2_, rstd2_;
  float *pre0_ = nullptr, *mean0_ = nullptr, *rstd0_ = nullptr;
  float* dX_[2] = {nullptr, nullptr};
  float* res_[2] = {nullptr, nullptr};   // fp32 LayerNorm outputs: the residual stream of the current forward pass
  float* ds32_ = nullptr; bf16_t* do_ = nullptr;
  bf16_t* ds16_[2][2] = {}; bf16_t* dpre_[2] = {}; bf16_t* dqkv_[2] = {};   // [layer parity]
  float* lnpart_[2][2] = {}; float* cspart_[2][2] = {};
  hipStream_t side_ = nullptr; hipEvent_t ev_chain_[2] = {}, ev_side_[2] = {}, ev_last_[2] = {};
  bool side_busy_[2] = {false, false}, side_failed_ = false;
};
}  // namespace

Model* make_encoder(const sama_config& c, const std::vector<TensorInfo>& layout, std::string& err) {
  const int d = c.dims[1], heads = c.dims[2], ffn = c.dims[3], S = c.dims[4];
  if (!attention_supports(S)) { err = "the encoder kernels are built for S = 64, 128 or 256"; return nullptr; }
  if (d / heads != 64 || d % heads != 0) { err = "the attention kernels are built for head width d/heads = 64"; return nullptr; }
  if (d > LN_MAX_D) { err = "d must be <= 2048"; return nullptr; }
  if (ffn % 64 != 0) { err = "ffn must be a multiple of 64"; return nullptr; }
  const int tb = c.max_batch + (c.aux_mlm ? c.max_aux_batch : 0);
  const int mb = tb > c.max_meta_batch ? tb : c.max_meta_batch;
  if ((int64_t)mb * S > MAX_TOKENS) { err = "max batch (+ max auxiliary batch) * S must be <= 8192 tokens"; return nullptr; }
  if (c.aux_mlm && c.dims[5] % 64 != 0) { err = "the masked-token head needs a vocabulary size that is a multiple of 64"; return nullptr; }
  return new EncoderModel(c, layout);
}

}  // namespace sama
