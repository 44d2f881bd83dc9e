// Post-LN transformer encoder classifier in bf16 with fp32 accumulation: the explicit forward / backward kernel
// sequence (no autograd).  x0 = LN(tok[ids] + pos); per layer x <- LN1(x + Attn(x)), x <- LN2(x + FFN(x));
// logits = x_L[:, 0] Wc^T + bc.  Residual sums and every LayerNorm input stay fp32; GEMM operands are bf16.
#include "kernels.h"
#include "model.h"

namespace sama {
namespace {

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
  }
  int n_classes() const override { return C_; }

  void plan(BumpAlloc& ws, int max_b) override {
    const size_t M = (size_t)max_b * S_;
    X_.resize(L_ + 1); qkv_.resize(L_); lse_.resize(L_); ao_.resize(L_); pre1_.resize(L_); mean1_.resize(L_); rstd1_.resize(L_);
    x1_.resize(L_); fpre_.resize(L_); fact_.resize(L_); pre2_.resize(L_); mean2_.resize(L_); rstd2_.resize(L_);
    for (int l = 0; l <= L_; ++l) X_[l] = ws.take<bf16_t>(M * d_);
    for (int l = 0; l < L_; ++l) {
      qkv_[l] = ws.take<bf16_t>(M * 3 * d_); lse_[l] = ws.take<float>((size_t)max_b * heads_ * S_);
      ao_[l] = ws.take<bf16_t>(M * d_); pre1_[l] = ws.take<float>(M * d_); mean1_[l] = ws.take<float>(M); rstd1_[l] = ws.take<float>(M);
      x1_[l] = ws.take<bf16_t>(M * d_); fpre_[l] = ws.take<bf16_t>(M * ffn_); fact_[l] = ws.take<bf16_t>(M * ffn_);
      pre2_[l] = ws.take<float>(M * d_); mean2_[l] = ws.take<float>(M); rstd2_[l] = ws.take<float>(M);
    }
    pre0_ = ws.take<float>(M * d_); mean0_ = ws.take<float>(M); rstd0_ = ws.take<float>(M);
    dX_[0] = ws.take<float>(M * d_); dX_[1] = ws.take<float>(M * d_);
    res_[0] = ws.take<float>(M * d_); res_[1] = ws.take<float>(M * d_);
    ds32_ = ws.take<float>(M * d_); ds16_ = ws.take<bf16_t>(M * d_);
    dpre_ = ws.take<bf16_t>(M * ffn_); do_ = ws.take<bf16_t>(M * d_); dqkv_ = ws.take<bf16_t>(M * 3 * d_);
    const size_t nblk = (M + LN_BWD_ROWS - 1) / LN_BWD_ROWS, nrb = (M + COLSUM_ROWS - 1) / COLSUM_ROWS;
    const size_t wide = (size_t)(3 * d_ > ffn_ ? 3 * d_ : ffn_);
    lnpart_ = ws.take<float>(nblk * 3 * d_);
    cspart_ = ws.take<float>(nrb * wide);
  }

  GemmBf16Args fwd_gemm(const PassWeights& w, const bf16_t* A, int K, int64_t woff, int N, int64_t boff, int M) const {
    GemmBf16Args g{};
    g.A = A; g.lda = K; g.a_trans = 0;
    g.B = w.hi + woff; g.B2 = w.lo ? w.lo + woff : nullptr; g.ldb = K; g.b_trans = 1;
    g.M = M; g.N = N; g.K = K; g.ldc = N;
    g.bias = w.theta + boff;
    if (w.sign != 0.f) { g.bias_v = w.vdir + boff; g.beps = w.eps_ptr; g.bsign = w.sign; }
    return g;
  }

  void forward(hipStream_t st, const PassWeights& w, const sama_batch& b, bool keep, float* logits) override {
    const int B = b.n, M = B * S_;
    const ParamView pv{w.theta, w.vdir, w.eps_ptr, w.sign};
    LnFwdArgs e{};
    e.x = nullptr; e.ids = (const int32_t*)b.x; e.S = S_; e.tok_off = tok_; e.pos_off = pos_; e.x_out = keep ? pre0_ : nullptr;
    e.pv = pv; e.g_off = eg_; e.b_off = eb_; e.y = X_[0]; e.y32 = res_[0]; e.mean = keep ? mean0_ : nullptr; e.rstd = keep ? rstd0_ : nullptr;
    e.M = M; e.d = d_;
    launch_ln_fwd(st, e);
    for (int l = 0; l < L_; ++l) {
      const int s = keep ? l : 0;                       // activation slot: forward-only passes reuse slot 0
      const bf16_t* xin = keep ? X_[l] : X_[l & 1];
      bf16_t* xout = keep ? X_[l + 1] : X_[(l + 1) & 1];
      const LayerOff& o = off_[l];
      GemmBf16Args g = fwd_gemm(w, xin, d_, o.Wqkv, 3 * d_, o.bqkv, M);
      g.C16 = qkv_[s];
      launch_gemm_bf16(st, g);
      launch_attention_fwd(st, qkv_[s], ao_[s], keep ? lse_[s] : nullptr, B, heads_, d_);
      g = fwd_gemm(w, ao_[s], d_, o.Wo, d_, o.bo, M);
      g.res32 = res_[0]; g.C32 = pre1_[s];          // the residual stream stays fp32
      launch_gemm_bf16(st, g);
      LnFwdArgs n1{};
      n1.x = pre1_[s]; n1.pv = pv; n1.g_off = o.ln1g; n1.b_off = o.ln1b; n1.y = x1_[s]; n1.y32 = res_[1];
      n1.mean = keep ? mean1_[s] : nullptr; n1.rstd = keep ? rstd1_[s] : nullptr; n1.M = M; n1.d = d_;
      launch_ln_fwd(st, n1);
      g = fwd_gemm(w, x1_[s], d_, o.W1, ffn_, o.b1, M);
      g.act = GEMM_ACT_GELU_FWD; g.C16_pre = fpre_[s]; g.C16 = fact_[s];
      launch_gemm_bf16(st, g);
      g = fwd_gemm(w, fact_[s], ffn_, o.W2, d_, o.b2, M);
      g.res32 = res_[1]; g.C32 = pre2_[s];
      launch_gemm_bf16(st, g);
      LnFwdArgs n2{};
      n2.x = pre2_[s]; n2.pv = pv; n2.g_off = o.ln2g; n2.b_off = o.ln2b; n2.y = xout; n2.y32 = res_[0];
      n2.mean = keep ? mean2_[s] : nullptr; n2.rstd = keep ? rstd2_[s] : nullptr; n2.M = M; n2.d = d_;
      launch_ln_fwd(st, n2);
    }
    launch_head_fwd(st, res_[0], S_, d_, B, C_, pv, wc_, bc_, logits);   // res_[0] = fp32 output of the last LayerNorm
  }

  // dW[N x K] = dY^T . X into grad + woff
  void wgrad(hipStream_t st, const bf16_t* dY, int N, const bf16_t* X, int K, int M, float* out) const {
    GemmBf16Args g{};
    g.A = dY; g.lda = N; g.a_trans = 1;
    g.B = X; g.ldb = K; g.b_trans = 0;
    g.M = N; g.N = K; g.K = M; g.ldc = K; g.C32 = out;
    launch_gemm_bf16(st, g);
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
    const int B = b.n, M = B * S_;
    const int nblk = (M + LN_BWD_ROWS - 1) / LN_BWD_ROWS;
    float* dx = dX_[0];
    float* dx_next = dX_[1];
    launch_fill_f32(st, dx, 0.f, (int64_t)M * d_);
    launch_head_bwd(st, res_[0], S_, d_, B, C_, w.theta, wc_, bc_, dlogits, grad, dx);
    for (int l = L_ - 1; l >= 0; --l) {
      const LayerOff& o = off_[l];
      // LN2
      LnBwdArgs n2{dx, pre2_[l], mean2_[l], rstd2_[l], w.theta + o.ln2g, ds32_, ds16_, lnpart_, M, d_};
      launch_ln_bwd(st, n2);
      launch_reduce_rows(st, lnpart_, nblk, 3 * d_, d_, d_, grad + o.ln2g, grad + o.ln2b, grad + o.b2);
      // FFN
      wgrad(st, ds16_, d_, fact_[l], ffn_, M, grad + o.W2);
      GemmBf16Args g = dgrad(w, ds16_, d_, o.W2, ffn_, M);
      g.act = GEMM_ACT_GELU_BWD; g.aux16 = fpre_[l]; g.C16 = dpre_;
      launch_gemm_bf16(st, g);
      launch_colsum_bf16(st, dpre_, M, ffn_, cspart_, grad + o.b1);
      wgrad(st, dpre_, ffn_, x1_[l], d_, M, grad + o.W1);
      g = dgrad(w, dpre_, ffn_, o.W1, d_, M);
      g.res32 = ds32_; g.C32 = dx_next;                       // + the residual branch
      launch_gemm_bf16(st, g);
      // LN1
      LnBwdArgs n1{dx_next, pre1_[l], mean1_[l], rstd1_[l], w.theta + o.ln1g, ds32_, ds16_, lnpart_, M, d_};
      launch_ln_bwd(st, n1);
      launch_reduce_rows(st, lnpart_, nblk, 3 * d_, d_, d_, grad + o.ln1g, grad + o.ln1b, grad + o.bo);
      // attention
      wgrad(st, ds16_, d_, ao_[l], d_, M, grad + o.Wo);
      g = dgrad(w, ds16_, d_, o.Wo, d_, M);
      g.C16 = do_;
      launch_gemm_bf16(st, g);
      launch_attention_bwd(st, qkv_[l], ao_[l], do_, lse_[l], dqkv_, B, heads_, d_);
      launch_colsum_bf16(st, dqkv_, M, 3 * d_, cspart_, grad + o.bqkv);
      wgrad(st, dqkv_, 3 * d_, X_[l], d_, M, grad + o.Wqkv);
      g = dgrad(w, dqkv_, 3 * d_, o.Wqkv, d_, M);
      g.res32 = ds32_; g.C32 = dx;                            // gradient w.r.t. the layer input
      launch_gemm_bf16(st, g);
    }
    LnBwdArgs n0{dx, pre0_, mean0_, rstd0_, w.theta + eg_, ds32_, nullptr, lnpart_, M, d_};
    launch_ln_bwd(st, n0);
    launch_reduce_rows(st, lnpart_, nblk, 3 * d_, d_, d_, grad + eg_, grad + eb_, nullptr);
    launch_fill_f32(st, grad + tok_, 0.f, (int64_t)V_ * d_);
    launch_embedding_bwd(st, ds32_, (const int32_t*)b.x, B, S_, d_, grad + tok_, grad + pos_);
  }

 private:
  int L_, d_, heads_, ffn_, S_, V_, C_;
  std::vector<LayerOff> off_;
  int64_t tok_, pos_, eg_, eb_, wc_, bc_;
  std::vector<bf16_t*> X_, qkv_, ao_, x1_, fpre_, fact_;
  std::vector<float*> lse_, pre1_, mean1_, rstd1_, pre2_, mean2_, rstd2_;
  float *pre0_ = nullptr, *mean0_ = nullptr, *rstd0_ = nullptr;
  float* dX_[2] = {nullptr, nullptr};
  float* res_[2] = {nullptr, nullptr};   // fp32 LayerNorm outputs: the residual stream of the current forward pass
  float* ds32_ = nullptr; bf16_t* ds16_ = nullptr; bf16_t* dpre_ = nullptr; bf16_t* do_ = nullptr; bf16_t* dqkv_ = nullptr;
  float* lnpart_ = nullptr; float* cspart_ = nullptr;
};
}  // namespace

Model* make_encoder(const sama_config& c, const std::vector<TensorInfo>& layout, std::string& err) {
  const int d = c.dims[1], heads = c.dims[2], ffn = c.dims[3], S = c.dims[4];
  if (S != 128) { err = "the attention kernels are built for S = 128"; return nullptr; }
  if (d / heads != 64 || d % heads != 0) { err = "the attention kernels are built for head width d/heads = 64"; return nullptr; }
  if (d > LN_MAX_D) { err = "d must be <= 1024"; return nullptr; }
  if (ffn % 64 != 0) { err = "ffn must be a multiple of 64"; return nullptr; }
  const int mb = c.max_batch > c.max_meta_batch ? c.max_batch : c.max_meta_batch;
  if ((int64_t)mb * S > 4096) { err = "max batch * S must be <= 4096 tokens"; return nullptr; }
  return new EncoderModel(c, layout);
}

}  // namespace sama
