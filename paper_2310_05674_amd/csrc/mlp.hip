// ReLU MLP / multinomial logistic regression base learner in fp32: each layer is one forward GEMM with a fused
// bias + ReLU epilogue; backward is one wgrad GEMM, one column sum and one dgrad GEMM with the ReLU gate fused.
#include "kernels.h"
#include "model.h"

namespace sama {
namespace {

class MlpModel : public Model {
 public:
  MlpModel(const sama_config& cfg, const std::vector<TensorInfo>& layout) {
    L_ = cfg.n_dims - 1;
    for (int i = 0; i < cfg.n_dims; ++i) dims_.push_back(cfg.dims[i]);
    for (int l = 0; l < L_; ++l) { woff_.push_back(layout[l].offset); boff_.push_back(layout[L_ + l].offset); }
  }
  void plan(BumpAlloc& ws, int max_b) override {
    act_.assign(L_ + 1, nullptr);
    int wmax = 0;
    for (int l = 1; l < L_; ++l) { act_[l] = ws.take<float>((size_t)max_b * dims_[l]); wmax = dims_[l] > wmax ? dims_[l] : wmax; }
    d_[0] = ws.take<float>((size_t)max_b * (wmax > 0 ? wmax : 1));
    d_[1] = ws.take<float>((size_t)max_b * (wmax > 0 ? wmax : 1));
  }
  int n_classes() const override { return dims_[L_]; }

  void forward(hipStream_t st, const PassWeights& w, const sama_batch& b, bool /*keep*/, float* logits) override {
    const float* in = (const float*)b.x;
    for (int l = 0; l < L_; ++l) {
      GemmF32Args g{};
      g.A = in; g.sa_i = dims_[l]; g.sa_k = 1;
      g.B = w.theta + woff_[l]; g.sb_k = 1; g.sb_j = dims_[l];
      g.bias = w.theta + boff_[l];
      if (w.sign != 0.f) { g.Bv = w.vdir + woff_[l]; g.beps = w.eps_ptr; g.bsign = w.sign; g.bias_v = w.vdir + boff_[l]; }
      g.C = (l == L_ - 1) ? logits : act_[l + 1]; g.ldc = dims_[l + 1];
      g.M = b.n; g.N = dims_[l + 1]; g.K = dims_[l];
      g.relu = (l < L_ - 1);
      launch_gemm_f32(st, g);
      in = g.C;
    }
  }

  void backward(hipStream_t st, const PassWeights& w, const sama_batch& b, const float* dlogits, float* grad) override {
    const float* d = dlogits;
    for (int l = L_ - 1; l >= 0; --l) {
      const float* in = (l == 0) ? (const float*)b.x : act_[l];
      GemmF32Args g{};  // dW[d_{l+1} x d_l] = d^T . in
      g.A = d; g.sa_i = 1; g.sa_k = dims_[l + 1];
      g.B = in; g.sb_k = dims_[l]; g.sb_j = 1;
      g.C = grad + woff_[l]; g.ldc = dims_[l];
      g.M = dims_[l + 1]; g.N = dims_[l]; g.K = b.n;
      launch_gemm_f32(st, g);
      launch_colsum_f32(st, d, dims_[l + 1], b.n, dims_[l + 1], grad + boff_[l]);
      if (l > 0) {
        GemmF32Args h{};  // dprev[B x d_l] = (d . W_l) * (act_l > 0)
        h.A = d; h.sa_i = dims_[l + 1]; h.sa_k = 1;
        h.B = w.theta + woff_[l]; h.sb_k = dims_[l]; h.sb_j = 1;
        float* out = d_[l & 1];
        h.C = out; h.ldc = dims_[l];
        h.M = b.n; h.N = dims_[l]; h.K = dims_[l + 1];
        h.gate = act_[l];
        launch_gemm_f32(st, h);
        d = out;
      }
    }
  }

 private:
  int L_;
  std::vector<int> dims_;
  std::vector<int64_t> woff_, boff_;
  std::vector<float*> act_;
  float* d_[2] = {nullptr, nullptr};
};
}  // namespace

Model* make_mlp(const sama_config& cfg, const std::vector<TensorInfo>& layout) { return new MlpModel(cfg, layout); }

}  // namespace sama
