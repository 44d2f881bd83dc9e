// Base-learner interface used by the SAMA driver: explicit forward / backward kernel sequences, no autograd.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <utility>
#include <vector>
#include "../../include/sama.h"
#include "common.h"

namespace sama {

struct TensorInfo {
  std::string name;
  int64_t offset, rows, cols;
  bool is_matrix;  // a GEMM weight (leading part of theta)
};

// Builds the flat layout table documented in include/sama.h.  Returns false on an invalid config.
bool build_layout(const sama_config& cfg, std::vector<TensorInfo>& out, int64_t& n, int64_t& n_gemm, std::string& err);

// How one pass sees theta.  Non-GEMM tensors: theta[k] + sign * eps * vdir[k].  GEMM weights: fp32 models read
// theta + sign*eps*vdir inside the GEMM loader; bf16 models contract with hi (+ lo when perturbed).
struct PassWeights {
  const float* theta;
  const float* vdir;
  const float* eps_ptr;
  float sign;  // 0 = unperturbed
  const bf16_t* hi;
  const bf16_t* lo;  // null when unperturbed
};

class BumpAlloc {  // carves 256-byte aligned pieces out of the caller's workspace (base may be null to measure)
 public:
  explicit BumpAlloc(void* base) : base_((char*)base), off_(0) {}
  template <typename T>
  T* take(size_t count) {
    size_t bytes = (count * sizeof(T) + 255) & ~(size_t)255;
    T* p = base_ ? (T*)(base_ + off_) : nullptr;
    off_ += bytes;
    return p;
  }
  size_t used() const { return off_; }

 private:
  char* base_;
  size_t off_;
};

// Masked-token positions of an auxiliary-task batch (device arrays; values are clamped into range by the kernels).
struct MlmBatch {
  const int32_t* rows;  // [n_mask] token row (sequence * S + position) inside the auxiliary sequences, all distinct
  const int32_t* tgt;   // [n_mask] target token ids
  int n_mask;
  int row_base;         // token row of the first auxiliary sequence within the batch the model ran on
  int rows_in_batch;    // token rows of the auxiliary sequences (n_pt * S)
};

// A consumer of finished gradient ranges.  A model that runs part of its backward pass on a stream of its own may
// call ready() there as soon as grad[off, off + count) is final, so that the consumer's work on that range (the
// optimizer update of a layer) overlaps with the rest of the pass; the consumer may overwrite the parameters of that
// range (the pass no longer reads them).  Everything enqueued by ready() is complete, in stream order, when the
// stream backward() was called with continues after the pass.  Ranges never reported are the caller's to handle.
struct GradSink {
  virtual ~GradSink() {}
  virtual void ready(hipStream_t s, int64_t off, int64_t count) = 0;
};

class Model {
 public:
  virtual ~Model() {}
  void set_grad_sink(GradSink* s) { sink_ = s; }   // for the next backward() / backward_mlm(); null = none
  // carve activation buffers for batches up to max_b
  virtual void plan(BumpAlloc& ws, int max_b) = 0;
  // logits[B x C] (fp32, row stride C) for batch `b`; keep = retain what backward needs
  virtual void forward(hipStream_t st, const PassWeights& w, const sama_batch& b, bool keep, float* logits) = 0;
  // The theta + eps v and theta - eps v passes of Eq. 5 on the same batch, forward only: logits [2B x C], the + pass
  // first.  Models that gain from it run the two passes stacked in the same launches.
  virtual void forward_pair(hipStream_t st, const PassWeights& wp, const PassWeights& wm, const sama_batch& b, float* logits) {
    forward(st, wp, b, false, logits);
    forward(st, wm, b, false, logits + (size_t)b.n * n_classes());
  }
  // grad[n] = d/dtheta sum_i sum_c dlogits[i][c] z_ic, at the unperturbed theta of the last keep=true forward
  virtual void backward(hipStream_t st, const PassWeights& w, const sama_batch& b, const float* dlogits, float* grad) = 0;
  virtual int n_classes() const = 0;
  // ---- masked-token head (models built with one)
  virtual bool has_mlm() const { return false; }
  virtual int mlm_stride() const { return 0; }   // positions per pass in loss_pos (the padded maximum)
  // loss_pos[k * mlm_stride() + j] = masked-token loss of position j under pass k (k < nw) of the last forward
  // (kept = true, nw = 1) or forward_pair (kept = false, nw = 2); pass_rows = token rows of one pass.
  virtual void mlm_forward(hipStream_t, const PassWeights*, int /*nw*/, int /*pass_rows*/, bool /*kept*/, const MlmBatch&,
                           float* /*loss_pos*/) {}
  // backward() with the head's loss added: grad = d/dtheta [sum dlogits . z + sum_j coef_pos[j] loss_pos_j], after a
  // kept forward and mlm_forward on the same batch
  virtual void backward_mlm(hipStream_t, const PassWeights&, const sama_batch&, const float* /*dlogits*/, float* /*grad*/,
                            const MlmBatch&, const float* /*coef_pos*/) {}
 protected:
  GradSink* sink_ = nullptr;
};

Model* make_mlp(const sama_config& cfg, const std::vector<TensorInfo>& layout);
Model* make_encoder(const sama_config& cfg, const std::vector<TensorInfo>& layout, std::string& err);

}  // namespace sama
