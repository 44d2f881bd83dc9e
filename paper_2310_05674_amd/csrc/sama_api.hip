// C ABI of libsama (include/sama.h): context, workspace carving, and the kernel sequence of one SAMA
// iteration (Sec. 3.2, Eq. 5; workflow of Fig. 2) on one HIP stream.
#include <math.h>
#include <stdio.h>
#include <string.h>
#include <algorithm>
#include <memory>
#include <utility>
#include <vector>
#include "kernels.h"
#include "model.h"

using namespace sama;

namespace sama {

bool build_layout(const sama_config& c, std::vector<TensorInfo>& out, int64_t& n, int64_t& n_gemm, std::string& err) {
  out.clear();
  std::vector<TensorInfo> mats, vecs;
  auto M = [&](const std::string& nm, int64_t r, int64_t cc) { mats.push_back({nm, 0, r, cc, true}); };
  auto V = [&](const std::string& nm, int64_t r, int64_t cc) { vecs.push_back({nm, 0, r, cc, false}); };
  if (c.model_kind == SAMA_MODEL_MLP) {
    if (c.n_dims < 2 || c.n_dims > 8) { err = "MLP needs 2..8 dims"; return false; }
    for (int i = 0; i < c.n_dims; ++i)
      if (c.dims[i] < 1) { err = "MLP widths must be positive"; return false; }
    if (c.dims[c.n_dims - 1] < 2 || c.dims[c.n_dims - 1] > 64) { err = "class count must be 2..64"; return false; }
    for (int l = 0; l + 1 < c.n_dims; ++l) {
      M("W" + std::to_string(l), c.dims[l + 1], c.dims[l]);
      V("b" + std::to_string(l), c.dims[l + 1], 1);
    }
  } else if (c.model_kind == SAMA_MODEL_ENCODER) {
    if (c.n_dims != 7) { err = "ENCODER needs dims = {L, d, heads, ffn, S, V, C}"; return false; }
    const int64_t L = c.dims[0], d = c.dims[1], heads = c.dims[2], ffn = c.dims[3], S = c.dims[4], Vv = c.dims[5], C = c.dims[6];
    if (L < 1 || d < 1 || heads < 1 || ffn < 1 || S < 1 || Vv < 1 || C < 2 || C > 64 || d % heads != 0) {
      err = "bad ENCODER dims"; return false;
    }
    for (int64_t l = 0; l < L; ++l) {
      const std::string p = "l" + std::to_string(l) + ".";
      M(p + "Wqkv", 3 * d, d); M(p + "Wo", d, d); M(p + "W1", ffn, d); M(p + "W2", d, ffn);
      V(p + "bqkv", 3 * d, 1); V(p + "bo", d, 1); V(p + "ln1_g", d, 1); V(p + "ln1_b", d, 1);
      V(p + "b1", ffn, 1); V(p + "b2", d, 1); V(p + "ln2_g", d, 1); V(p + "ln2_b", d, 1);
    }
    V("tok_emb", Vv, d); V("pos_emb", S, d); V("emb_ln_g", d, 1); V("emb_ln_b", d, 1);
    if (c.aux_mlm) { M("Wmlm", Vv, d); V("bmlm", Vv, 1); }   // masked-token head of the auxiliary task (bmlm 16-byte aligned)
    V("Wc", C, d); V("bc", C, 1);
  } else {
    err = "unknown model_kind"; return false;
  }
  int64_t off = 0;
  for (auto& t : mats) { t.offset = off; off += t.rows * t.cols; out.push_back(t); }
  n_gemm = off;
  for (auto& t : vecs) { t.offset = off; off += t.rows * t.cols; out.push_back(t); }
  n = off;
  return true;
}

}  // namespace sama

struct sama_ctx {
  sama_config cfg;
  hipStream_t stream;
  std::vector<TensorInfo> layout;
  int64_t n, n_gemm;
  int nl;
  bool bf16;
  std::unique_ptr<Model> model;
  // device state (inside the caller's workspace)
  float *theta, *m, *v, *g, *gmeta, *vdir;
  bf16_t *theta16, *lo_0, *lo_p, *lo_m;   // bf16 working copy; residual half of the current theta; halves of theta +- eps v
  float *lambda, *meta_m, *meta_v, *hyper, *glam_p32, *glam_m32;
  double *glam_p, *glam_m, *partial, *corr_scratch;
  float* scalars;     // {eps, ||v||, L_base, L_meta}
  float* step;        // step-dependent optimizer scalars (launch_step_scalars)
  int64_t* counters;  // {t (mirror), meta_t, status, 0}
  float *logits, *dlogits, *losses;
  // auxiliary task: concatenated [ft | pt] batch, per-position losses (two stacked passes) and coefficients
  int32_t *ids_cat, *y_cat, *len_cat; uint8_t* mask_cat; float *loss_pos, *coef_pos;
  int64_t t;  // base step count (host)
  float lr_step = 0.f;           // base_lr of the last base step (a schedule may have moved cfg.base_lr since)
  std::string err;
};

static thread_local std::string g_init_err;

// largest number of samples / sequences one pass runs over
static int max_rows(const sama_config& c) {
  const int tb = c.max_batch + (c.aux_mlm ? c.max_aux_batch : 0);
  return tb > c.max_meta_batch ? tb : c.max_meta_batch;
}

static int lambda_count(const sama_config& c) {
  const int C = c.dims[c.n_dims - 1], Hc = c.corr_hidden;
  return 3 * c.wnet_hidden + 1 + (Hc > 0 ? Hc * 2 * C + Hc + C * Hc + C : 0);
}

static bool validate(const sama_config* c, std::string& err) {
  if (!c) { err = "null config"; return false; }
  std::vector<TensorInfo> lay; int64_t n, ng;
  if (!build_layout(*c, lay, n, ng, err)) return false;
  if (c->wnet_hidden < 1 || c->wnet_hidden > MAX_WNET_HIDDEN) { err = "wnet_hidden must be 1..256"; return false; }
  if (c->max_batch < 1 || c->max_batch > MAX_BATCH || c->max_meta_batch < 1 || c->max_meta_batch > MAX_BATCH) {
    err = "max_batch / max_meta_batch must be 1..2048"; return false;
  }
  if (c->model_kind == SAMA_MODEL_MLP && c->param_dtype != SAMA_DTYPE_FP32) { err = "the MLP runs in fp32"; return false; }
  if (c->model_kind == SAMA_MODEL_ENCODER && c->param_dtype != SAMA_DTYPE_BF16) { err = "the encoder runs in bf16"; return false; }
  if (c->base_opt != SAMA_OPT_SGD && c->base_opt != SAMA_OPT_ADAM) { err = "unknown base_opt"; return false; }
  if (c->adapt_mode != SAMA_ADAPT_OPTIMIZER && c->adapt_mode != SAMA_ADAPT_NONE) { err = "unknown adapt_mode"; return false; }
  if (!(c->base_lr > 0.f) || !(c->meta_lr > 0.f) || !(c->alpha > 0.f)) { err = "base_lr, meta_lr, alpha must be > 0"; return false; }
  if (!(c->beta1 >= 0.f && c->beta1 < 1.f && c->beta2 >= 0.f && c->beta2 < 1.f && c->meta_beta1 >= 0.f &&
        c->meta_beta1 < 1.f && c->meta_beta2 >= 0.f && c->meta_beta2 < 1.f)) { err = "betas must be in [0, 1)"; return false; }
  if (c->fast_meta_pass != 0 && c->fast_meta_pass != 1) { err = "fast_meta_pass must be 0 or 1"; return false; }
  if (c->fast_base_pass != 0 && c->fast_base_pass != 1) { err = "fast_base_pass must be 0 or 1"; return false; }
  if (!(c->momentum >= 0.f && c->momentum < 1.f)) { err = "momentum must be in [0, 1)"; return false; }
  if (c->momentum != 0.f && c->base_opt != SAMA_OPT_SGD) { err = "momentum belongs to the SGD base solver"; return false; }
  if (c->adam_eps < 0.f || c->meta_eps < 0.f || c->weight_decay < 0.f) { err = "negative eps / weight_decay"; return false; }
  if (c->corr_hidden < 0 || c->corr_hidden > MAX_CORR_HIDDEN) { err = "corr_hidden must be 0..128"; return false; }
  if (c->corr_hidden > 0 && c->dims[c->n_dims - 1] > MAX_CORR_CLASSES) { err = "label correction supports at most 16 classes"; return false; }
  if (c->corr_hidden > 0 && !(c->corr_kappa >= 0.f)) { err = "corr_kappa must be >= 0"; return false; }
  if (c->aux_mlm != 0) {
    if (c->aux_mlm != 1) { err = "aux_mlm must be 0 or 1"; return false; }
    if (c->model_kind != SAMA_MODEL_ENCODER) { err = "aux_mlm needs the ENCODER model"; return false; }
    if (c->corr_hidden > 0) { err = "aux_mlm cannot be combined with label correction"; return false; }
    if (c->max_aux_batch < 1) { err = "max_aux_batch must be >= 1"; return false; }
    if (c->max_aux_masked < 1 || (int64_t)c->max_aux_masked > (int64_t)c->max_aux_batch * c->dims[4]) {
      err = "max_aux_masked must be 1..max_aux_batch * S"; return false;
    }
  }
  return true;
}

// Carves the workspace; with ctx->* pointers null-based when base == nullptr (size query).
static size_t carve(sama_ctx* c, void* base) {
  BumpAlloc ws(base);
  const int64_t n = c->n, ng = c->n_gemm;
  const int nl = c->nl;
  c->theta = ws.take<float>(n); c->m = ws.take<float>(n); c->v = ws.take<float>(n);
  c->g = ws.take<float>(n); c->gmeta = ws.take<float>(n); c->vdir = ws.take<float>(n);
  if (c->bf16) { c->theta16 = ws.take<bf16_t>(ng); c->lo_0 = ws.take<bf16_t>(ng); c->lo_p = ws.take<bf16_t>(ng); c->lo_m = ws.take<bf16_t>(ng); }
  else { c->theta16 = c->lo_0 = c->lo_p = c->lo_m = nullptr; }
  c->lambda = ws.take<float>(nl); c->meta_m = ws.take<float>(nl); c->meta_v = ws.take<float>(nl);
  c->hyper = ws.take<float>(nl); c->glam_p32 = ws.take<float>(nl); c->glam_m32 = ws.take<float>(nl);
  c->glam_p = ws.take<double>(nl); c->glam_m = ws.take<double>(nl);
  c->partial = ws.take<double>(EW_MAX_BLOCKS);
  c->scalars = ws.take<float>(4);
  c->step = ws.take<float>(8);
  c->counters = ws.take<int64_t>(4);
  const int mb = max_rows(c->cfg);
  const int C = c->cfg.dims[c->cfg.n_dims - 1];
  c->logits = ws.take<float>((size_t)2 * mb * C);   // room for the stacked + and - passes
  c->dlogits = ws.take<float>((size_t)mb * C);
  c->losses = ws.take<float>(mb);
  c->corr_scratch = c->cfg.corr_hidden > 0 ? ws.take<double>((size_t)c->cfg.max_batch * 2 * C) : nullptr;
  if (c->cfg.aux_mlm) {
    const size_t P = (size_t)(c->cfg.max_aux_masked + 63) / 64 * 64;
    c->ids_cat = ws.take<int32_t>((size_t)mb * c->cfg.dims[4]); c->y_cat = ws.take<int32_t>(mb); c->len_cat = ws.take<int32_t>(mb); c->mask_cat = ws.take<uint8_t>(mb);
    c->loss_pos = ws.take<float>(2 * P); c->coef_pos = ws.take<float>(P);
  } else {
    c->ids_cat = c->y_cat = c->len_cat = nullptr; c->mask_cat = nullptr; c->loss_pos = c->coef_pos = nullptr;
  }
  if (c->model) c->model->plan(ws, mb);
  return ws.used();
}

static sama_ctx* make_host_ctx(const sama_config* cfg, std::string& err) {
  if (!validate(cfg, err)) return nullptr;
  std::unique_ptr<sama_ctx> c(new sama_ctx());
  c->cfg = *cfg;
  build_layout(*cfg, c->layout, c->n, c->n_gemm, err);
  c->nl = lambda_count(*cfg);
  c->bf16 = cfg->param_dtype == SAMA_DTYPE_BF16;
  if (cfg->model_kind == SAMA_MODEL_MLP) c->model.reset(make_mlp(*cfg, c->layout));
  else c->model.reset(make_encoder(*cfg, c->layout, err));
  if (!c->model) return nullptr;
  c->t = 0;
  c->stream = nullptr;
  return c.release();
}

static sama_status fail(sama_ctx* c, sama_status s, const std::string& msg) {
  if (c) c->err = msg; else g_init_err = msg;
  return s;
}
static sama_status check_hip(sama_ctx* c, const char* what) {
  if (const char* le = take_launch_error()) return fail(c, SAMA_EINVAL, std::string(what) + ": a kernel was not launched: " + le);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, SAMA_EHIP, std::string(what) + ": " + hipGetErrorString(e));
  return SAMA_OK;
}
static sama_status check_batch(sama_ctx* c, const sama_batch* b, int maxb, const char* nm) {
  if (!b || !b->x || !b->y) return fail(c, SAMA_EINVAL, std::string(nm) + ": null batch / x / y");
  if (b->n < 1 || b->n > maxb) return fail(c, SAMA_EINVAL, std::string(nm) + ": batch size outside 1..max_batch");
  return SAMA_OK;
}

// The base solver's update (App. C for Adam) of theta[off, off + count) with the gradient in c->g, for step number t.
static void base_update_range(sama_ctx* c, hipStream_t st, int64_t t, int64_t off, int64_t count) {
  if (count <= 0) return;
  const sama_config& f = c->cfg;
  const int64_t n16 = off < c->n_gemm ? (off + count <= c->n_gemm ? count : c->n_gemm - off) : 0;   // leading part with a bf16 copy
  bf16_t* t16 = (c->theta16 != nullptr && n16 > 0) ? c->theta16 + off : nullptr;
  bf16_t* lo0 = t16 != nullptr ? c->lo_0 + off : nullptr;   // every pass that writes theta keeps its residual half current
  if (f.base_opt == SAMA_OPT_ADAM) {
    AdamArgs a{};
    a.beta1 = f.beta1; a.one_m_beta1 = (float)(1.0 - (double)f.beta1);
    a.beta2 = f.beta2; a.one_m_beta2 = (float)(1.0 - (double)f.beta2);
    a.lr_c1 = (float)((double)f.base_lr / (1.0 - pow((double)f.beta1, (double)t)));
    a.c2 = (float)(1.0 / sqrt(1.0 - pow((double)f.beta2, (double)t)));
    a.eps = f.adam_eps; a.weight_decay = f.weight_decay;
    a.dev = c->step;   // the device's own step count decides (the host values above are what it holds in eager use)
    a.lo = lo0;
    launch_adam(st, c->g + off, c->m + off, c->v + off, c->theta + off, t16, count, n16, a);
  } else {
    launch_sgd(st, c->g + off, c->m + off, c->theta + off, t16, lo0, count, n16, f.base_lr, f.weight_decay, f.momentum);
  }
}

// Updates the ranges of theta whose gradients the model reports final while its backward pass still runs.
struct UpdateSink : GradSink {
  sama_ctx* c; int64_t t;
  std::vector<std::pair<int64_t, int64_t>> done;
  UpdateSink(sama_ctx* c_, int64_t t_) : c(c_), t(t_) {}
  void ready(hipStream_t s, int64_t off, int64_t count) override {
    if (off % 4 != 0 || count % 4 != 0 || off < 0 || off + count > c->n) return;   // left to the pass over the rest
    base_update_range(c, s, t, off, count);
    done.push_back({off, count});
  }
};

// Everything the sink has not updated, on the context's stream; advances the step count.
static void base_update_rest(sama_ctx* c, UpdateSink& sink) {
  hipStream_t st = c->stream;
  std::sort(sink.done.begin(), sink.done.end());
  int64_t pos = 0;
  for (auto& r : sink.done) {   // gaps start where a reported range ends (a multiple of 4) or at 0: vector-aligned
    if (r.first > pos) base_update_range(c, st, sink.t, pos, r.first - pos);
    pos = r.first + r.second;
  }
  if (pos < c->n) base_update_range(c, st, sink.t, pos, c->n - pos);
  c->t = sink.t;   // the device's counter was advanced by launch_step_scalars at the start of the step
  c->lr_step = c->cfg.base_lr;
}

// v = D . g_meta and the partial sums of ||v||^2 for the ranges of g_meta the model reports final during its backward
// pass; the partials of successive ranges follow each other in c->partial.
struct AdaptSink : GradSink {
  sama_ctx* c; AdaptArgs ad;
  std::vector<std::pair<int64_t, int64_t>> done;
  int used = 0;                                   // partials handed out so far
  static constexpr int SLICE_BLOCKS = 1024;       // per reported range; leaves most of the EW_MAX_BLOCKS partials to the rest
  AdaptSink(sama_ctx* c_, const AdaptArgs& a) : c(c_), ad(a) {}
  void slice(hipStream_t s, int64_t off, int64_t count, int max_blocks) {
    used += launch_adapt_slice(s, c->g + off, c->m + off, c->v + off, c->gmeta + off, c->vdir + off, c->partial + used, count, ad, max_blocks);
  }
  void ready(hipStream_t s, int64_t off, int64_t count) override {
    if (off % 4 != 0 || count % 4 != 0 || off < 0 || off + count > c->n || used + SLICE_BLOCKS > EW_MAX_BLOCKS / 2) return;
    slice(s, off, count, SLICE_BLOCKS);
    done.push_back({off, count});
  }
};

extern "C" {

int64_t sama_param_count(const sama_config* cfg) {
  std::string e; std::vector<TensorInfo> l; int64_t n, ng;
  if (!cfg || !build_layout(*cfg, l, n, ng, e)) return -1;
  return n;
}
int64_t sama_gemm_param_count(const sama_config* cfg) {
  std::string e; std::vector<TensorInfo> l; int64_t n, ng;
  if (!cfg || !build_layout(*cfg, l, n, ng, e)) return -1;
  return ng;
}
int32_t sama_lambda_count(const sama_config* cfg) {
  std::string err;
  if (!validate(cfg, err)) return 0;
  return lambda_count(*cfg);
}
int32_t sama_param_tensor_count(const sama_config* cfg) {
  std::string e; std::vector<TensorInfo> l; int64_t n, ng;
  if (!cfg || !build_layout(*cfg, l, n, ng, e)) return 0;
  return (int32_t)l.size();
}
sama_status sama_param_tensor(const sama_config* cfg, int32_t idx, char* name_out, int64_t* offset, int64_t* rows,
                              int64_t* cols) {
  std::string e; std::vector<TensorInfo> l; int64_t n, ng;
  if (!cfg || !build_layout(*cfg, l, n, ng, e)) return fail(nullptr, SAMA_EINVAL, e);
  if (idx < 0 || idx >= (int32_t)l.size()) return fail(nullptr, SAMA_EINVAL, "tensor index out of range");
  if (name_out) { strncpy(name_out, l[idx].name.c_str(), 31); name_out[31] = 0; }
  if (offset) *offset = l[idx].offset;
  if (rows) *rows = l[idx].rows;
  if (cols) *cols = l[idx].cols;
  return SAMA_OK;
}

size_t sama_workspace_bytes(const sama_config* cfg) {
  std::string err;
  std::unique_ptr<sama_ctx> c(make_host_ctx(cfg, err));
  if (!c) { g_init_err = err; return 0; }
  return carve(c.get(), nullptr);
}

sama_status sama_init(const sama_config* cfg, void* workspace, size_t workspace_bytes, const float* theta0,
                      const float* lambda0, void* hip_stream, sama_ctx** out) {
  if (!out) return fail(nullptr, SAMA_EINVAL, "null out");
  std::string err;
  std::unique_ptr<sama_ctx> c(make_host_ctx(cfg, err));
  if (!c) return fail(nullptr, SAMA_EINVAL, err);
  if (!theta0 || !lambda0) return fail(nullptr, SAMA_EINVAL, "null theta0 / lambda0");
  if (!workspace || ((uintptr_t)workspace & 255) != 0) return fail(nullptr, SAMA_EWORKSPACE, "workspace null or not 256-byte aligned");
  const size_t need = carve(c.get(), nullptr);
  if (workspace_bytes < need) return fail(nullptr, SAMA_EWORKSPACE, "workspace smaller than sama_workspace_bytes()");
  carve(c.get(), workspace);
  c->stream = (hipStream_t)hip_stream;
  hipStream_t st = c->stream;
  (void)hipGetLastError();
  launch_copy_f32(st, c->theta, theta0, c->n);
  launch_copy_f32(st, c->lambda, lambda0, c->nl);
  launch_fill_f32(st, c->m, 0.f, c->n); launch_fill_f32(st, c->v, 0.f, c->n);
  launch_fill_f32(st, c->g, 0.f, c->n); launch_fill_f32(st, c->gmeta, 0.f, c->n); launch_fill_f32(st, c->vdir, 0.f, c->n);
  launch_fill_f32(st, c->meta_m, 0.f, c->nl); launch_fill_f32(st, c->meta_v, 0.f, c->nl);
  launch_fill_f32(st, c->hyper, 0.f, c->nl); launch_fill_f32(st, c->glam_p32, 0.f, c->nl); launch_fill_f32(st, c->glam_m32, 0.f, c->nl);
  launch_fill_f32(st, c->scalars, 0.f, 4);
  launch_fill_f32(st, c->step, 0.f, 8);
  launch_fill_i64x4(st, c->counters, 0, 0, 0, 0, 15);
  if (c->bf16) { launch_to_bf16(st, c->theta16, c->theta, c->n_gemm); launch_residual_lo(st, c->theta, c->lo_0, c->n_gemm); }
  sama_status s = check_hip(nullptr, "sama_init");
  if (s != SAMA_OK) return s;
  *out = c.release();
  return SAMA_OK;
}

// How a pass sees theta: sign = 0 with lo = null contracts with the bf16 working copy alone, with lo = lo_0 (the
// residual half) at theta itself; sign = +-1 with the matching half of theta +- eps v.
static PassWeights pass_weights(sama_ctx* c, float sign, const bf16_t* lo) {
  PassWeights w{};
  w.theta = c->theta; w.vdir = c->vdir; w.eps_ptr = c->scalars; w.sign = sign;
  w.hi = c->theta16;
  w.lo = lo;
  return w;
}
// the base step's (and the forward-only evaluation's) view
static PassWeights base_weights(sama_ctx* c) { return pass_weights(c, 0.f, (c->bf16 && !c->cfg.fast_base_pass) ? c->lo_0 : nullptr); }

sama_status sama_base_step(sama_ctx* c, const sama_batch* train, float* loss_out) {
  if (!c) return SAMA_EINVAL;
  sama_status s = check_batch(c, train, c->cfg.max_batch, "train");
  if (s != SAMA_OK) return s;
  hipStream_t st = c->stream;
  (void)hipGetLastError();
  launch_step_scalars(st, c->counters, 1, c->cfg.base_lr, c->cfg.beta1, c->cfg.beta2, c->step);
  const PassWeights w = base_weights(c);
  c->model->forward(st, w, *train, true, c->logits);
  SampleStageArgs sa{};
  sa.logits = c->logits; sa.ld = c->model->n_classes(); sa.C = sa.ld; sa.B = train->n; sa.H = c->cfg.wnet_hidden;
  sa.mode = STAGE_BASE; sa.Hc = c->cfg.corr_hidden; sa.kappa = c->cfg.corr_kappa; sa.y = train->y; sa.mask = train->sample_mask; sa.lambda = c->lambda;
  sa.losses = c->losses; sa.dlogits = c->dlogits; sa.loss_scalar = c->scalars + 2; sa.loss_user = loss_out;
  launch_sample_stage(st, sa);
  UpdateSink sink(c, c->t + 1);
  c->model->set_grad_sink(&sink);
  c->model->backward(st, w, *train, c->dlogits, c->g);
  c->model->set_grad_sink(nullptr);
  base_update_rest(c, sink);
  return check_hip(c, "sama_base_step");
}

sama_status sama_eval(sama_ctx* c, const sama_batch* batch, float* logits_out, float* losses_out, float* weights_out) {
  if (!c) return SAMA_EINVAL;
  const int maxb = c->cfg.max_batch > c->cfg.max_meta_batch ? c->cfg.max_batch : c->cfg.max_meta_batch;
  sama_status s = check_batch(c, batch, maxb, "eval");
  if (s != SAMA_OK) return s;
  hipStream_t st = c->stream;
  (void)hipGetLastError();
  const PassWeights w = base_weights(c);
  float* logits = logits_out != nullptr ? logits_out : c->logits;
  c->model->forward(st, w, *batch, false, logits);
  if (losses_out != nullptr || weights_out != nullptr) {
    SampleStageArgs sa{};
    sa.logits = logits; sa.ld = c->model->n_classes(); sa.C = sa.ld; sa.B = batch->n; sa.H = c->cfg.wnet_hidden;
    sa.mode = STAGE_EVAL; sa.Hc = c->cfg.corr_hidden; sa.kappa = c->cfg.corr_kappa; sa.y = batch->y; sa.mask = nullptr;
    sa.lambda = c->lambda; sa.losses = losses_out; sa.weights = weights_out;
    launch_sample_stage(st, sa);
  }
  return check_hip(c, "sama_eval");
}

// First half of a meta gradient: g_meta = dL_meta/dtheta on the clean batch (Eq. 1), v = (du/dg) . g_meta,
// eps = alpha / ||v|| (Eq. 4-5, App. C), and the low halves of theta +- eps v.  Returns whether the GEMM block of
// theta was nudged already (sama_meta_step on bf16 models: one pass over theta and v instead of two).
static bool meta_direction(sama_ctx* c, const sama_batch* meta, bool update) {
  hipStream_t st = c->stream;
  const sama_config& f = c->cfg;
  const int C = c->model->n_classes();
  // hi + lo of the master weights: the gradient is taken at theta, not bf16(theta)
  const PassWeights w0 = pass_weights(c, 0.f, (c->bf16 && !f.fast_meta_pass) ? c->lo_0 : nullptr);
  c->model->forward(st, w0, *meta, true, c->logits);
  SampleStageArgs sa{};
  sa.logits = c->logits; sa.ld = C; sa.C = C; sa.B = meta->n; sa.H = f.wnet_hidden; sa.mode = STAGE_META;
  sa.y = meta->y; sa.mask = meta->sample_mask; sa.lambda = c->lambda; sa.losses = c->losses; sa.dlogits = c->dlogits;
  sa.loss_scalar = c->scalars + 3;
  launch_sample_stage(st, sa);
  AdaptArgs ad{};
  if (f.adapt_mode == SAMA_ADAPT_NONE) { ad.mode = 1; ad.scalar = 1.f; }
  else if (f.base_opt == SAMA_OPT_SGD) { ad.mode = 1; ad.scalar = c->lr_step; }
  else {
    const double c1 = 1.0 / (1.0 - pow((double)f.beta1, (double)c->t));
    const double c2 = 1.0 / sqrt(1.0 - pow((double)f.beta2, (double)c->t));
    ad.mode = 0; ad.one_m_beta1 = (float)(1.0 - (double)f.beta1); ad.one_m_beta2 = (float)(1.0 - (double)f.beta2);
    ad.lr_c1_c2 = (float)((double)c->lr_step * c1 * c2); ad.c2 = (float)c2; ad.eps = f.adam_eps;
    ad.dev = c->step;
  }
  // v = D . g_meta layer by layer while the backward pass still runs, the rest after it, then the norm
  AdaptSink sink(c, ad);
  c->model->set_grad_sink(&sink);
  c->model->backward(st, w0, *meta, c->dlogits, c->gmeta);
  c->model->set_grad_sink(nullptr);
  std::sort(sink.done.begin(), sink.done.end());
  {
    std::vector<std::pair<int64_t, int64_t>> gaps;
    int64_t pos = 0;
    for (auto& r : sink.done) { if (r.first > pos) gaps.push_back({pos, r.first - pos}); pos = r.first + r.second; }
    if (pos < c->n) gaps.push_back({pos, c->n - pos});
    const int per_gap = gaps.empty() ? 0 : (EW_MAX_BLOCKS - sink.used) / (int)gaps.size();
    for (auto& r : gaps) sink.slice(st, r.first, r.second, per_gap);
  }
  launch_eps_from_partials(st, c->partial, sink.used, f.alpha, c->scalars, c->counters + 2);
  // A step that is applied nudges the GEMM block of theta in the same pass that writes the low halves; the non-GEMM
  // tail is nudged after the two passes, which read it as theta +- eps v.
  const bool fused_nudge = update && c->bf16 && c->n_gemm % 4 == 0;
  // (the low half of theta_old - eps v against the new working copy IS the residual half of the new theta: lo_0)
  if (fused_nudge) launch_perturb_nudge(st, c->theta, c->vdir, c->scalars, c->theta16, c->lo_p, c->lo_0, c->n_gemm);
  else if (c->bf16) launch_perturb_lo(st, c->theta, c->vdir, c->scalars, c->lo_p, c->lo_m, c->n_gemm);
  return fused_nudge;
}

// Second half: h from the two lambda-gradients (Eq. 5), Adam on lambda and the nudge of theta when `update`.
static void meta_finish(sama_ctx* c, float* hyper_out, float* eps_out, bool update, bool fused_nudge) {
  hipStream_t st = c->stream;
  const sama_config& f = c->cfg;
  MetaUpdateArgs mu{};
  mu.glam_p = c->glam_p; mu.glam_m = c->glam_m; mu.scalars = c->scalars; mu.counters = c->counters;
  mu.hypergrad = c->hyper; mu.hypergrad_user = hyper_out; mu.eps_user = eps_out;
  mu.glam_p_f32 = c->glam_p32; mu.glam_m_f32 = c->glam_m32;
  mu.lambda = c->lambda; mu.meta_m = c->meta_m; mu.meta_v = c->meta_v; mu.nl = c->nl; mu.do_update = update ? 1 : 0;
  mu.lr = f.meta_lr; mu.beta1 = f.meta_beta1; mu.beta2 = f.meta_beta2; mu.eps = f.meta_eps;
  launch_meta_update(st, mu);
  // a hypergradient that is not finite skips the step (status word): the tail is then left alone and the GEMM block's
  // early nudge is taken back
  if (update && fused_nudge) {
    launch_unnudge(st, c->theta, c->vdir, c->scalars, c->counters + 2, c->theta16, c->lo_0, c->n_gemm);
    launch_nudge(st, c->theta + c->n_gemm, c->vdir + c->n_gemm, c->scalars, c->counters + 2, nullptr, nullptr, c->n - c->n_gemm, 0);
  } else if (update) {
    launch_nudge(st, c->theta, c->vdir, c->scalars, c->counters + 2, c->theta16, c->lo_0, c->n, c->n_gemm);
  }
}

static sama_status meta_common(sama_ctx* c, const sama_batch* train, const sama_batch* meta, float* hyper_out,
                               float* eps_out, bool update) {
  if (!c) return SAMA_EINVAL;
  sama_status s = check_batch(c, train, c->cfg.max_batch, "train");
  if (s != SAMA_OK) return s;
  s = check_batch(c, meta, c->cfg.max_meta_batch, "meta");
  if (s != SAMA_OK) return s;
  if (c->t < 1) return fail(c, SAMA_ESTATE, "meta gradient requested before any sama_base_step");
  hipStream_t st = c->stream;
  (void)hipGetLastError();
  const sama_config& f = c->cfg;
  const int C = c->model->n_classes();
  const bool fused_nudge = meta_direction(c, meta, update);
  // passes 2 and 3: dL_base/dlambda at theta +- eps v; forward only, then the weight net's backward
  c->model->forward_pair(st, pass_weights(c, 1.f, c->lo_p), pass_weights(c, -1.f, fused_nudge ? c->lo_0 : c->lo_m), *train, c->logits);
  for (int pass = 0; pass < 2; ++pass) {
    SampleStageArgs sg{};
    sg.logits = c->logits + (size_t)pass * train->n * C; sg.ld = C; sg.C = C; sg.B = train->n; sg.H = f.wnet_hidden; sg.mode = STAGE_GLAM;
    sg.Hc = f.corr_hidden; sg.kappa = f.corr_kappa; sg.corr_scratch = c->corr_scratch;
    sg.y = train->y; sg.mask = train->sample_mask; sg.lambda = c->lambda; sg.losses = c->losses;
    sg.glam = pass == 0 ? c->glam_p : c->glam_m;
    launch_sample_stage(st, sg);
  }
  meta_finish(c, hyper_out, eps_out, update, fused_nudge);
  return check_hip(c, update ? "sama_meta_step" : "sama_meta_grad");
}

// ------------------------------------------------------------------ auxiliary-task reweighting (Sec. 4.3)
static sama_status check_aux(sama_ctx* c, const sama_aux_batch* pt) {
  if (!c->cfg.aux_mlm || !c->model->has_mlm()) return fail(c, SAMA_EINVAL, "the context was not created with aux_mlm = 1");
  if (!pt || !pt->ids || !pt->mask_row || !pt->mask_tgt) return fail(c, SAMA_EINVAL, "aux: null batch / ids / mask_row / mask_tgt");
  if (pt->n_seq < 1 || pt->n_seq > c->cfg.max_aux_batch) return fail(c, SAMA_EINVAL, "aux: n_seq outside 1..max_aux_batch");
  if (pt->n_mask < 1 || pt->n_mask > c->cfg.max_aux_masked) return fail(c, SAMA_EINVAL, "aux: n_mask outside 1..max_aux_masked");
  if ((int64_t)pt->n_mask > (int64_t)pt->n_seq * c->cfg.dims[4]) return fail(c, SAMA_EINVAL, "aux: more masked positions than tokens");
  return SAMA_OK;
}

// the sequence-mode stage on the masked-token losses of one pass
static void aux_stage(sama_ctx* c, const sama_aux_batch* pt, int mode, const float* loss_pos, float* losses, double* glam,
                      float* loss_user) {
  SampleStageArgs sa{};
  sa.B = pt->n_seq; sa.H = c->cfg.wnet_hidden; sa.mode = mode; sa.lambda = c->lambda; sa.losses = losses;
  sa.pos_loss = loss_pos; sa.pos_row = pt->mask_row; sa.n_pos = pt->n_mask; sa.S = c->cfg.dims[4];
  sa.pos_coef = c->coef_pos; sa.loss_scalar = c->scalars + 2; sa.loss_user = loss_user; sa.glam = glam;
  launch_sample_stage(c->stream, sa);
}

sama_status sama_aux_base_step(sama_ctx* c, const sama_batch* ft, const sama_aux_batch* pt, float* loss_out) {
  if (!c) return SAMA_EINVAL;
  sama_status s = check_batch(c, ft, c->cfg.max_batch, "ft");
  if (s != SAMA_OK) return s;
  s = check_aux(c, pt);
  if (s != SAMA_OK) return s;
  hipStream_t st = c->stream;
  (void)hipGetLastError();
  const int S = c->cfg.dims[4], C = c->model->n_classes(), n_ft = ft->n, n_pt = pt->n_seq;
  launch_step_scalars(st, c->counters, 1, c->cfg.base_lr, c->cfg.beta1, c->cfg.beta2, c->step);
  const bool padded = ft->seq_len != nullptr || pt->seq_len != nullptr;
  launch_aux_cat(st, (const int32_t*)ft->x, ft->y, ft->sample_mask, n_ft, pt->ids, n_pt, S, c->ids_cat, c->y_cat, c->mask_cat,
                 ft->seq_len, pt->seq_len, padded ? c->len_cat : nullptr);
  const sama_batch cat{c->ids_cat, c->y_cat, c->mask_cat, n_ft + n_pt, padded ? c->len_cat : nullptr};
  const PassWeights w = base_weights(c);
  c->model->forward(st, w, cat, true, c->logits);
  // finetuning term: mean cross-entropy over the ft rows (the auxiliary rows are masked out of the classifier loss)
  SampleStageArgs sa{};
  sa.logits = c->logits; sa.ld = C; sa.C = C; sa.B = cat.n; sa.H = c->cfg.wnet_hidden; sa.mode = STAGE_META;
  sa.y = cat.y; sa.mask = cat.sample_mask; sa.lambda = c->lambda; sa.losses = c->losses; sa.dlogits = c->dlogits;
  sa.loss_scalar = c->scalars + 2; sa.loss_user = loss_out;
  launch_sample_stage(st, sa);
  // weighted pretraining term
  const MlmBatch mb{pt->mask_row, pt->mask_tgt, pt->n_mask, n_ft * S, n_pt * S};
  c->model->mlm_forward(st, &w, 1, cat.n * S, true, mb, c->loss_pos);
  aux_stage(c, pt, STAGE_BASE, c->loss_pos, c->losses + n_ft, nullptr, loss_out);
  UpdateSink sink(c, c->t + 1);
  c->model->set_grad_sink(&sink);
  c->model->backward_mlm(st, w, cat, c->dlogits, c->g, mb, c->coef_pos);
  c->model->set_grad_sink(nullptr);
  base_update_rest(c, sink);
  return check_hip(c, "sama_aux_base_step");
}

sama_status sama_aux_eval(sama_ctx* c, const sama_aux_batch* pt, float* losses_out, float* weights_out) {
  if (!c) return SAMA_EINVAL;
  sama_status s = check_aux(c, pt);
  if (s != SAMA_OK) return s;
  hipStream_t st = c->stream;
  (void)hipGetLastError();
  const int S = c->cfg.dims[4];
  const sama_batch ptb{pt->ids, nullptr, nullptr, pt->n_seq, pt->seq_len};
  const PassWeights w = base_weights(c);
  c->model->forward(st, w, ptb, true, c->logits);        // the head reads the kept last hidden state
  const MlmBatch mb{pt->mask_row, pt->mask_tgt, pt->n_mask, 0, pt->n_seq * S};
  c->model->mlm_forward(st, &w, 1, pt->n_seq * S, true, mb, c->loss_pos);
  SampleStageArgs sa{};
  sa.B = pt->n_seq; sa.H = c->cfg.wnet_hidden; sa.mode = STAGE_EVAL; sa.lambda = c->lambda;
  sa.losses = losses_out; sa.weights = weights_out;
  sa.pos_loss = c->loss_pos; sa.pos_row = pt->mask_row; sa.n_pos = pt->n_mask; sa.S = S;
  launch_sample_stage(st, sa);
  return check_hip(c, "sama_aux_eval");
}

static sama_status aux_meta_common(sama_ctx* c, const sama_aux_batch* pt, const sama_batch* meta, float* hyper_out,
                                   float* eps_out, bool update) {
  if (!c) return SAMA_EINVAL;
  sama_status s = check_aux(c, pt);
  if (s != SAMA_OK) return s;
  s = check_batch(c, meta, c->cfg.max_meta_batch, "meta");
  if (s != SAMA_OK) return s;
  if (c->t < 1) return fail(c, SAMA_ESTATE, "meta gradient requested before any base step");
  hipStream_t st = c->stream;
  (void)hipGetLastError();
  const int S = c->cfg.dims[4];
  const bool fused_nudge = meta_direction(c, meta, update);
  // passes 2 and 3 on the auxiliary sequences alone: the finetuning term of L_base does not depend on lambda
  const sama_batch ptb{pt->ids, nullptr, nullptr, pt->n_seq, pt->seq_len};
  const PassWeights w[2] = {pass_weights(c, 1.f, c->lo_p), pass_weights(c, -1.f, fused_nudge ? c->lo_0 : c->lo_m)};
  c->model->forward_pair(st, w[0], w[1], ptb, c->logits);
  const MlmBatch mb{pt->mask_row, pt->mask_tgt, pt->n_mask, 0, pt->n_seq * S};
  c->model->mlm_forward(st, w, 2, pt->n_seq * S, false, mb, c->loss_pos);
  const int P = c->model->mlm_stride();
  for (int pass = 0; pass < 2; ++pass)
    aux_stage(c, pt, STAGE_GLAM, c->loss_pos + (size_t)pass * P, c->losses, pass == 0 ? c->glam_p : c->glam_m, nullptr);
  meta_finish(c, hyper_out, eps_out, update, fused_nudge);
  return check_hip(c, update ? "sama_aux_meta_step" : "sama_aux_meta_grad");
}

sama_status sama_meta_grad(sama_ctx* c, const sama_batch* train, const sama_batch* meta, float* hypergrad_out,
                           float* eps_out) {
  return meta_common(c, train, meta, hypergrad_out, eps_out, false);
}
sama_status sama_meta_step(sama_ctx* c, const sama_batch* train, const sama_batch* meta) {
  return meta_common(c, train, meta, nullptr, nullptr, true);
}
sama_status sama_aux_meta_grad(sama_ctx* c, const sama_aux_batch* pt, const sama_batch* meta, float* hypergrad_out,
                               float* eps_out) {
  return aux_meta_common(c, pt, meta, hypergrad_out, eps_out, false);
}
sama_status sama_aux_meta_step(sama_ctx* c, const sama_aux_batch* pt, const sama_batch* meta) {
  return aux_meta_common(c, pt, meta, nullptr, nullptr, true);
}

static bool state_ptr(sama_ctx* c, int32_t which, void** p, size_t* bytes, bool* writable) {
  const size_t nb = (size_t)c->n * 4, lb = (size_t)c->nl * 4;
  *writable = true;
  switch (which) {
    case SAMA_STATE_THETA: *p = c->theta; *bytes = nb; return true;
    case SAMA_STATE_M: *p = c->m; *bytes = nb; return true;
    case SAMA_STATE_V: *p = c->v; *bytes = nb; return true;
    case SAMA_STATE_G: *p = c->g; *bytes = nb; return true;
    case SAMA_STATE_GMETA: *p = c->gmeta; *bytes = nb; return true;
    case SAMA_STATE_VDIR: *p = c->vdir; *bytes = nb; return true;
    case SAMA_STATE_LAMBDA: *p = c->lambda; *bytes = lb; return true;
    case SAMA_STATE_META_M: *p = c->meta_m; *bytes = lb; return true;
    case SAMA_STATE_META_V: *p = c->meta_v; *bytes = lb; return true;
    case SAMA_STATE_COUNTERS: *p = c->counters; *bytes = 32; return true;
    case SAMA_STATE_HYPERGRAD: *p = c->hyper; *bytes = lb; *writable = false; return true;
    case SAMA_STATE_GLAM_PLUS: *p = c->glam_p32; *bytes = lb; *writable = false; return true;
    case SAMA_STATE_GLAM_MINUS: *p = c->glam_m32; *bytes = lb; *writable = false; return true;
    case SAMA_STATE_SCALARS: *p = c->scalars; *bytes = 16; *writable = false; return true;
    case SAMA_STATE_LOSSES: {
      const int mb = max_rows(c->cfg);
      *p = c->losses; *bytes = (size_t)mb * 4; *writable = false; return true;
    }
  }
  return false;
}

sama_status sama_get_state(sama_ctx* c, int32_t which, void* dst) {
  if (!c) return SAMA_EINVAL;
  if (!dst) return fail(c, SAMA_EINVAL, "null dst");
  void* p; size_t bytes; bool wr;
  if (!state_ptr(c, which, &p, &bytes, &wr)) return fail(c, SAMA_EINVAL, "unknown state selector");
  if (hipMemcpyAsync(dst, p, bytes, hipMemcpyDeviceToDevice, c->stream) != hipSuccess)
    return fail(c, SAMA_EHIP, "sama_get_state: copy failed");
  return SAMA_OK;
}

sama_status sama_set_state(sama_ctx* c, int32_t which, const void* src) {
  if (!c) return SAMA_EINVAL;
  if (!src) return fail(c, SAMA_EINVAL, "null src");
  void* p; size_t bytes; bool wr;
  if (!state_ptr(c, which, &p, &bytes, &wr)) return fail(c, SAMA_EINVAL, "unknown state selector");
  if (!wr) return fail(c, SAMA_EINVAL, "state selector is read-only");
  if (hipMemcpyAsync(p, src, bytes, hipMemcpyDeviceToDevice, c->stream) != hipSuccess)
    return fail(c, SAMA_EHIP, "sama_set_state: copy failed");
  if (which == SAMA_STATE_THETA && c->bf16) {
    launch_to_bf16(c->stream, c->theta16, c->theta, c->n_gemm);
    launch_residual_lo(c->stream, c->theta, c->lo_0, c->n_gemm);
  }
  if (which == SAMA_STATE_COUNTERS) {
    int64_t host[4];
    if (hipMemcpyAsync(host, c->counters, 32, hipMemcpyDeviceToHost, c->stream) != hipSuccess ||
        hipStreamSynchronize(c->stream) != hipSuccess)
      return fail(c, SAMA_EHIP, "sama_set_state: counter read-back failed");
    if (host[0] < 0 || host[1] < 0) return fail(c, SAMA_EINVAL, "negative counters");
    c->t = host[0];
    c->lr_step = c->cfg.base_lr;   // a state put in from outside is taken to have been reached at the rate in force
    launch_step_scalars(c->stream, c->counters, 0, c->cfg.base_lr, c->cfg.beta1, c->cfg.beta2, c->step);
  }
  return check_hip(c, "sama_set_state");
}

sama_status sama_set_lr(sama_ctx* c, float base_lr, float meta_lr) {
  if (!c) return SAMA_EINVAL;
  if (!(base_lr > 0.f) || !(meta_lr > 0.f) || !isfinite(base_lr) || !isfinite(meta_lr))
    return fail(c, SAMA_EINVAL, "base_lr and meta_lr must be finite and > 0");
  c->cfg.base_lr = base_lr; c->cfg.meta_lr = meta_lr;
  return SAMA_OK;
}

int32_t sama_profile_family_count(void) { return F_COUNT; }
sama_status sama_profile_enable(sama_ctx* c, int32_t on) {
  if (!c) return SAMA_EINVAL;
  prof_enable(on != 0);
  return SAMA_OK;
}
sama_status sama_profile_read(sama_ctx* c, int32_t family, const char** name, int64_t* launches, double* total_ms,
                              double* units) {
  if (!c) return SAMA_EINVAL;
  if (!prof_read(family, name, launches, total_ms, units)) return fail(c, SAMA_EINVAL, "unknown kernel family");
  return SAMA_OK;
}

const char* sama_last_error(const sama_ctx* c) { return c ? c->err.c_str() : g_init_err.c_str(); }

void sama_destroy(sama_ctx* c) { delete c; }

}  // extern "C"
