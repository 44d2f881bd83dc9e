// Host-side launchers of every gfx950 kernel in libsama.  Internal; the C ABI is include/sama.h.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <tuple>
#include <utility>
#include "common.h"

namespace sama {
namespace detail {
template <typename Tuple, size_t... I>
inline void arg_pointers(Tuple& t, void** out, std::index_sequence<I...>) {
  ((out[I] = const_cast<void*>(static_cast<const void*>(&std::get<I>(t)))), ...);
}
}  // namespace detail

// ------------------------------------------------------------------ optional per-launch timing (profile.hip)
enum Family {
  F_GEMM_NT = 0, F_GEMM_NN, F_GEMM_TN, F_GEMM_NT_HILO, F_GEMM_NN_HILO, F_GEMM_F32, F_ATTN_FWD, F_ATTN_BWD, F_LN_FWD, F_LN_BWD, F_ADAM, F_ADAPT_NORM,
  F_PERTURB, F_RESIDUAL, F_NUDGE, F_SAMPLE_STAGE, F_MLM_SOFTMAX, F_OTHER, F_COUNT
};
// While profiling is enabled every launch made through launch_kernel carries a start and a stop event that take the
// kernel's own begin and end timestamps (hipExtLaunchKernel), so a recorded duration is the kernel's execution time as
// a kernel trace shows it, without the dispatch gap in front of it.  A scope names the family and the work of what its
// launcher enqueues; `units` = algorithmic flops (GEMM, attention) or algorithmic bytes (everything else), credited to
// the scope's first launch.
struct ProfScope {
  ProfScope(hipStream_t st, int family, double units);
  bool on() const { return on_; }
  void next_events(hipEvent_t* start, hipEvent_t* stop);   // registers one more launch of this scope (profiling on only)
  hipStream_t st_;
  int family_;
  double units_;
  bool on_;
};
// kernel<<<grid, block, lds, st>>>(args...), timed when the scope is live.  The actual arguments are converted to the
// kernel's formal parameter types first, as the launch syntax would.
template <typename... P, typename... A>
inline void launch_kernel(ProfScope& ps, void (*kernel)(P...), dim3 grid, dim3 block, unsigned lds, hipStream_t st, A&&... a) {
  static_assert(sizeof...(P) == sizeof...(A), "argument count");
  std::tuple<P...> params(std::forward<A>(a)...);
  void* ptrs[sizeof...(P) > 0 ? sizeof...(P) : 1];
  detail::arg_pointers(params, ptrs, std::index_sequence_for<P...>{});
  if (ps.on()) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ps.next_events(&e0, &e1);
    (void)hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, st, e0, e1, 0);
  } else {
    (void)hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds, st);
  }
}
void prof_enable(bool on);
bool prof_read(int family, const char** name, int64_t* launches, double* total_ms, double* units);

constexpr int EW_MAX_BLOCKS = 65536;  // grid cap of the elementwise kernels (also the size of the norm partials)
// A launcher that is handed a shape its kernel cannot run records the reason here and launches nothing; the C entry
// points report it as an error (take_launch_error returns and clears it, null = none).
void note_launch_error(const char* what);
const char* take_launch_error();

constexpr int MAX_BATCH = 2048;
constexpr int MAX_TOKENS = 8192;   // encoder: token rows of one batch (the token-gradient kernel lists them in LDS)
constexpr int MAX_WNET_HIDDEN = 256;
constexpr int MAX_CORR_HIDDEN = 128;   // label corrector: hidden width and number of classes it supports
constexpr int MAX_CORR_CLASSES = 16;

// ------------------------------------------------------------------ elementwise chain (elementwise.hip)
struct AdamArgs {
  float beta1, one_m_beta1, beta2, one_m_beta2;
  float lr_c1;  // lr / (1 - beta1^t)
  float c2;     // 1 / sqrt(1 - beta2^t)
  float eps, weight_decay;
  const float* dev;  // non-null: lr_c1 = dev[0], c2 = dev[1] read on the device (launch_step_scalars), the two fields above unused
  bf16_t* lo;        // non-null: also lo[k] = bf16(theta'[k] - float(bf16(theta'[k]))) for the first n16 elements (what
                     // launch_residual_lo would compute afterwards)
};
struct AdaptArgs {
  int mode;  // 0: Adam closed form, 1: scalar
  float scalar;
  float one_m_beta1, one_m_beta2;
  float lr_c1_c2;  // lr c1 c2
  float c2, eps;
  const float* dev;  // non-null: lr_c1_c2 = dev[2], c2 = dev[3] read on the device
};
// The step-dependent scalars of Adam and of its adaptation, kept on the device so that a captured sequence of launches
// stays valid from replay to replay: t = (counters[0] += advance); step[0..3] = {lr / (1 - beta1^t),
// 1 / sqrt(1 - beta2^t), lr c1 c2, c2} in double arithmetic (left alone while t < 1).
void launch_step_scalars(hipStream_t, int64_t* counters, int advance, float lr, float beta1, float beta2, float* step);
// With a non-zero weight decay the L2 term is added to g in place (g then is the gradient the solver was given).
void launch_adam(hipStream_t, float* g, float* m, float* v, float* theta, bf16_t* theta16, int64_t n, int64_t n16,
                 const AdamArgs&);
// SGD with heavy-ball momentum mu (velocity in buf, untouched when mu = 0); lo as in AdamArgs (may be null)
void launch_sgd(hipStream_t, float* g, float* buf, float* theta, bf16_t* theta16, bf16_t* lo, int64_t n, int64_t n16, float lr,
                float wd, float mu);
// v = D . gmeta, then eps = alpha/||v|| -> scalars[0], ||v|| -> scalars[1], status[0] = (norm unusable)
void launch_adapt_norm(hipStream_t, const float* g, const float* m, const float* v, const float* gmeta, float* vdir,
                       double* partial /*[EW_MAX_BLOCKS]*/, int64_t n, const AdaptArgs&, float alpha, float* scalars,
                       int64_t* status);
// The same in pieces: v = D . gmeta over one range, its per-block sums of squares into partial[0 .. returned count)
// (at most max_blocks), and, once every range is done, eps and the status word from all the partials in index order.
int launch_adapt_slice(hipStream_t, const float* g, const float* m, const float* v, const float* gmeta, float* vdir,
                       double* partial, int64_t n, const AdaptArgs&, int max_blocks);
void launch_eps_from_partials(hipStream_t, const double* partial, int count, float alpha, float* scalars, int64_t* status);
void launch_perturb_lo(hipStream_t, const float* theta, const float* vdir, const float* eps_ptr, bf16_t* lo_p,
                       bf16_t* lo_m, int64_t n16);
// perturb_lo and the nudge of the first n16 elements (n16 % 4 == 0) in one pass: theta, theta16 <- theta - eps v,
// lo_p / lo_m = low halves of theta_old +- eps v against the NEW theta16
void launch_perturb_nudge(hipStream_t, float* theta, const float* vdir, const float* eps_ptr, bf16_t* theta16, bf16_t* lo_p,
                          bf16_t* lo_m, int64_t n16);
// lo[k] = bf16(theta[k] - float(bf16(theta[k]))): the part of the master weights the bf16 working copy cannot hold
void launch_residual_lo(hipStream_t, const float* theta, bf16_t* lo, int64_t n16);
// theta <- theta - eps v; theta16 / lo (either may be null) receive the rounded copy and its residual half over the first
// n16 elements; nothing happens when eps = 0 or *status != 0 (status may be null)
void launch_nudge(hipStream_t, float* theta, const float* vdir, const float* eps_ptr, const int64_t* status, bf16_t* theta16,
                  bf16_t* lo, int64_t n, int64_t n16);
// undoes launch_perturb_nudge's nudge of the first n16 elements when *status != 0 although eps > 0 (early exit otherwise)
void launch_unnudge(hipStream_t, float* theta, const float* vdir, const float* eps_ptr, const int64_t* status, bf16_t* theta16,
                    bf16_t* lo, int64_t n16);
void launch_fill_f32(hipStream_t, float* p, float val, int64_t n);
void launch_copy_f32(hipStream_t, float* dst, const float* src, int64_t n);
void launch_to_bf16(hipStream_t, bf16_t* dst, const float* src, int64_t n);
void launch_fill_i64x4(hipStream_t, int64_t* p, int64_t a, int64_t b, int64_t c, int64_t d, int mask);

// ------------------------------------------------------------------ per-sample stage (sample_stage.hip)
enum { STAGE_BASE = 0, STAGE_META = 1, STAGE_GLAM = 2, STAGE_EVAL = 3 };   // EVAL: BASE's losses and weights only
struct SampleStageArgs {
  const float* logits;  // [B x C], row stride ld
  int ld, C, B, H, mode;
  const int32_t* y;
  const uint8_t* mask;  // may be null
  const float* lambda;  // [3H+1] weighting net, then the corrector [Hc*2C + Hc + C*Hc + C] when Hc > 0
  int Hc; float kappa;  // label corrector (BASE and GLAM): Hc = 0 turns it off
  double* corr_scratch; // [B x 2C] device scratch of the corrector's backward (GLAM with Hc > 0)
  float* losses;        // [B] out (may be null in EVAL)
  float* weights;       // [B] out, w(l_i; lambda), or null
  float* dlogits;       // [B x C] out, row stride C (BASE, META)
  float* loss_scalar;   // out: sum_i coef_i l_i
  float* loss_user;     // optional second destination
  double* glam;         // [n_lambda] out (GLAM), same layout as lambda
  // Sequence mode (pos_loss != null; BASE or GLAM): sample i is sequence i of B, its loss the mean of pos_loss[j] over
  // the positions with pos_row[j] / S == i (0 without any); logits, y, dlogits are unused.  BASE writes
  // pos_coef[j] = mask_i w_i / (B_eff count_i) and ADDS sum_i coef_i l_i to *loss_scalar (and *loss_user).
  const float* pos_loss; const int32_t* pos_row; int n_pos, S;
  float* pos_coef;
};
void launch_sample_stage(hipStream_t, const SampleStageArgs&);
struct MetaUpdateArgs {
  const double* glam_p; const double* glam_m;
  const float* scalars;   // [0] = eps
  int64_t* counters;      // [1] = meta step count, [2] = status
  float* hypergrad;       // [nl] out
  float* hypergrad_user;  // optional
  float* eps_user;        // optional
  float* glam_p_f32; float* glam_m_f32;  // fp32 copies for inspection
  float* lambda; float* meta_m; float* meta_v;
  int nl, do_update;
  float lr, beta1, beta2, eps;
};
void launch_meta_update(hipStream_t, const MetaUpdateArgs&);

// ------------------------------------------------------------------ fp32 GEMM (gemm_f32.hip)
// C[M x N] = sum_k A(i,k) B(k,j), A(i,k) = A[i*sa_i + k*sa_k], B(k,j) = Bh[k*sb_k + j*sb_j] (+ bscale * Bv[same]),
// bscale = bsign * (*beps) when Bv != null.  Epilogue: + bias(j) (a ParamView index bias_off + j), then
// relu, or multiplication by (gate[i*ldc + j] > 0).
struct GemmF32Args {
  const float* A; int64_t sa_i, sa_k;
  const float* B; const float* Bv; const float* beps; float bsign; int64_t sb_k, sb_j;
  float* C; int64_t ldc;
  int M, N, K;
  const float* bias; const float* bias_v;  // null = no bias; perturbed with the same bscale
  const float* gate;                       // null = none
  int relu;
};
void launch_gemm_f32(hipStream_t, const GemmF32Args&);
// out[j] = sum_i X[i*ld + j], fixed order.
void launch_colsum_f32(hipStream_t, const float* X, int64_t ld, int M, int N, float* out);

// ------------------------------------------------------------------ bf16 MFMA GEMM (gemm_bf16.hip)
enum { GEMM_ACT_NONE = 0, GEMM_ACT_GELU_FWD = 1, GEMM_ACT_GELU_BWD = 2 };
// C[M x N] = A . (B + B2).  a_trans = 0: A stored [M][K]; 1: stored [K][M].  b_trans = 1: B stored [N][K]
// (a weight matrix [out x in] used forward); 0: stored [K][N].  B2 (same storage as B) may be null.
// Epilogue, in this order: + bias[j] (+ bsign * *beps * bias_v[j]); + res16 / res32 [i*ldc + j];
// GELU_FWD: C16_pre = bf16(c) (stored when C16_pre is given), c = gelu(that);  GELU_BWD: c *= gelu'(aux16[i*ldc + j]);  stores to C32 and/or C16.
struct GemmBf16Args {
  const bf16_t* A; int64_t lda; int a_trans;
  const bf16_t* B; const bf16_t* B2; int64_t ldb; int b_trans;
  int M, N, K;
  int64_t ldc;
  const float* bias; const float* bias_v; const float* beps; float bsign;
  const bf16_t* res16; const float* res32;
  int act; const bf16_t* aux16; bf16_t* C16_pre;
  float* C32; bf16_t* C16;
};
const char* check_gemm_bf16(const GemmBf16Args&);  // null if the shapes / alignments are supported
void launch_gemm_bf16(hipStream_t, const GemmBf16Args&);
// Up to GEMM_MAX_BATCH independent problems in one launch; they must agree in a_trans, b_trans and in whether B2 is
// given (shapes, K and epilogues may differ).
constexpr int GEMM_MAX_BATCH = 4;
const char* check_gemm_bf16_batch(const GemmBf16Args* p, int count);
void launch_gemm_bf16_batch(hipStream_t, const GemmBf16Args* p, int count);
void encoder_side_sink(bool on);         // tuning hook: per-layer gradient consumers on that stream (default on)
void encoder_side_stream(bool on);      // tuning hook: weight-gradient launches on a second stream (default on)
void gemm_bf16_force_shape(int shape);  // tuning hook: 0 = heuristic, else 100 * tile-order group + tile configuration id

// ------------------------------------------------------------------ encoder ops (encoder_ops.hip)
constexpr int LN_MAX_D = 2048;       // LayerNorm kernels keep a row in registers (4 or 8 16-byte pieces per lane)
constexpr int LN_BWD_ROWS = 8;       // rows per block in the LayerNorm backward (size of its partial sums)
constexpr int COLSUM_ROWS = 16;      // rows per block in the column-sum kernel
struct LnFwdArgs {
  const float* x;          // [M x d] input, or null: embedding mode (x = tok_emb[id] + pos_emb[m % S])
  const int32_t* ids; int S; int64_t tok_off, pos_off; float* x_out;  // embedding mode; x_out [M x d] may be null
  int V;                   // embedding mode: vocabulary size, ids are clamped into [0, V)
  int ids_rows;            // embedding mode: row r reads ids[r % ids_rows] (0 = M; stacked passes share one id array)
  ParamView pv; int64_t g_off, b_off;                                 // gamma / beta inside theta
  bf16_t* y; float* y32; float* mean; float* rstd;                    // y32 (fp32 copy for the residual path), mean, rstd may be null
  int M, d;
};
void launch_ln_fwd(hipStream_t, const LnFwdArgs&);
struct LnBwdArgs {
  const float* dy; const float* x; const float* mean; const float* rstd; const float* gamma;
  float* dx32; bf16_t* dx16;
  float* partial;          // [ceil(M / LN_BWD_ROWS)][3][d]: dgamma, dbeta, column sums of dx
  int M, d;
};
void launch_ln_bwd(hipStream_t, const LnBwdArgs&);
// out_v[c] = sum_r partial[r*stride + v*vstride + c] for the non-null outputs v = 0, 1, 2, in a fixed order
void launch_reduce_rows(hipStream_t, const float* partial, int nrows, int64_t stride, int64_t vstride, int N, float* out0,
                        float* out1, float* out2);
// the same for up to REDUCE_MAX_JOBS independent reductions in one launch (a job with fewer than three outputs
// leaves the trailing out[] null)
constexpr int REDUCE_MAX_JOBS = 4;
struct ReduceRowsJob { const float* partial; int nrows; int64_t stride, vstride; int N; float* out[3]; };
void launch_reduce_rows_multi(hipStream_t, const ReduceRowsJob* jobs, int count);
// first stage of the column sums of up to two bf16 matrices [M x N] (ld = N): partial [ceil(M / COLSUM_ROWS)][N]
struct ColsumJob { const bf16_t* X; int M, N; float* partial; };
void launch_colsum_partial_multi(hipStream_t, const ColsumJob* jobs, int count);
// column sums of a bf16 matrix [M x N] (ld = N) through partial [ceil(M / COLSUM_ROWS)][N]
void launch_colsum_bf16(hipStream_t, const bf16_t* X, int M, int N, float* partial, float* out);
// softmax(q k^T / 8) v for S in {64, 128, 256} (attention_supports), head width 64; qkv [B*S x 3d] bf16; out [B*S x d]
// bf16; lse [B][heads][S].  lens (device, or null = all S): sequence b has lens[b % lens_period] real tokens (clamped into
// [1, S]); keys beyond get no weight.
bool attention_supports(int S);
void launch_attention_fwd(hipStream_t, const bf16_t* qkv, bf16_t* out, float* lse, int B, int S, int heads, int d,
                          const int32_t* lens, int lens_period);
void launch_attention_bwd(hipStream_t, const bf16_t* qkv, const bf16_t* out, const bf16_t* dout, const float* lse,
                          bf16_t* dqkv, int B, int S, int heads, int d, const int32_t* lens, int lens_period);
// classifier on the position-0 hidden state: logits[b][c] = x[b*S] . Wc[c] + bc[c]
void launch_head_fwd(hipStream_t, const float* x, int S, int d, int B, int C, ParamView pv, int64_t wc_off, int64_t bc_off,
                     float* logits);
// dWc, dbc into grad; dx[b*S][:] = dlogits[b] . Wc written into the zero-filled dx [B*S x d]
void launch_head_bwd(hipStream_t, const float* x, int S, int d, int B, int C, const float* theta, int64_t wc_off,
                     int64_t bc_off, const float* dlogits, float* grad, float* dx);
// embedding gradients from demb [B*S x d]: pos_emb rows summed over the batch; tok_emb rows summed over the
// occurrences of each id in ascending position order (the tok_emb part of grad must be zero on entry)
// (ids outside [0, V) are clamped into it, here and in the forward pass)
void launch_embedding_bwd(hipStream_t, const float* demb, const int32_t* ids, int B, int S, int d, int V, float* g_tok, float* g_pos);


// ------------------------------------------------------------------ masked-token head (mlm_head.hip)
// ids_out = [ids_ft | ids_pt] ([n x S] token rows), y_out = [y_ft | 0], mask_out = [mask_ft (null = ones) | 0]
void launch_aux_cat(hipStream_t, const int32_t* ids_ft, const int32_t* y_ft, const uint8_t* mask_ft, int n_ft,
                    const int32_t* ids_pt, int n_pt, int S, int32_t* ids_out, int32_t* y_out, uint8_t* mask_out,
                    const int32_t* len_ft, const int32_t* len_pt, int32_t* len_out);
// out[(k P + j)][:] = X[k pass_rows + row_base + rows[j]][:], j < n_mask, k < nw; rows n_mask..P-1 zero; rows[] is
// clamped to [0, rows_in_batch)
void launch_gather_rows(hipStream_t, const bf16_t* X, int pass_rows, int row_base, int rows_in_batch, const int32_t* rows,
                        int n_mask, int P, int d, int nw, bf16_t* out);
// the same from an fp32 source, as the two-term split hi = bf16(x), lo = bf16(x - hi)
void launch_gather_rows_split(hipStream_t, const float* X, int pass_rows, int row_base, int rows_in_batch, const int32_t* rows,
                              int n_mask, int P, int d, int nw, bf16_t* hi, bf16_t* lo);
// loss_pos[k P + j] = logsumexp(Z[k P + j][:V]) - Z[k P + j][tgt[j]], lse_pos likewise (V % 4 == 0)
void launch_mlm_ce(hipStream_t, const float* Z, int V, int P, const int32_t* tgt, int n_mask, int nw, float* loss_pos,
                   float* lse_pos);
// dZ [P x V] bf16 = coef_pos[j] (softmax(Z[j]) - onehot(tgt[j])), zero rows from n_mask on
void launch_mlm_dz(hipStream_t, const float* Z, int V, const int32_t* tgt, const float* coef_pos, const float* lse_pos,
                   int n_mask, int P, bf16_t* dZ);
// dx[row_base + rows[j]][:] += sum_{k < nparts} part[k * part_stride + j * d + :]; the rows must be distinct
void launch_scatter_add_rows(hipStream_t, const float* part, int nparts, int64_t part_stride, int row_base, int rows_in_batch,
                             const int32_t* rows, int n_mask, int d, float* dx);

}  // namespace sama
