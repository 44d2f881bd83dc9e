// Host-side launchers of every gfx950 kernel in libsama.  Internal; the C ABI is include/sama.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "common.h"

namespace sama {

constexpr int EW_MAX_BLOCKS = 4096;  // grid cap of the elementwise kernels (also the size of the norm partials)
constexpr int MAX_BATCH = 2048;
constexpr int MAX_WNET_HIDDEN = 256;

// ------------------------------------------------------------------ elementwise chain (elementwise.hip)
struct AdamArgs {
  float beta1, one_m_beta1, beta2, one_m_beta2;
  float lr_c1;  // lr / (1 - beta1^t)
  float c2;     // 1 / sqrt(1 - beta2^t)
  float eps, weight_decay;
};
struct AdaptArgs {
  int mode;  // 0: Adam closed form, 1: scalar
  float scalar;
  float one_m_beta1, one_m_beta2;
  float lr_c1_c2;  // lr c1 c2
  float c2, eps;
};
void launch_adam(hipStream_t, const float* g, float* m, float* v, float* theta, bf16_t* theta16, int64_t n, int64_t n16,
                 const AdamArgs&);
void launch_sgd(hipStream_t, const float* g, float* theta, bf16_t* theta16, int64_t n, int64_t n16, float lr, float wd);
// v = D . gmeta, then eps = alpha/||v|| -> scalars[0], ||v|| -> scalars[1], status[0] = (norm unusable)
void launch_adapt_norm(hipStream_t, const float* g, const float* m, const float* v, const float* gmeta, float* vdir,
                       double* partial /*[EW_MAX_BLOCKS]*/, int64_t n, const AdaptArgs&, float alpha, float* scalars,
                       int64_t* status);
void launch_perturb_lo(hipStream_t, const float* theta, const float* vdir, const float* eps_ptr, bf16_t* lo_p,
                       bf16_t* lo_m, int64_t n16);
void launch_nudge(hipStream_t, float* theta, const float* vdir, const float* eps_ptr, bf16_t* theta16, int64_t n,
                  int64_t n16);
void launch_fill_f32(hipStream_t, float* p, float val, int64_t n);
void launch_copy_f32(hipStream_t, float* dst, const float* src, int64_t n);
void launch_to_bf16(hipStream_t, bf16_t* dst, const float* src, int64_t n);
void launch_fill_i64x4(hipStream_t, int64_t* p, int64_t a, int64_t b, int64_t c, int64_t d, int mask);

// ------------------------------------------------------------------ per-sample stage (sample_stage.hip)
enum { STAGE_BASE = 0, STAGE_META = 1, STAGE_GLAM = 2 };
struct SampleStageArgs {
  const float* logits;  // [B x C], row stride ld
  int ld, C, B, H, mode;
  const int32_t* y;
  const uint8_t* mask;  // may be null
  const float* lambda;  // [3H+1]
  float* losses;        // [B] out
  float* dlogits;       // [B x C] out, row stride C (BASE, META)
  float* loss_scalar;   // out: sum_i coef_i l_i
  float* loss_user;     // optional second destination
  double* glam;         // [3H+1] out (GLAM)
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

}  // namespace sama
