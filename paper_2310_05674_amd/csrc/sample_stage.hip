// Per-sample stage between the model's logits and its backward pass (Sec. 4.1):
//   l_i = logsumexp(z_i) - z_i[y_i];  w_i = sigmoid(W2 . relu(W1 l_i + b1) + b2);  B_eff = sum mask
//   BASE: coef_i = mask_i w_i / B_eff   META: coef_i = mask_i / B_eff   -> dz_i = coef_i (softmax(z_i) - e_{y_i})
//   GLAM: dL_base/dlambda = (1/B_eff) sum_i mask_i l_i dw(l_i; lambda)/dlambda   (weight-net backward only)
// and the finite-difference combine + Adam step on lambda (Eq. 5, Table 4).
// Batches are at most a few hundred samples: one workgroup, samples staged in LDS, every sum in a fixed order,
// arithmetic in double so that the +-eps difference of Eq. 5 is not lost to rounding.
#include "common.h"
#include "kernels.h"

namespace sama {
namespace {

__device__ __forceinline__ double block_sum_d(double x, double* red) {
  __syncthreads();
  red[threadIdx.x] = x;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  const double r = red[0];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(256) void k_sample_stage(SampleStageArgs a) {
  __shared__ double s_l[MAX_BATCH];    // l_i
  __shared__ double s_dz[MAX_BATCH];   // per-sample dL/dz of the weight net (GLAM) or coef (BASE/META)
  __shared__ float s_lam[3 * MAX_WNET_HIDDEN + 1];
  __shared__ double red[256];
  const int tid = threadIdx.x, H = a.H, B = a.B, C = a.C;
  for (int i = tid; i < 3 * H + 1; i += 256) s_lam[i] = a.lambda[i];
  __syncthreads();
  const float* W1 = s_lam; const float* b1 = s_lam + H; const float* W2 = s_lam + 2 * H;
  const double b2 = (double)s_lam[3 * H];

  double cnt = 0.0;
  for (int i = tid; i < B; i += 256) cnt += (a.mask == nullptr || a.mask[i] != 0) ? 1.0 : 0.0;
  const double beff = block_sum_d(cnt, red);
  const double inv_beff = beff > 0.0 ? 1.0 / beff : 0.0;

  double lsum = 0.0;
  for (int i = tid; i < B; i += 256) {
    const float* z = a.logits + (int64_t)i * a.ld;
    double zmax = (double)z[0];
    for (int c = 1; c < C; ++c) zmax = fmax(zmax, (double)z[c]);
    double se = 0.0;
    for (int c = 0; c < C; ++c) se += exp((double)z[c] - zmax);
    const double lse = log(se) + zmax;
    const int yi = a.y[i];
    const double l = lse - (double)z[yi];
    const double mk = (a.mask == nullptr || a.mask[i] != 0) ? 1.0 : 0.0;
    a.losses[i] = (float)l;
    s_l[i] = l;
    double w = 1.0;
    if (a.mode != STAGE_META) {
      double zz = b2;
      for (int h = 0; h < H; ++h) zz += (double)W2[h] * fmax((double)W1[h] * l + (double)b1[h], 0.0);
      w = 1.0 / (1.0 + exp(-zz));
    }
    if (a.mode == STAGE_GLAM) {
      s_dz[i] = w * (1.0 - w) * l * mk * inv_beff;
    } else {
      const double coef = mk * w * inv_beff;
      lsum += coef * l;
      for (int c = 0; c < C; ++c) {
        const double p = exp((double)z[c] - lse);
        a.dlogits[(int64_t)i * C + c] = (float)(coef * (p - (c == yi ? 1.0 : 0.0)));
      }
    }
  }
  if (a.mode != STAGE_GLAM) {
    const double L = block_sum_d(lsum, red);
    if (tid == 0) {
      if (a.loss_scalar) *a.loss_scalar = (float)L;
      if (a.loss_user) *a.loss_user = (float)L;
    }
    return;
  }
  __syncthreads();
  // weight-net backward: thread h owns hidden unit h and walks the samples in order
  for (int h = tid; h < H; h += 256) {
    const double w1 = W1[h], bb = b1[h], w2 = W2[h];
    double dW1 = 0.0, db1 = 0.0, dW2 = 0.0;
    for (int i = 0; i < B; ++i) {
      const double l = s_l[i], dz = s_dz[i];
      const double pre = w1 * l + bb;
      if (pre > 0.0) {
        const double da = dz * w2;
        dW1 += da * l;
        db1 += da;
        dW2 += dz * pre;
      }
    }
    a.glam[h] = dW1; a.glam[H + h] = db1; a.glam[2 * H + h] = dW2;
  }
  double dsum = 0.0;
  for (int i = tid; i < B; i += 256) dsum += s_dz[i];
  const double db2 = block_sum_d(dsum, red);
  if (tid == 0) a.glam[3 * H] = db2;
}

// h = -(glam+ - glam-) / (2 eps); then (optionally) Adam on lambda.  A raised status word (counters[2]) zeroes h
// and skips the update.
__global__ __launch_bounds__(256) void k_meta_update(MetaUpdateArgs a) {
  const float eps = a.scalars[0];
  const bool skip = (a.counters[2] != 0) || !(eps > 0.f);
  const int64_t t = a.counters[1] + 1;
  const double c1 = 1.0 / (1.0 - pow((double)a.beta1, (double)t));
  const double c2 = 1.0 / sqrt(1.0 - pow((double)a.beta2, (double)t));
  for (int i = threadIdx.x; i < a.nl; i += 256) {
    const double gp = a.glam_p[i], gm = a.glam_m[i];
    const double h = skip ? 0.0 : -(gp - gm) / (2.0 * (double)eps);
    a.hypergrad[i] = (float)h;
    if (a.hypergrad_user) a.hypergrad_user[i] = (float)h;
    a.glam_p_f32[i] = (float)gp;
    a.glam_m_f32[i] = (float)gm;
    if (a.do_update && !skip) {
      const double m = (double)a.beta1 * a.meta_m[i] + (1.0 - (double)a.beta1) * h;
      const double v = (double)a.beta2 * a.meta_v[i] + (1.0 - (double)a.beta2) * h * h;
      a.meta_m[i] = (float)m;
      a.meta_v[i] = (float)v;
      a.lambda[i] = (float)((double)a.lambda[i] - (double)a.lr * c1 * m / (c2 * sqrt(v) + (double)a.eps));
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (a.eps_user) *a.eps_user = skip ? 0.f : eps;
    if (a.do_update && !skip) a.counters[1] = t;
  }
}
}  // namespace

void launch_sample_stage(hipStream_t st, const SampleStageArgs& a) {
  ProfScope ps(st, F_SAMPLE_STAGE, 0.0);
  k_sample_stage<<<1, 256, 0, st>>>(a);
}
void launch_meta_update(hipStream_t st, const MetaUpdateArgs& a) { k_meta_update<<<1, 256, 0, st>>>(a); }

}  // namespace sama
