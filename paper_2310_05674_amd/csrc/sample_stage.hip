// Per-sample stage between the model's logits and its backward pass (Sec. 4.1):
//   l_i = logsumexp(z_i) - z_i[y_i];  w_i = sigmoid(W2 . relu(W1 l_i + b1) + b2);  B_eff = sum mask
//   BASE: coef_i = mask_i w_i / B_eff   META: coef_i = mask_i / B_eff   -> dz_i = coef_i (softmax(z_i) - e_{y_i})
//   GLAM: dL_base/dlambda = (1/B_eff) sum_i mask_i l_i dw(l_i; lambda)/dlambda   (weight-net backward only)
// With label correction (Sec. 4.1; Hc > 0) the BASE and GLAM modes compare the prediction with the corrected soft label
//   c_i = softmax(kappa e_{y_i} + W2c relu(W1c [e_{y_i}, softmax(z_i)] + b1c) + b2c),  l_i = -sum_k c_ik log softmax(z_i)_k,
//   BASE: dz_i = coef_i (softmax(z_i) - c_i)
//   GLAM: additionally d/dlambda_c = sum_i coef_i sum_k (-log p_ik) dc_ik/dlambda_c  (corrector backward; its inputs are constants)
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
  __shared__ float s_lc[MAX_CORR_HIDDEN * 2 * MAX_CORR_CLASSES + MAX_CORR_HIDDEN + MAX_CORR_CLASSES * MAX_CORR_HIDDEN + MAX_CORR_CLASSES];
  const int tid = threadIdx.x, H = a.H, B = a.B, C = a.C;
  const bool seq_mode = a.pos_loss != nullptr;          // per-sequence losses from masked-token positions
  const int Hc = (a.mode == STAGE_META || seq_mode) ? 0 : a.Hc;      // the clean batch keeps its hard labels
  for (int i = tid; i < 3 * H + 1; i += 256) s_lam[i] = a.lambda[i];
  const int nlc = Hc > 0 ? Hc * 2 * C + Hc + C * Hc + C : 0;
  for (int i = tid; i < nlc; i += 256) s_lc[i] = a.lambda[3 * H + 1 + i];
  __syncthreads();
  const float* W1 = s_lam; const float* b1 = s_lam + H; const float* W2 = s_lam + 2 * H;
  const double b2 = (double)s_lam[3 * H];
  const float* W1c = s_lc; const float* b1c = s_lc + Hc * 2 * C; const float* W2c = b1c + Hc; const float* b2c = W2c + C * Hc;

  double cnt = 0.0;
  for (int i = tid; i < B; i += 256) cnt += (a.mask == nullptr || a.mask[i] != 0) ? 1.0 : 0.0;
  const double beff = block_sum_d(cnt, red);
  const double inv_beff = beff > 0.0 ? 1.0 / beff : 0.0;

  double lsum = 0.0;
  float* s_cnt = s_lc;                                  // sequence mode: positions per sequence (the corrector is off)
  // wave w takes sequences w, w + 4, ...: its lanes stride over the positions (coalesced), keep the matching losses,
  // and a shuffle tree adds the 64 partial sums in a fixed order
  for (int i = tid >> 6; seq_mode && i < B; i += 4) {
    double acc = 0.0, n_i = 0.0;
    for (int j = tid & 63; j < a.n_pos; j += 64) {
      int r = a.pos_row[j];
      r = r < 0 ? 0 : (r >= B * a.S ? B * a.S - 1 : r);
      if (r / a.S == i) { acc += (double)a.pos_loss[j]; n_i += 1.0; }
    }
    for (int o = 32; o > 0; o >>= 1) { acc += __shfl_xor(acc, o, 64); n_i += __shfl_xor(n_i, o, 64); }
    if ((tid & 63) == 0) { s_l[i] = n_i > 0.0 ? acc / n_i : 0.0; s_cnt[i] = (float)n_i; }
  }
  if (seq_mode) __syncthreads();
  for (int i = tid; seq_mode && i < B; i += 256) {
    const double l = s_l[i];
    const double mk = (a.mask == nullptr || a.mask[i] != 0) ? 1.0 : 0.0;
    if (a.losses != nullptr) a.losses[i] = (float)l;
    double zz = b2;
    for (int h = 0; h < H; ++h) zz += (double)W2[h] * fmax((double)W1[h] * l + (double)b1[h], 0.0);
    const double w = 1.0 / (1.0 + exp(-zz));
    if (a.weights != nullptr) a.weights[i] = (float)w;
    if (a.mode == STAGE_EVAL) continue;
    if (a.mode == STAGE_GLAM) {
      s_dz[i] = w * (1.0 - w) * l * mk * inv_beff;
    } else {
      s_dz[i] = mk * w * inv_beff;
      lsum += s_dz[i] * l;
    }
  }
  if (seq_mode && a.mode != STAGE_GLAM && a.mode != STAGE_EVAL) {   // uniform over the block
    __syncthreads();
    for (int j = tid; j < a.n_pos; j += 256) {
      int r = a.pos_row[j];
      r = r < 0 ? 0 : (r >= B * a.S ? B * a.S - 1 : r);
      const int i = r / a.S;
      a.pos_coef[j] = (float)(s_dz[i] / (double)s_cnt[i]);     // s_cnt[i] >= 1: position j itself belongs to i
    }
  }
  for (int i = tid; !seq_mode && i < B; i += 256) {
    const float* z = a.logits + (int64_t)i * a.ld;
    double zmax = (double)z[0];
    for (int c = 1; c < C; ++c) zmax = fmax(zmax, (double)z[c]);
    double se = 0.0;
    for (int c = 0; c < C; ++c) se += exp((double)z[c] - zmax);
    const double lse = log(se) + zmax;
    const int yi = min(max(a.y[i], 0), C - 1);   // labels outside [0, C) are clamped
    const double mk = (a.mask == nullptr || a.mask[i] != 0) ? 1.0 : 0.0;
    double l;
    double cs[MAX_CORR_CLASSES];                       // corrected soft label (Hc > 0)
    if (Hc > 0) {
      double sc[MAX_CORR_CLASSES], pk[MAX_CORR_CLASSES];
      for (int k = 0; k < C; ++k) { sc[k] = (double)b2c[k] + (k == yi ? (double)a.kappa : 0.0); pk[k] = exp((double)z[k] - lse); }
      for (int j = 0; j < Hc; ++j) {
        double aj = (double)b1c[j] + (double)W1c[j * 2 * C + yi];
        for (int k = 0; k < C; ++k) aj += (double)W1c[j * 2 * C + C + k] * pk[k];
        if (aj > 0.0)
          for (int k = 0; k < C; ++k) sc[k] += (double)W2c[k * Hc + j] * aj;
      }
      double smax = sc[0];
      for (int k = 1; k < C; ++k) smax = fmax(smax, sc[k]);
      double ssum = 0.0;
      for (int k = 0; k < C; ++k) { cs[k] = exp(sc[k] - smax); ssum += cs[k]; }
      l = 0.0;
      for (int k = 0; k < C; ++k) { cs[k] /= ssum; l -= cs[k] * ((double)z[k] - lse); }
    } else {
      l = lse - (double)z[yi];
    }
    if (a.losses != nullptr) a.losses[i] = (float)l;
    s_l[i] = l;
    double w = 1.0;
    if (a.mode != STAGE_META) {
      double zz = b2;
      for (int h = 0; h < H; ++h) zz += (double)W2[h] * fmax((double)W1[h] * l + (double)b1[h], 0.0);
      w = 1.0 / (1.0 + exp(-zz));
    }
    if (a.weights != nullptr) a.weights[i] = (float)w;
    if (a.mode == STAGE_EVAL) continue;
    if (a.mode == STAGE_GLAM) {
      s_dz[i] = w * (1.0 - w) * l * mk * inv_beff;
      if (Hc > 0) {
        // ds_ik = c_ik (dc_ik - sum_k' c_ik' dc_ik'), dc_ik = -coef_i log p_ik; kept with p_i for the second phase
        const double coef = mk * w * inv_beff;
        double dot = 0.0;
        for (int k = 0; k < C; ++k) dot += cs[k] * (-coef * ((double)z[k] - lse));
        for (int k = 0; k < C; ++k) {
          a.corr_scratch[(int64_t)i * 2 * C + k] = cs[k] * (-coef * ((double)z[k] - lse) - dot);
          a.corr_scratch[(int64_t)i * 2 * C + C + k] = exp((double)z[k] - lse);
        }
      }
    } else {
      const double coef = mk * w * inv_beff;
      lsum += coef * l;
      for (int c = 0; c < C; ++c) {
        const double p = exp((double)z[c] - lse);
        const double target = Hc > 0 ? cs[c] : (c == yi ? 1.0 : 0.0);
        a.dlogits[(int64_t)i * C + c] = (float)(coef * (p - target));
      }
    }
  }
  if (a.mode != STAGE_GLAM) {
    const double L = block_sum_d(lsum, red);
    if (tid == 0) {
      if (a.loss_scalar) *a.loss_scalar = seq_mode ? *a.loss_scalar + (float)L : (float)L;
      if (a.loss_user) *a.loss_user = seq_mode ? *a.loss_user + (float)L : (float)L;
    }
    return;
  }
  __syncthreads();
  // weight-net backward: hidden unit h is shared by nch consecutive lanes of a wave (the largest power of two <= 256 / H,
  // at most 64), each walking a contiguous run of the samples in order; every lane then adds the nch partial sums of its
  // unit in chunk order through shuffles (fixed order, no atomics)
  {
    int nch = 1;
    while (2 * nch * H <= 256 && nch < 64) nch *= 2;
    const int run = (B + nch - 1) / nch;
    const int h = tid / nch, c = tid % nch;              // 256 / nch >= H units in one trip
    double part[3] = {0.0, 0.0, 0.0};                    // dW1, db1, dW2
    if (h < H) {
      const double w1 = W1[h], bb = b1[h], w2 = W2[h];
      const int i1 = (c + 1) * run < B ? (c + 1) * run : B;
      for (int i = c * run; i < i1; ++i) {
        const double l = s_l[i], dz = s_dz[i];
        const double pre = w1 * l + bb;
        if (pre > 0.0) {
          const double da = dz * w2;
          part[0] += da * l;
          part[1] += da;
          part[2] += dz * pre;
        }
      }
    }
    const int base = (tid & 63) & ~(nch - 1);
    double tot[3] = {0.0, 0.0, 0.0};
    for (int k = 0; k < nch; ++k)
#pragma unroll
      for (int q = 0; q < 3; ++q) tot[q] += __shfl(part[q], base + k, 64);
    if (h < H && c == 0) { a.glam[h] = tot[0]; a.glam[H + h] = tot[1]; a.glam[2 * H + h] = tot[2]; }
  }
  double dsum = 0.0;
  for (int i = tid; i < B; i += 256) dsum += s_dz[i];
  const double db2 = block_sum_d(dsum, red);
  if (tid == 0) a.glam[3 * H] = db2;
  if (Hc == 0) return;
  // corrector backward: thread j owns hidden unit j (row j of W1c, b1c[j], column j of W2c) and walks the samples in
  // order; threads Hc .. Hc + C - 1 own b2c.  The per-sample ds_i and p_i come back from the scratch written above
  // (same block: the barrier inside block_sum_d orders the writes before these reads).
  double* gc = a.glam + 3 * H + 1;
  for (int j = tid; j < Hc + C; j += 256) {
    if (j >= Hc) {
      const int k = j - Hc;
      double acc = 0.0;
      for (int i = 0; i < B; ++i) acc += a.corr_scratch[(int64_t)i * 2 * C + k];
      gc[Hc * 2 * C + Hc + C * Hc + k] = acc;
      continue;
    }
    double dW1[2 * MAX_CORR_CLASSES], dW2[MAX_CORR_CLASSES];
    for (int q = 0; q < 2 * C; ++q) dW1[q] = 0.0;
    for (int k = 0; k < C; ++k) dW2[k] = 0.0;
    double db1 = 0.0;
    for (int i = 0; i < B; ++i) {
      const double* ds = a.corr_scratch + (int64_t)i * 2 * C;
      const double* p = ds + C;
      const int yi = min(max(a.y[i], 0), C - 1);   // labels outside [0, C) are clamped
      double aj = (double)b1c[j] + (double)W1c[j * 2 * C + yi];
      for (int k = 0; k < C; ++k) aj += (double)W1c[j * 2 * C + C + k] * p[k];
      if (aj > 0.0) {
        double t = 0.0;
        for (int k = 0; k < C; ++k) { dW2[k] += ds[k] * aj; t += (double)W2c[k * Hc + j] * ds[k]; }
        db1 += t;
        dW1[yi] += t;
        for (int k = 0; k < C; ++k) dW1[C + k] += t * p[k];
      }
    }
    for (int q = 0; q < 2 * C; ++q) gc[j * 2 * C + q] = dW1[q];
    gc[Hc * 2 * C + j] = db1;
    for (int k = 0; k < C; ++k) gc[Hc * 2 * C + Hc + k * Hc + j] = dW2[k];
  }
}

// h = -(glam+ - glam-) / (2 eps); then (optionally) Adam on lambda.  A raised status word (counters[2]) or a
// hypergradient with a non-finite component zeroes h and skips the update; the latter raises the status word itself.
__global__ __launch_bounds__(256) void k_meta_update(MetaUpdateArgs a) {
  const float eps = a.scalars[0];
  bool skip = (a.counters[2] != 0) || !(eps > 0.f);
  int bad = 0;
  if (!skip)
    for (int i = threadIdx.x; i < a.nl; i += 256) {
      const double h = -(a.glam_p[i] - a.glam_m[i]) / (2.0 * (double)eps);
      if (!(fabs(h) <= 3.0e38)) bad = 1;   // NaN, infinite, or beyond what the fp32 outputs hold
    }
  if (__syncthreads_or(bad)) {   // every thread has read counters[2] above
    skip = true;
    if (threadIdx.x == 0) a.counters[2] = 1;
  }
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
  launch_kernel(ps, k_sample_stage, 1, 256, 0, st, a);
}
void launch_meta_update(hipStream_t st, const MetaUpdateArgs& a) { k_meta_update<<<1, 256, 0, st>>>(a); }

}  // namespace sama
