// Masked-token head of the auxiliary task (Sec. 4.3): token logits z_j = x_L[row_j] Wmlm^T + bmlm over the whole
// vocabulary at each masked position j, loss_j = logsumexp(z_j) - z_j[tgt_j].  The logit GEMMs run in gemm_bf16.hip;
// here are the HBM-bound kernels around them: gathering the masked rows, the softmax / cross-entropy pass over the
// [positions x V] logits and its backward, and the scatter of the hidden-state gradient back to the token rows.
// Position and target indices arrive from the caller's device buffers and are clamped into range before use.
#include "kernels.h"

namespace sama {
namespace {

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// ids_out = [ids_ft | ids_pt], y_out = [y_ft | 0], mask_out = [mask_ft or 1 | 0], len_out (if given) = [len_ft or S | len_pt or S]
__global__ __launch_bounds__(256) void k_aux_cat(const int32_t* ids_ft, const int32_t* y_ft, const uint8_t* mask_ft, int n_ft,
                                                 const int32_t* ids_pt, int n_pt, int S, int32_t* ids_out, int32_t* y_out,
                                                 uint8_t* mask_out, const int32_t* len_ft, const int32_t* len_pt, int32_t* len_out) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int nf = n_ft * S, n = (n_ft + n_pt) * S;
  if (i < n) ids_out[i] = i < nf ? ids_ft[i] : ids_pt[i - nf];
  if (i < n_ft + n_pt) {
    y_out[i] = i < n_ft ? y_ft[i] : 0;
    mask_out[i] = i < n_ft ? (mask_ft ? mask_ft[i] : (uint8_t)1) : (uint8_t)0;
    if (len_out != nullptr) len_out[i] = i < n_ft ? (len_ft ? len_ft[i] : S) : (len_pt ? len_pt[i - n_ft] : S);
  }
}

// out[(k P + j)][:] = X[k pass_rows + row_base + rows[j]][:] for j < n_mask, zero rows up to P (d % 8 == 0)
__global__ __launch_bounds__(128) void k_gather_rows(const bf16_t* X, int pass_rows, int row_base, int rows_in_batch,
                                                     const int32_t* rows, int n_mask, int P, int d, bf16_t* out) {
  const int j = blockIdx.x, k = blockIdx.y;
  uint4* o = reinterpret_cast<uint4*>(out + ((int64_t)k * P + j) * d);
  if (j < n_mask) {
    const int r = clampi(rows[j], 0, rows_in_batch - 1);
    const uint4* s = reinterpret_cast<const uint4*>(X + ((int64_t)k * pass_rows + row_base + r) * d);
    for (int c = threadIdx.x; c < d / 8; c += 128) o[c] = s[c];
  } else {
    for (int c = threadIdx.x; c < d / 8; c += 128) o[c] = make_uint4(0u, 0u, 0u, 0u);
  }
}

// The same rows from an fp32 source as a two-term split: hi = bf16(x), lo = bf16(x - hi)  (d % 4 == 0)
__global__ __launch_bounds__(128) void k_gather_rows_split(const float* X, int pass_rows, int row_base, int rows_in_batch,
                                                           const int32_t* rows, int n_mask, int P, int d, bf16_t* hi, bf16_t* lo) {
  const int j = blockIdx.x, k = blockIdx.y;
  uint2* oh = reinterpret_cast<uint2*>(hi + ((int64_t)k * P + j) * d);
  uint2* ol = reinterpret_cast<uint2*>(lo + ((int64_t)k * P + j) * d);
  if (j < n_mask) {
    const int r = clampi(rows[j], 0, rows_in_batch - 1);
    const float4* s = reinterpret_cast<const float4*>(X + ((int64_t)k * pass_rows + row_base + r) * d);
    for (int c = threadIdx.x; c < d / 4; c += 128) {
      const float4 x = s[c];
      const uint2 h = make_uint2(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w));
      oh[c] = h;
      ol[c] = make_uint2(pack_bf16x2(x.x - bf16_to_f32((bf16_t)h.x), x.y - bf16_to_f32((bf16_t)(h.x >> 16))),
                         pack_bf16x2(x.z - bf16_to_f32((bf16_t)h.y), x.w - bf16_to_f32((bf16_t)(h.y >> 16))));
    }
  } else {
    for (int c = threadIdx.x; c < d / 4; c += 128) { oh[c] = make_uint2(0u, 0u); ol[c] = make_uint2(0u, 0u); }
  }
}

// One workgroup of 1024 threads per masked position and pass: a single sweep over the row's V logits, four
// independent 16-byte loads per thread and trip, keeps a running maximum and the sum of exponentials relative to it in
// every thread; the 1024 pairs are merged in a fixed order (wave shuffles, then the 16 wave results serially).
constexpr int CE_THREADS = 1024;
__device__ __forceinline__ void ce_merge(float& m, float& s, float m2, float s2) {
  const float mm = fmaxf(m, m2);
  s = (m == mm ? s : s * __expf(m - mm)) + (m2 == mm ? s2 : s2 * __expf(m2 - mm));   // equal maxima (also -inf) need no scaling
  m = mm;
}
__global__ __launch_bounds__(CE_THREADS) void k_mlm_ce(const float* Z, int V, int P, const int32_t* tgt, int n_mask,
                                                       float* loss_pos, float* lse_pos) {
  __shared__ float s_m[CE_THREADS / 64];
  __shared__ float s_s[CE_THREADS / 64];
  const int j = blockIdx.x, k = blockIdx.y, tid = threadIdx.x;
  const float4* z4 = reinterpret_cast<const float4*>(Z + ((int64_t)k * P + j) * V);
  const int n4 = V / 4;                            // V % 4 == 0
  float m = -INFINITY, s = 0.f;
  for (int c0 = tid; c0 < n4; c0 += 4 * CE_THREADS) {
    float4 q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * CE_THREADS;
      q[u] = c < n4 ? z4[c] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
    float qm = m;
#pragma unroll
    for (int u = 0; u < 4; ++u) qm = fmaxf(qm, fmaxf(fmaxf(q[u].x, q[u].y), fmaxf(q[u].z, q[u].w)));
    if (qm > m) { s *= __expf(m - qm); m = qm; }
#pragma unroll
    for (int u = 0; u < 4; ++u) s += __expf(q[u].x - m) + __expf(q[u].y - m) + __expf(q[u].z - m) + __expf(q[u].w - m);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ce_merge(m, s, __shfl_xor(m, o, 64), __shfl_xor(s, o, 64));
  if ((tid & 63) == 0) { s_m[tid >> 6] = m; s_s[tid >> 6] = s; }
  __syncthreads();
  if (tid == 0) {
    float mm = s_m[0];
    for (int t = 1; t < CE_THREADS / 64; ++t) mm = fmaxf(mm, s_m[t]);
    double tot = 0.0;
    for (int t = 0; t < CE_THREADS / 64; ++t) tot += (double)s_s[t] * exp((double)s_m[t] - (double)mm);
    const double lse = log(tot) + (double)mm;
    const int t = clampi(tgt[j], 0, V - 1);
    loss_pos[k * P + j] = (float)(lse - (double)Z[((int64_t)k * P + j) * V + t]);
    lse_pos[k * P + j] = (float)lse;
  }
}

// dZ[j][c] = bf16(coef_j (exp(z_jc - lse_j) - [c == tgt_j])) for j < n_mask, zero rows up to P
__global__ __launch_bounds__(CE_THREADS) void k_mlm_dz(const float* Z, int V, const int32_t* tgt, const float* coef_pos,
                                                       const float* lse_pos, int n_mask, bf16_t* dZ) {
  const int j = blockIdx.x, tid = threadIdx.x;
  uint2* o = reinterpret_cast<uint2*>(dZ + (int64_t)j * V);
  const int n4 = V / 4;
  if (j >= n_mask) {
    for (int c = tid; c < n4; c += CE_THREADS) o[c] = make_uint2(0u, 0u);
    return;
  }
  const float4* z4 = reinterpret_cast<const float4*>(Z + (int64_t)j * V);
  const float coef = coef_pos[j], lse = lse_pos[j];
  const int t = clampi(tgt[j], 0, V - 1);
  for (int c0 = tid; c0 < n4; c0 += 4 * CE_THREADS) {
    float4 q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * CE_THREADS;
      q[u] = c < n4 ? z4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * CE_THREADS;
      if (c >= n4) break;
      float p[4] = {__expf(q[u].x - lse), __expf(q[u].y - lse), __expf(q[u].z - lse), __expf(q[u].w - lse)};
      if ((t >> 2) == c) p[t & 3] -= 1.f;
      o[c] = make_uint2(pack_bf16x2(coef * p[0], coef * p[1]), pack_bf16x2(coef * p[2], coef * p[3]));
    }
  }
}

// dx[row_base + rows[j]][:] += sum_k part[k][j][:]  (positions are distinct: one workgroup owns one row of dx)
__global__ __launch_bounds__(256) void k_scatter_add_rows(const float* part, int nparts, int64_t part_stride, int row_base,
                                                          int rows_in_batch, const int32_t* rows, int d, float* dx) {
  const int j = blockIdx.x;
  const int r = clampi(rows[j], 0, rows_in_batch - 1);
  float* o = dx + (int64_t)(row_base + r) * d;
  for (int c = threadIdx.x; c < d; c += 256) {
    float acc = 0.f;
    for (int k = 0; k < nparts; ++k) acc += part[k * part_stride + (int64_t)j * d + c];
    o[c] += acc;
  }
}

}  // namespace

void launch_aux_cat(hipStream_t st, const int32_t* ids_ft, const int32_t* y_ft, const uint8_t* mask_ft, int n_ft,
                    const int32_t* ids_pt, int n_pt, int S, int32_t* ids_out, int32_t* y_out, uint8_t* mask_out,
                    const int32_t* len_ft, const int32_t* len_pt, int32_t* len_out) {
  ProfScope ps(st, F_OTHER, 8.0 * (n_ft + n_pt) * S);
  launch_kernel(ps, k_aux_cat, ((n_ft + n_pt) * S + 255) / 256, 256, 0, st, ids_ft, y_ft, mask_ft, n_ft, ids_pt, n_pt, S, ids_out, y_out, mask_out,
                                                             len_ft, len_pt, len_out);
}
void launch_gather_rows(hipStream_t st, const bf16_t* X, int pass_rows, int row_base, int rows_in_batch, const int32_t* rows,
                        int n_mask, int P, int d, int nw, bf16_t* out) {
  ProfScope ps(st, F_OTHER, 4.0 * nw * P * d);
  launch_kernel(ps, k_gather_rows, dim3(P, nw), 128, 0, st, X, pass_rows, row_base, rows_in_batch, rows, n_mask, P, d, out);
}
void launch_gather_rows_split(hipStream_t st, const float* X, int pass_rows, int row_base, int rows_in_batch, const int32_t* rows,
                              int n_mask, int P, int d, int nw, bf16_t* hi, bf16_t* lo) {
  ProfScope ps(st, F_OTHER, 8.0 * nw * P * d);
  launch_kernel(ps, k_gather_rows_split, dim3(P, nw), 128, 0, st, X, pass_rows, row_base, rows_in_batch, rows, n_mask, P, d, hi, lo);
}
void launch_mlm_ce(hipStream_t st, const float* Z, int V, int P, const int32_t* tgt, int n_mask, int nw, float* loss_pos,
                   float* lse_pos) {
  ProfScope ps(st, F_MLM_SOFTMAX, 4.0 * nw * n_mask * (double)V);
  launch_kernel(ps, k_mlm_ce, dim3(n_mask, nw), CE_THREADS, 0, st, Z, V, P, tgt, n_mask, loss_pos, lse_pos);
}
void launch_mlm_dz(hipStream_t st, const float* Z, int V, const int32_t* tgt, const float* coef_pos, const float* lse_pos,
                   int n_mask, int P, bf16_t* dZ) {
  ProfScope ps(st, F_MLM_SOFTMAX, 6.0 * n_mask * (double)V + 2.0 * (P - n_mask) * (double)V);
  launch_kernel(ps, k_mlm_dz, P, CE_THREADS, 0, st, Z, V, tgt, coef_pos, lse_pos, n_mask, dZ);
}
void launch_scatter_add_rows(hipStream_t st, const float* part, int nparts, int64_t part_stride, int row_base, int rows_in_batch,
                             const int32_t* rows, int n_mask, int d, float* dx) {
  ProfScope ps(st, F_OTHER, 4.0 * (nparts + 2) * n_mask * d);
  launch_kernel(ps, k_scatter_add_rows, n_mask, 256, 0, st, part, nparts, part_stride, row_base, rows_in_batch, rows, d, dx);
}

}  // namespace sama
