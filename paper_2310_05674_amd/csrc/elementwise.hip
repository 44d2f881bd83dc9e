// The HBM-bound elementwise chain of one SAMA iteration over the n base parameters:
//   base solver update (Adam / SGD)                                  -- Sec. 2, Kingma & Ba Alg. 1
//   adaptation v = (du/dg) . dL_meta/dtheta fused with ||v||^2       -- Eq. 4-5, App. C
//   eps = alpha / ||v||_2                                            -- below Eq. 5
//   low-order halves of theta +- eps v for the two extra passes      -- Eq. 5
//   nudge theta <- theta - eps v                                     -- end of Sec. 3.2
// Each kernel streams every array exactly once with 16-byte accesses; nothing is re-read.
#include "common.h"
#include "kernels.h"

namespace sama {

namespace {
// Streaming layout of every kernel below (measured best on MI355X for a 4-read / 4-write stream mix, 5.7 TB/s):
// a block owns a contiguous run of EW_U * 256 16-byte vectors per trip, a thread takes EW_U of them 256 apart, all
// loads of a trip are issued before the first store, and loads and stores are non-temporal (nothing is reused).
constexpr int EW_THREADS = 256;
constexpr int EW_VEC = 4;
constexpr int EW_U = 4;
constexpr int EW_TRIP = EW_U * EW_THREADS;   // vectors per block per trip
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

inline int ew_grid(int64_t n) {
  int64_t b = (n / EW_VEC + EW_TRIP - 1) / EW_TRIP;
  if (b < 1) b = 1;
  if (b > EW_MAX_BLOCKS) b = EW_MAX_BLOCKS;
  return (int)b;
}

__device__ __forceinline__ f4 ld_nt(const float* p, int64_t j) { return __builtin_nontemporal_load(reinterpret_cast<const f4*>(p) + j); }
__device__ __forceinline__ void st_nt(float* p, int64_t j, f4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f4*>(p) + j); }
// four bf16 (round to nearest even) at element offset 4 j
__device__ __forceinline__ void st_bf16x4_nt(bf16_t* p, int64_t j, float a, float b, float c, float d) {
  u2 pk;
  pk.x = pack_bf16x2(a, b);
  pk.y = pack_bf16x2(c, d);
  __builtin_nontemporal_store(pk, reinterpret_cast<u2*>(p) + j);
}
// the bf16 copy covers only the first n16 elements: whole vectors inside it, element by element across its end
__device__ __forceinline__ void st_bf16_prefix(bf16_t* p, int64_t j, int64_t n16, f4 t) {
  if (p == nullptr) return;
  if (j * EW_VEC + EW_VEC <= n16) st_bf16x4_nt(p, j, t.x, t.y, t.z, t.w);
  else
    for (int e = 0; e < EW_VEC; ++e)
      if (j * EW_VEC + e < n16) p[j * EW_VEC + e] = f32_to_bf16(t[e]);
}
__device__ __forceinline__ float bf16_residual(float t) { return t - bf16_to_f32(f32_to_bf16(t)); }

// ---------------------------------------------------------------------------------------------------------
// Adam: m' = b1 m + (1-b1) g ; v' = b2 v + (1-b2) g^2 ; theta' = theta - lr c1 m' / (c2 sqrt(v') + eps)
// with c1 = 1/(1-b1^t), c2 = 1/sqrt(1-b2^t) computed on the host in double.  Optionally refreshes the bf16
// working copy of the first n16 elements (the GEMM weight matrices).
__device__ __forceinline__ void adam_one(float g, float& m, float& v, float& th, const AdamArgs& a) {   // g includes the L2 term
  m = fmaf(a.beta1, m, a.one_m_beta1 * g);
  v = fmaf(a.beta2, v, a.one_m_beta2 * g * g);
  th = th - a.lr_c1 * m / (fmaf(a.c2, sqrtf(v), a.eps));
}

__global__ __launch_bounds__(EW_THREADS) void k_adam(float* __restrict__ g, float* __restrict__ m,
                                                     float* __restrict__ v, float* __restrict__ theta,
                                                     bf16_t* __restrict__ theta16, int64_t n, int64_t n16,
                                                     AdamArgs a) {
  if (a.dev != nullptr) { a.lr_c1 = a.dev[0]; a.c2 = a.dev[1]; }
  const int64_t nv = n / EW_VEC, trip = (int64_t)gridDim.x * EW_TRIP;
  for (int64_t base = (int64_t)blockIdx.x * EW_TRIP + threadIdx.x; base < nv; base += trip) {
    f4 G[EW_U], M[EW_U], V[EW_U], T[EW_U];
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) { G[u] = ld_nt(g, j); M[u] = ld_nt(m, j); V[u] = ld_nt(v, j); T[u] = ld_nt(theta, j); }
    }
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) {
#pragma unroll
        for (int e = 0; e < EW_VEC; ++e) {
          float mm = M[u][e], vv = V[u][e], tt = T[u][e];
          G[u][e] = fmaf(a.weight_decay, tt, G[u][e]);
          adam_one(G[u][e], mm, vv, tt, a);
          M[u][e] = mm; V[u][e] = vv; T[u][e] = tt;
        }
        if (a.weight_decay != 0.f) st_nt(g, j, G[u]);   // the gradient the solver was given, kept for the adaptation
        st_nt(m, j, M[u]); st_nt(v, j, V[u]); st_nt(theta, j, T[u]);
        st_bf16_prefix(theta16, j, n16, T[u]);
        if (a.lo != nullptr) {
          f4 r;
          r.x = bf16_residual(T[u].x); r.y = bf16_residual(T[u].y); r.z = bf16_residual(T[u].z); r.w = bf16_residual(T[u].w);
          st_bf16_prefix(a.lo, j, n16, r);
        }
      }
    }
  }
  // ragged tail (n not a multiple of 4)
  const int64_t k = nv * EW_VEC + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n) {
    float mm = m[k], vv = v[k], tt = theta[k];
    const float ge = fmaf(a.weight_decay, tt, g[k]);
    adam_one(ge, mm, vv, tt, a);
    if (a.weight_decay != 0.f) g[k] = ge;
    m[k] = mm; v[k] = vv; theta[k] = tt;
    if (theta16 != nullptr && k < n16) theta16[k] = f32_to_bf16(tt);
    if (a.lo != nullptr && k < n16) a.lo[k] = f32_to_bf16(bf16_residual(tt));
  }
}

__global__ void k_step_scalars(int64_t* counters, int advance, float lr, float beta1, float beta2, float* step) {
  const int64_t t = counters[0] + advance;
  if (advance != 0) counters[0] = t;
  if (t < 1) return;
  const double c1 = 1.0 / (1.0 - pow((double)beta1, (double)t));
  const double c2 = 1.0 / sqrt(1.0 - pow((double)beta2, (double)t));
  step[0] = (float)((double)lr * c1); step[1] = (float)c2;
  step[2] = (float)((double)lr * c1 * c2); step[3] = (float)c2;
}

// SGD: theta' = theta - lr b, b = mu b_prev + (g + wd theta) (heavy-ball momentum; b lives in `buf`, untouched when
// mu = 0).  Also refreshes the bf16 working copy and its residual half over the first n16 elements.
__global__ __launch_bounds__(EW_THREADS) void k_sgd(float* __restrict__ g, float* __restrict__ buf, float* __restrict__ theta,
                                                    bf16_t* __restrict__ theta16, bf16_t* __restrict__ lo, int64_t n,
                                                    int64_t n16, float lr, float wd, float mu) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride) {
    float t = theta[k];
    const float ge = fmaf(wd, t, g[k]);
    if (wd != 0.f) g[k] = ge;   // the gradient the solver was given
    float b = ge;
    if (mu != 0.f) { b = fmaf(mu, buf[k], ge); buf[k] = b; }
    t = t - lr * b;
    theta[k] = t;
    if (theta16 != nullptr && k < n16) theta16[k] = f32_to_bf16(t);
    if (lo != nullptr && k < n16) lo[k] = f32_to_bf16(bf16_residual(t));
  }
}

// ---------------------------------------------------------------------------------------------------------
// Adaptation fused with the squared norm.  mode 0: Adam, D = lr c1 c2 [(1-b1) v' - (1-b2) m' g] / [s (c2 s + eps)^2],
// s = sqrt(v'), D = 0 where s = 0 (m', v' are the moments after the step that consumed g; the eps term of the
// numerator is dropped as in App. C).  mode 1: D = scalar (lr for SGD, 1 for SAMA-NA).
__device__ __forceinline__ float adapt_one(float g, float m, float v, float gm, const AdaptArgs& a) {
  if (a.mode != 0) return a.scalar * gm;
  const float s = sqrtf(v);
  const float num = a.one_m_beta1 * v - a.one_m_beta2 * m * g;
  const float q = fmaf(a.c2, s, a.eps);
  const float D = s > 0.f ? a.lr_c1_c2 * num / (s * q * q) : 0.f;
  return D * gm;
}

__global__ __launch_bounds__(EW_THREADS) void k_adapt_norm(const float* __restrict__ g, const float* __restrict__ m,
                                                           const float* __restrict__ v, const float* __restrict__ gmeta,
                                                           float* __restrict__ vdir, double* __restrict__ partial,
                                                           int64_t n, AdaptArgs a) {
  __shared__ float red[16];
  if (a.dev != nullptr) { a.lr_c1_c2 = a.dev[2]; a.c2 = a.dev[3]; }
  const int64_t nv = n / EW_VEC, trip = (int64_t)gridDim.x * EW_TRIP;
  float acc = 0.f;
  for (int64_t base = (int64_t)blockIdx.x * EW_TRIP + threadIdx.x; base < nv; base += trip) {
    f4 G[EW_U], M[EW_U], V[EW_U], Q[EW_U];
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) {
        Q[u] = ld_nt(gmeta, j);
        if (a.mode == 0) { G[u] = ld_nt(g, j); M[u] = ld_nt(m, j); V[u] = ld_nt(v, j); }
      }
    }
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) {
        f4 o;
        if (a.mode == 0) {
          o.x = adapt_one(G[u].x, M[u].x, V[u].x, Q[u].x, a);
          o.y = adapt_one(G[u].y, M[u].y, V[u].y, Q[u].y, a);
          o.z = adapt_one(G[u].z, M[u].z, V[u].z, Q[u].z, a);
          o.w = adapt_one(G[u].w, M[u].w, V[u].w, Q[u].w, a);
        } else {
          o = a.scalar * Q[u];
        }
        st_nt(vdir, j, o);
        acc = fmaf(o.x, o.x, acc); acc = fmaf(o.y, o.y, acc); acc = fmaf(o.z, o.z, acc); acc = fmaf(o.w, o.w, acc);
      }
    }
  }
  const int64_t k = nv * EW_VEC + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n) {
    const float o = a.mode == 0 ? adapt_one(g[k], m[k], v[k], gmeta[k], a) : a.scalar * gmeta[k];
    vdir[k] = o;
    acc = fmaf(o, o, acc);
  }
  const float s = block_sum(acc, red);
  if (threadIdx.x == 0) partial[blockIdx.x] = (double)s;
}

// Second stage: fixed-order sum of the per-block partials in double, eps = alpha / ||v||.
// scalars[0] = eps, scalars[1] = ||v||.  A zero or non-finite norm gives eps = 0 and raises status[0] = 1
// (status is cleared to 0 otherwise), which turns the rest of the meta step into a no-op.
__global__ __launch_bounds__(1024) void k_eps_from_partials(const double* __restrict__ partial, int nparts, float alpha,
                                                            float* __restrict__ scalars, int64_t* __restrict__ status) {
  __shared__ double red[1024];
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;   // four loads in flight per thread: the sweep is latency-bound
  int i = threadIdx.x;
  for (; i + 3072 < nparts; i += 4096) {
    s0 += partial[i]; s1 += partial[i + 1024]; s2 += partial[i + 2048]; s3 += partial[i + 3072];
  }
  for (; i < nparts; i += 1024) s0 += partial[i];
  red[threadIdx.x] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double nrm = sqrt(red[0]);
    const bool ok = (nrm > 0.0) && (nrm < 1e300) && (nrm == nrm);
    const float eps = ok ? (float)((double)alpha / nrm) : 0.f;
    const bool ok2 = ok && eps > 0.f && eps < 3.0e38f;
    scalars[0] = ok2 ? eps : 0.f;
    scalars[1] = (float)nrm;
    status[0] = ok2 ? 0 : 1;
  }
}

// ---------------------------------------------------------------------------------------------------------
// Low-order halves for the +-eps v passes: lo+-[k] = bf16((theta[k] +- eps v[k]) - float(bf16(theta[k]))).
// The GEMMs of those passes contract with hi + lo, hi = the bf16 working copy, so the perturbation survives
// even where eps |v| is far below one bf16 ulp of theta.
__global__ __launch_bounds__(EW_THREADS) void k_perturb_lo(const float* __restrict__ theta, const float* __restrict__ vdir,
                                                           const float* __restrict__ eps_ptr, bf16_t* __restrict__ lo_p,
                                                           bf16_t* __restrict__ lo_m, int64_t n16) {
  const float eps = *eps_ptr;
  const int64_t nv = n16 / EW_VEC, trip = (int64_t)gridDim.x * EW_TRIP;
  for (int64_t base = (int64_t)blockIdx.x * EW_TRIP + threadIdx.x; base < nv; base += trip) {
    f4 T[EW_U], V[EW_U];
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) { T[u] = ld_nt(theta, j); V[u] = ld_nt(vdir, j); }
    }
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) {
        float p[4], q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float hi = bf16_to_f32(f32_to_bf16(T[u][e]));
          p[e] = fmaf(eps, V[u][e], T[u][e]) - hi;
          q[e] = fmaf(-eps, V[u][e], T[u][e]) - hi;
        }
        st_bf16x4_nt(lo_p, j, p[0], p[1], p[2], p[3]);
        st_bf16x4_nt(lo_m, j, q[0], q[1], q[2], q[3]);
      }
    }
  }
  const int64_t k = nv * EW_VEC + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n16) {
    const float hi = bf16_to_f32(f32_to_bf16(theta[k]));
    lo_p[k] = f32_to_bf16(fmaf(eps, vdir[k], theta[k]) - hi);
    lo_m[k] = f32_to_bf16(fmaf(-eps, vdir[k], theta[k]) - hi);
  }
}

// The same for a step that will also be applied (sama_meta_step): theta <- theta - eps v on the GEMM block right
// away, hi = bf16 of the NEW theta, lo+- = bf16((theta_old +- eps v) - hi).  The +- passes then contract with the same
// values theta_old +- eps v as above, and the later nudge only has the non-GEMM tail left.  eps = 0 (a skipped
// step): theta and hi stay as they are, lo+- = the plain residual.
__global__ __launch_bounds__(EW_THREADS) void k_perturb_nudge(float* __restrict__ theta, const float* __restrict__ vdir,
                                                              const float* __restrict__ eps_ptr, bf16_t* __restrict__ theta16,
                                                              bf16_t* __restrict__ lo_p, bf16_t* __restrict__ lo_m, int64_t n16) {
  const float eps = *eps_ptr;
  const bool skip = eps == 0.f;
  const int64_t nv = n16 / EW_VEC, trip = (int64_t)gridDim.x * EW_TRIP;
  for (int64_t base = (int64_t)blockIdx.x * EW_TRIP + threadIdx.x; base < nv; base += trip) {
    f4 T[EW_U], V[EW_U];
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) { T[u] = ld_nt(theta, j); V[u] = ld_nt(vdir, j); }
    }
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) {
        f4 tn;
        float p[4], q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          tn[e] = skip ? T[u][e] : fmaf(-eps, V[u][e], T[u][e]);
          const float hi = bf16_to_f32(f32_to_bf16(tn[e]));
          p[e] = (skip ? T[u][e] : fmaf(eps, V[u][e], T[u][e])) - hi;
          q[e] = tn[e] - hi;
        }
        if (!skip) {
          st_nt(theta, j, tn);
          st_bf16x4_nt(theta16, j, tn.x, tn.y, tn.z, tn.w);
        }
        st_bf16x4_nt(lo_p, j, p[0], p[1], p[2], p[3]);
        st_bf16x4_nt(lo_m, j, q[0], q[1], q[2], q[3]);
      }
    }
  }
}

__global__ __launch_bounds__(EW_THREADS) void k_residual_lo(const float* __restrict__ theta, bf16_t* __restrict__ lo, int64_t n16) {
  const int64_t nv = n16 / EW_VEC, trip = (int64_t)gridDim.x * EW_TRIP;
  for (int64_t base = (int64_t)blockIdx.x * EW_TRIP + threadIdx.x; base < nv; base += trip) {
    f4 T[EW_U];
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) T[u] = ld_nt(theta, j);
    }
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) st_bf16x4_nt(lo, j, bf16_residual(T[u].x), bf16_residual(T[u].y), bf16_residual(T[u].z), bf16_residual(T[u].w));
    }
  }
  const int64_t k = nv * EW_VEC + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n16) lo[k] = f32_to_bf16(bf16_residual(theta[k]));
}

// theta <- theta - eps v (and the bf16 working copy with its residual half).  eps = 0 or a raised status word (a
// skipped step) leaves everything as it is.
__global__ __launch_bounds__(EW_THREADS) void k_nudge(float* __restrict__ theta, const float* __restrict__ vdir,
                                                      const float* __restrict__ eps_ptr, const int64_t* __restrict__ status,
                                                      bf16_t* __restrict__ theta16, bf16_t* __restrict__ lo, int64_t n, int64_t n16) {
  const float eps = *eps_ptr;
  if (eps == 0.f || (status != nullptr && *status != 0)) return;
  const int64_t nv = n / EW_VEC, trip = (int64_t)gridDim.x * EW_TRIP;
  for (int64_t base = (int64_t)blockIdx.x * EW_TRIP + threadIdx.x; base < nv; base += trip) {
    f4 T[EW_U], V[EW_U];
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) { T[u] = ld_nt(theta, j); V[u] = ld_nt(vdir, j); }
    }
#pragma unroll
    for (int u = 0; u < EW_U; ++u) {
      const int64_t j = base + u * EW_THREADS;
      if (j < nv) {
        f4 t;
        t.x = fmaf(-eps, V[u].x, T[u].x); t.y = fmaf(-eps, V[u].y, T[u].y);
        t.z = fmaf(-eps, V[u].z, T[u].z); t.w = fmaf(-eps, V[u].w, T[u].w);
        st_nt(theta, j, t);
        st_bf16_prefix(theta16, j, n16, t);
        if (lo != nullptr) {
          f4 r;
          r.x = bf16_residual(t.x); r.y = bf16_residual(t.y); r.z = bf16_residual(t.z); r.w = bf16_residual(t.w);
          st_bf16_prefix(lo, j, n16, r);
        }
      }
    }
  }
  const int64_t k = nv * EW_VEC + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n) {
    const float t = fmaf(-eps, vdir[k], theta[k]);
    theta[k] = t;
    if (theta16 != nullptr && k < n16) theta16[k] = f32_to_bf16(t);
    if (lo != nullptr && k < n16) lo[k] = f32_to_bf16(bf16_residual(t));
  }
}

// Takes back the nudge k_perturb_nudge applied to the first n16 elements when the step turned out to be skipped after
// all (a non-finite hypergradient: status raised although eps > 0): theta <- theta + eps v, with the working copy and
// its residual half.  Returns at once otherwise, which is the ordinary case.
__global__ __launch_bounds__(EW_THREADS) void k_unnudge(float* __restrict__ theta, const float* __restrict__ vdir,
                                                        const float* __restrict__ eps_ptr, const int64_t* __restrict__ status,
                                                        bf16_t* __restrict__ theta16, bf16_t* __restrict__ lo, int64_t n16) {
  const float eps = *eps_ptr;
  if (*status == 0 || eps == 0.f) return;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n16; k += stride) {
    const float t = fmaf(eps, vdir[k], theta[k]);
    theta[k] = t;
    theta16[k] = f32_to_bf16(t);
    lo[k] = f32_to_bf16(bf16_residual(t));
  }
}

__global__ __launch_bounds__(EW_THREADS) void k_fill_f32(float* __restrict__ p, float val, int64_t n) {
  const int64_t nv = n / EW_VEC;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const float4 v4 = make_float4(val, val, val, val);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nv; i += stride) reinterpret_cast<float4*>(p)[i] = v4;
  const int64_t k = nv * EW_VEC + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n) p[k] = val;
}

__global__ __launch_bounds__(EW_THREADS) void k_copy_f32(float* __restrict__ dst, const float* __restrict__ src, int64_t n) {
  const int64_t nv = n / EW_VEC;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nv; i += stride)
    reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
  const int64_t k = nv * EW_VEC + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k < n) dst[k] = src[k];
}

__global__ __launch_bounds__(EW_THREADS) void k_to_bf16(bf16_t* __restrict__ dst, const float* __restrict__ src, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += stride) dst[k] = f32_to_bf16(src[k]);
}

__global__ void k_fill_i64(int64_t* p, int64_t a, int64_t b, int64_t c, int64_t d, int mask) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    if (mask & 1) p[0] = a;
    if (mask & 2) p[1] = b;
    if (mask & 4) p[2] = c;
    if (mask & 8) p[3] = d;
  }
}
}  // namespace

void launch_adam(hipStream_t st, float* g, float* m, float* v, float* theta, bf16_t* theta16, int64_t n,
                 int64_t n16, const AdamArgs& a) {
  if (n <= 0) return;
  ProfScope ps(st, F_ADAM, 28.0 * n + (theta16 ? 2.0 * n16 : 0.0) + (a.lo ? 2.0 * n16 : 0.0));
  launch_kernel(ps, k_adam, ew_grid(n), EW_THREADS, 0, st, g, m, v, theta, theta16, n, n16, a);
}
void launch_step_scalars(hipStream_t st, int64_t* counters, int advance, float lr, float beta1, float beta2, float* step) {
  k_step_scalars<<<1, 1, 0, st>>>(counters, advance, lr, beta1, beta2, step);
}
void launch_sgd(hipStream_t st, float* g, float* buf, float* theta, bf16_t* theta16, bf16_t* lo, int64_t n, int64_t n16,
                float lr, float wd, float mu) {
  if (n <= 0) return;
  k_sgd<<<ew_grid(n), EW_THREADS, 0, st>>>(g, buf, theta, theta16, lo, n, n16, lr, wd, mu);
}
void launch_adapt_norm(hipStream_t st, const float* g, const float* m, const float* v, const float* gmeta, float* vdir,
                       double* partial, int64_t n, const AdaptArgs& a, float alpha, float* scalars, int64_t* status) {
  const int grid = ew_grid(n);
  ProfScope ps(st, F_ADAPT_NORM, (a.mode == 0 ? 20.0 : 8.0) * n);
  launch_kernel(ps, k_adapt_norm, grid, EW_THREADS, 0, st, g, m, v, gmeta, vdir, partial, n, a);
  k_eps_from_partials<<<1, 1024, 0, st>>>(partial, grid, alpha, scalars, status);
}
int launch_adapt_slice(hipStream_t st, const float* g, const float* m, const float* v, const float* gmeta, float* vdir,
                       double* partial, int64_t n, const AdaptArgs& a, int max_blocks) {
  if (n <= 0) return 0;
  int grid = ew_grid(n);
  if (grid > max_blocks) grid = max_blocks;
  ProfScope ps(st, F_ADAPT_NORM, (a.mode == 0 ? 20.0 : 8.0) * n);
  launch_kernel(ps, k_adapt_norm, grid, EW_THREADS, 0, st, g, m, v, gmeta, vdir, partial, n, a);
  return grid;
}
void launch_eps_from_partials(hipStream_t st, const double* partial, int count, float alpha, float* scalars, int64_t* status) {
  k_eps_from_partials<<<1, 1024, 0, st>>>(partial, count, alpha, scalars, status);
}
void launch_perturb_lo(hipStream_t st, const float* theta, const float* vdir, const float* eps_ptr, bf16_t* lo_p,
                       bf16_t* lo_m, int64_t n16) {
  if (n16 <= 0) return;
  ProfScope ps(st, F_PERTURB, 12.0 * n16);
  launch_kernel(ps, k_perturb_lo, ew_grid(n16), EW_THREADS, 0, st, theta, vdir, eps_ptr, lo_p, lo_m, n16);
}
void launch_perturb_nudge(hipStream_t st, float* theta, const float* vdir, const float* eps_ptr, bf16_t* theta16, bf16_t* lo_p,
                          bf16_t* lo_m, int64_t n16) {
  if (n16 <= 0) return;
  ProfScope ps(st, F_PERTURB, 18.0 * n16);
  launch_kernel(ps, k_perturb_nudge, ew_grid(n16), EW_THREADS, 0, st, theta, vdir, eps_ptr, theta16, lo_p, lo_m, n16);
}
void launch_residual_lo(hipStream_t st, const float* theta, bf16_t* lo, int64_t n16) {
  if (n16 <= 0) return;
  ProfScope ps(st, F_RESIDUAL, 6.0 * n16);
  launch_kernel(ps, k_residual_lo, ew_grid(n16), EW_THREADS, 0, st, theta, lo, n16);
}
void launch_nudge(hipStream_t st, float* theta, const float* vdir, const float* eps_ptr, const int64_t* status,
                  bf16_t* theta16, bf16_t* lo, int64_t n, int64_t n16) {
  if (n <= 0) return;
  ProfScope ps(st, F_NUDGE, 12.0 * n + (theta16 ? 2.0 * n16 : 0.0) + (lo ? 2.0 * n16 : 0.0));
  launch_kernel(ps, k_nudge, ew_grid(n), EW_THREADS, 0, st, theta, vdir, eps_ptr, status, theta16, lo, n, n16);
}
void launch_unnudge(hipStream_t st, float* theta, const float* vdir, const float* eps_ptr, const int64_t* status,
                    bf16_t* theta16, bf16_t* lo, int64_t n16) {
  if (n16 <= 0) return;
  const int grid = ew_grid(n16) < 2048 ? ew_grid(n16) : 2048;   // almost always an early exit: keep the launch small
  k_unnudge<<<grid, EW_THREADS, 0, st>>>(theta, vdir, eps_ptr, status, theta16, lo, n16);
}
void launch_fill_f32(hipStream_t st, float* p, float val, int64_t n) {
  if (n <= 0) return;
  ProfScope ps(st, F_OTHER, 4.0 * n);
  launch_kernel(ps, k_fill_f32, ew_grid(n), EW_THREADS, 0, st, p, val, n);
}
void launch_copy_f32(hipStream_t st, float* dst, const float* src, int64_t n) {
  if (n <= 0) return;
  k_copy_f32<<<ew_grid(n), EW_THREADS, 0, st>>>(dst, src, n);
}
void launch_to_bf16(hipStream_t st, bf16_t* dst, const float* src, int64_t n) {
  if (n <= 0) return;
  k_to_bf16<<<ew_grid(n * EW_VEC * EW_U), EW_THREADS, 0, st>>>(dst, src, n);
}
void launch_fill_i64x4(hipStream_t st, int64_t* p, int64_t a, int64_t b, int64_t c, int64_t d, int mask) {
  k_fill_i64<<<1, 64, 0, st>>>(p, a, b, c, d, mask);
}

}  // namespace sama
