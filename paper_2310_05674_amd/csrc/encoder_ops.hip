// Non-GEMM pieces of the post-LN encoder base learner (Sec. 4.1 uses BERT / RoBERTa-shaped models):
// embedding gather + LayerNorm, LayerNorm forward / backward, fused attention forward / backward on the matrix
// cores, classifier head, column sums, embedding gradients.  All reductions run in a fixed order.
#include "common.h"
#include "kernels.h"

namespace sama {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float LN_EPS = 1e-5f;

// =========================================================================================== LayerNorm forward
// One wave per row; the row lives in registers, NV 16-byte pieces per lane (d <= 256 NV).  Statistics in fp32 with a centred
// second pass.
template <int NV>
__global__ __launch_bounds__(256) void k_ln_fwd(LnFwdArgs a) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.M) return;
  const int nq = a.d >> 2;  // float4 chunks per row
  const float sc = a.pv.scale_row(row);
  float4 xr[NV];
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int q = lane + 64 * j;
    xr[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (q < nq) {
      if (a.x != nullptr) {
        xr[j] = reinterpret_cast<const float4*>(a.x + (int64_t)row * a.d)[q];
      } else {
        const int id = min(max(a.ids[a.ids_rows > 0 ? row % a.ids_rows : row], 0), a.V - 1);   // ids outside [0, V) are clamped
        const int64_t to = a.tok_off + (int64_t)id * a.d + 4 * q, po = a.pos_off + (int64_t)(row % a.S) * a.d + 4 * q;
        float4 t = *reinterpret_cast<const float4*>(a.pv.theta + to), p = *reinterpret_cast<const float4*>(a.pv.theta + po);
        if (sc != 0.f) {
          const float4 tv = *reinterpret_cast<const float4*>(a.pv.vdir + to), pvv = *reinterpret_cast<const float4*>(a.pv.vdir + po);
          t.x = fmaf(sc, tv.x, t.x); t.y = fmaf(sc, tv.y, t.y); t.z = fmaf(sc, tv.z, t.z); t.w = fmaf(sc, tv.w, t.w);
          p.x = fmaf(sc, pvv.x, p.x); p.y = fmaf(sc, pvv.y, p.y); p.z = fmaf(sc, pvv.z, p.z); p.w = fmaf(sc, pvv.w, p.w);
        }
        xr[j] = make_float4(t.x + p.x, t.y + p.y, t.z + p.z, t.w + p.w);
        if (a.x_out != nullptr) reinterpret_cast<float4*>(a.x_out + (int64_t)row * a.d)[q] = xr[j];
      }
      sum += (xr[j].x + xr[j].y) + (xr[j].z + xr[j].w);
    }
  }
  const float mu = wave_sum(sum) / (float)a.d;
  float sq = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    if (lane + 64 * j < nq) {
      const float e0 = xr[j].x - mu, e1 = xr[j].y - mu, e2 = xr[j].z - mu, e3 = xr[j].w - mu;
      sq += (e0 * e0 + e1 * e1) + (e2 * e2 + e3 * e3);
    }
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)a.d + LN_EPS);
  if (lane == 0) {
    if (a.mean != nullptr) a.mean[row] = mu;
    if (a.rstd != nullptr) a.rstd[row] = rstd;
  }
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int q = lane + 64 * j;
    if (q < nq) {
      float4 g = *reinterpret_cast<const float4*>(a.pv.theta + a.g_off + 4 * q), b = *reinterpret_cast<const float4*>(a.pv.theta + a.b_off + 4 * q);
      if (sc != 0.f) {
        const float4 gv = *reinterpret_cast<const float4*>(a.pv.vdir + a.g_off + 4 * q), bv = *reinterpret_cast<const float4*>(a.pv.vdir + a.b_off + 4 * q);
        g.x = fmaf(sc, gv.x, g.x); g.y = fmaf(sc, gv.y, g.y); g.z = fmaf(sc, gv.z, g.z); g.w = fmaf(sc, gv.w, g.w);
        b.x = fmaf(sc, bv.x, b.x); b.y = fmaf(sc, bv.y, b.y); b.z = fmaf(sc, bv.z, b.z); b.w = fmaf(sc, bv.w, b.w);
      }
      const float4 o = make_float4(fmaf((xr[j].x - mu) * rstd, g.x, b.x), fmaf((xr[j].y - mu) * rstd, g.y, b.y),
                                   fmaf((xr[j].z - mu) * rstd, g.z, b.z), fmaf((xr[j].w - mu) * rstd, g.w, b.w));
      uint2 pk;
      pk.x = pack_bf16x2(o.x, o.y);
      pk.y = pack_bf16x2(o.z, o.w);
      *reinterpret_cast<uint2*>(a.y + (int64_t)row * a.d + 4 * q) = pk;
      if (a.y32 != nullptr) reinterpret_cast<float4*>(a.y32 + (int64_t)row * a.d)[q] = o;
    }
  }
}

// =========================================================================================== LayerNorm backward
// dx = rstd (dy g - mean(dy g) - xh mean(dy g xh)); per-block partial sums of dgamma = dy xh, dbeta = dy and of
// dx itself (the bias gradient of the linear layer feeding this LayerNorm).  A block owns LN_BWD_ROWS rows,
// each wave walks its rows in order, lanes keep per-column accumulators, the four waves are added in order.
template <int NV>
__global__ __launch_bounds__(256) void k_ln_bwd(LnBwdArgs a) {
  __shared__ float s_acc[4][3][256 * NV];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nq = a.d >> 2;
  float4 dg[NV], db[NV], dc[NV], gam[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    dg[j] = db[j] = dc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    gam[j] = (lane + 64 * j < nq) ? reinterpret_cast<const float4*>(a.gamma)[lane + 64 * j] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const int r0 = blockIdx.x * LN_BWD_ROWS + wave * (LN_BWD_ROWS / 4);
  constexpr int RW = LN_BWD_ROWS / 4;   // rows per wave: all of their loads are issued before the first row is reduced
  float4 xin[RW][NV], dyin[RW][NV];
  float mus[RW], rstds[RW];
#pragma unroll
  for (int rr = 0; rr < RW; ++rr) {
    const int row = r0 + rr;
    mus[rr] = rstds[rr] = 0.f;
    if (row < a.M) { mus[rr] = a.mean[row]; rstds[rr] = a.rstd[row]; }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int q = lane + 64 * j;
      xin[rr][j] = dyin[rr][j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row < a.M && q < nq) {
        xin[rr][j] = reinterpret_cast<const float4*>(a.x + (int64_t)row * a.d)[q];
        dyin[rr][j] = reinterpret_cast<const float4*>(a.dy + (int64_t)row * a.d)[q];
      }
    }
  }
#pragma unroll
  for (int rr = 0; rr < RW; ++rr) {
    const int row = r0 + rr;
    if (row >= a.M) break;
    const float mu = mus[rr], rstd = rstds[rr];
    float4 xh[NV], dyg[NV];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int q = lane + 64 * j;
      xh[j] = dyg[j] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (q < nq) {
        const float4 x = xin[rr][j];
        const float4 dy = dyin[rr][j];
        xh[j] = make_float4((x.x - mu) * rstd, (x.y - mu) * rstd, (x.z - mu) * rstd, (x.w - mu) * rstd);
        dyg[j] = make_float4(dy.x * gam[j].x, dy.y * gam[j].y, dy.z * gam[j].z, dy.w * gam[j].w);
        dg[j].x = fmaf(dy.x, xh[j].x, dg[j].x); dg[j].y = fmaf(dy.y, xh[j].y, dg[j].y);
        dg[j].z = fmaf(dy.z, xh[j].z, dg[j].z); dg[j].w = fmaf(dy.w, xh[j].w, dg[j].w);
        db[j].x += dy.x; db[j].y += dy.y; db[j].z += dy.z; db[j].w += dy.w;
        s1 += (dyg[j].x + dyg[j].y) + (dyg[j].z + dyg[j].w);
        s2 += (dyg[j].x * xh[j].x + dyg[j].y * xh[j].y) + (dyg[j].z * xh[j].z + dyg[j].w * xh[j].w);
      }
    }
    const float m1 = wave_sum(s1) / (float)a.d, m2 = wave_sum(s2) / (float)a.d;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int q = lane + 64 * j;
      if (q < nq) {
        float4 dx;
        dx.x = rstd * (dyg[j].x - m1 - xh[j].x * m2); dx.y = rstd * (dyg[j].y - m1 - xh[j].y * m2);
        dx.z = rstd * (dyg[j].z - m1 - xh[j].z * m2); dx.w = rstd * (dyg[j].w - m1 - xh[j].w * m2);
        dc[j].x += dx.x; dc[j].y += dx.y; dc[j].z += dx.z; dc[j].w += dx.w;
        if (a.dx32 != nullptr) reinterpret_cast<float4*>(a.dx32 + (int64_t)row * a.d)[q] = dx;
        if (a.dx16 != nullptr) {
          uint2 pk;
          pk.x = pack_bf16x2(dx.x, dx.y);
          pk.y = pack_bf16x2(dx.z, dx.w);
          *reinterpret_cast<uint2*>(a.dx16 + (int64_t)row * a.d + 4 * q) = pk;
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int q = lane + 64 * j;
    if (q < nq) {
      reinterpret_cast<float4*>(s_acc[wave][0])[q] = dg[j];
      reinterpret_cast<float4*>(s_acc[wave][1])[q] = db[j];
      reinterpret_cast<float4*>(s_acc[wave][2])[q] = dc[j];
    }
  }
  __syncthreads();
  float* out = a.partial + (int64_t)blockIdx.x * 3 * a.d;
  for (int i = threadIdx.x; i < 3 * a.d; i += 256) {
    const int v = i / a.d, c = i - v * a.d;
    out[i] = ((s_acc[0][v][c] + s_acc[1][v][c]) + s_acc[2][v][c]) + s_acc[3][v][c];
  }
}

// out_v[c] = sum_r partial[r*stride + v*vstride + c] for up to three vectors v per job, several jobs per launch.
// A block owns 32 columns of one vector of one job; eight row groups walk the rows with stride 8 (independent
// loads), then are added in a fixed order.
struct ReduceRowsMulti { ReduceRowsJob j[REDUCE_MAX_JOBS]; int first_block[REDUCE_MAX_JOBS + 1]; int count; };
__global__ __launch_bounds__(256) void k_reduce_rows(ReduceRowsMulti m) {
  __shared__ float s_part[8][33];
  int job = 0;
#pragma unroll
  for (int k = 1; k < REDUCE_MAX_JOBS; ++k)
    if (k < m.count && (int)blockIdx.x >= m.first_block[k]) job = k;
  const ReduceRowsJob& a = m.j[job];
  const int local = blockIdx.x - m.first_block[job], nbx = (a.N + 31) / 32;
  const int cl = threadIdx.x & 31, rg = threadIdx.x >> 5, c = (local % nbx) * 32 + cl, v = local / nbx;
  float acc = 0.f;
  if (c < a.N) {
    const float* p = a.partial + (int64_t)v * a.vstride + c;
#pragma unroll 4
    for (int r = rg; r < a.nrows; r += 8) acc += p[(int64_t)r * a.stride];
  }
  s_part[rg][cl] = acc;
  __syncthreads();
  if (rg == 0 && c < a.N) {
    float t = s_part[0][cl];
#pragma unroll
    for (int g = 1; g < 8; ++g) t += s_part[g][cl];
    a.out[v][c] = t;
  }
}

// partial[rb][c] = sum of COLSUM_ROWS rows of column c of a bf16 matrix, up to two matrices per launch
struct ColsumMulti { ColsumJob j[2]; int first_block[3]; int count; };
__global__ __launch_bounds__(256) void k_colsum_partial_bf16(ColsumMulti m) {
  // a thread owns 8 adjacent columns (one 16-byte load per row); N is a multiple of 8
  const int job = (m.count > 1 && (int)blockIdx.x >= m.first_block[1]) ? 1 : 0;
  const ColsumJob& a = m.j[job];
  const int local = blockIdx.x - m.first_block[job], nbx = (a.N + 2047) / 2048;
  const int c = ((local % nbx) * 256 + threadIdx.x) * 8, rb = local / nbx;
  if (c >= a.N) return;
  const int r0 = rb * COLSUM_ROWS;
  float s[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) s[e] = 0.f;
  uint4 v[COLSUM_ROWS];
#pragma unroll
  for (int r = 0; r < COLSUM_ROWS; ++r)
    v[r] = (r0 + r < a.M) ? *reinterpret_cast<const uint4*>(a.X + (int64_t)(r0 + r) * a.N + c) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
  for (int r = 0; r < COLSUM_ROWS; ++r) {
    if (r0 + r >= a.M) break;
    const uint32_t w[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] += bf16_to_f32((bf16_t)(w[e >> 1] >> ((e & 1) * 16)));
  }
  float* out = a.partial + (int64_t)rb * a.N + c;
  *reinterpret_cast<float4*>(out) = make_float4(s[0], s[1], s[2], s[3]);
  *reinterpret_cast<float4*>(out + 4) = make_float4(s[4], s[5], s[6], s[7]);
}

// =========================================================================================== attention
// Sequence length S = 32 NT (NT = 2, 4 or 8 tiles of 32 positions), head width 64.
constexpr int AD = 64;  // head width

__device__ __forceinline__ bf16x8 ld_bf16x8(const bf16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ s16x4 pack4(float a, float b, float c, float d) {
  s16x4 r;
  r[0] = (short)f32_to_bf16(a); r[1] = (short)f32_to_bf16(b); r[2] = (short)f32_to_bf16(c); r[3] = (short)f32_to_bf16(d);
  return r;
}

// A [ROWS x 64] bf16 tile (row stride ld) staged in LDS as it lies in memory, S[row][e] with row stride SLD (192 bytes:
// the four rows one transposing read touches fall into four different 64-byte bank windows), and its transposed MFMA
// operand: for the 32x32x8 MFMA, lane l gets S[k0 + 4 (l / 32) + 0..3][e32 + l % 32] through ds_read_b64_tr_b16.
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
constexpr int SLD = AD + 32;
template <int THREADS, int ROWS>
__device__ __forceinline__ void stage_rows(const bf16_t* __restrict__ src, int64_t ld, bf16_t* __restrict__ S) {
#pragma unroll
  for (int c0 = 0; c0 < ROWS * 8; c0 += THREADS) {
    const int c = c0 + threadIdx.x, row = c >> 3, ec = c & 7;
    if (ROWS * 8 % THREADS == 0 || c < ROWS * 8)
      *reinterpret_cast<uint4*>(S + row * SLD + ec * 8) = *reinterpret_cast<const uint4*>(src + (int64_t)row * ld + ec * 8);
  }
}
__device__ __forceinline__ s16x4 ld_transposed(const bf16_t* __restrict__ S, int e32, int k0, int lane) {
  const int g = lane >> 4, j = lane & 15;
  const bf16_t* p = S + (k0 + 4 * (g >> 1) + (j >> 2)) * SLD + e32 + 16 * (g & 1) + 4 * (j & 3);
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
}

// X^T-style product tile: acc[32 x 32] (+)= sum_e R[rbase + l%32][e] * Cc[cbase + l%32][e], both operands read
// from global rows of 64 contiguous bf16 (row stride ld).  Result lane layout: column = cbase + l%32,
// rows rbase + 8(r/4) + 4(l/32) + r%4.
__device__ __forceinline__ f32x16 rows_dot_rows(const bf16_t* __restrict__ R, const bf16_t* __restrict__ Cc, int64_t ld,
                                                int rbase, int cbase, int lane) {
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const bf16_t* rp = R + (int64_t)(rbase + (lane & 31)) * ld + 8 * (lane >> 5);
  const bf16_t* cp = Cc + (int64_t)(cbase + (lane & 31)) * ld + 8 * (lane >> 5);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_bf16x8(rp + 16 * ks), ld_bf16x8(cp + 16 * ks), acc, 0, 0, 0);
  return acc;
}

// lens (or null): real tokens of sequence b % lens_period, clamped into [1, S]; keys at positions beyond get no weight.
__device__ __forceinline__ int seq_len_of(const int32_t* __restrict__ lens, int lens_period, int b, int S) {
  if (lens == nullptr) return S;
  const int n = lens[b % lens_period];
  return n < 1 ? 1 : (n > S ? S : n);
}

// Forward.  Four waves; wave w owns the query tiles w, w + 4, ... (32 queries each).  S^T[key][q] tiles leave each lane
// with one query column, so the softmax over keys is an in-lane reduction plus one cross-half shuffle, and the
// probability tile is already in the B-operand layout of the 32x32x8 MFMA for O^T[e][q] = sum_key V^T[e][key] P^T[key][q].
template <int NT>
__device__ __forceinline__ void attn_scores(const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, int64_t ld, int qt, int len,
                                            int lane, f32x16 (&s)[NT], float& inv, float* __restrict__ lse_row) {
#pragma unroll
  for (int kt = 0; kt < NT; ++kt) s[kt] = rows_dot_rows(K, Q, ld, 32 * kt, 32 * qt, lane);
  float mx = -3.0e38f;
#pragma unroll
  for (int kt = 0; kt < NT; ++kt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = 32 * kt + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      s[kt][r] = key < len ? s[kt][r] * 0.125f : -3.0e38f;   // exp(-3e38 - mx) = 0: key 0 is always real
      mx = fmaxf(mx, s[kt][r]);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  float sum = 0.f;
#pragma unroll
  for (int kt = 0; kt < NT; ++kt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[kt][r] = __expf(s[kt][r] - mx); sum += s[kt][r]; }
  sum += __shfl_xor(sum, 32, 64);
  inv = 1.f / sum;
  if (lane < 32 && lse_row != nullptr) lse_row[32 * qt + lane] = mx + __logf(sum);
}

template <int NT, bool PADDED>   // PADDED = false: no lengths given, the comparisons against len fold away
__global__ __launch_bounds__(256) void k_attn_fwd(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ out, float* __restrict__ lse,
                                                  int heads, int d, const int32_t* __restrict__ lens, int lens_period) {
  constexpr int S = 32 * NT;
  __shared__ __attribute__((aligned(16))) bf16_t Vs[S * SLD];
  const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t ld = 3 * (int64_t)d;
  const bf16_t* Q = qkv + (int64_t)b * S * ld + h * AD;
  const bf16_t* K = Q + d;
  const bf16_t* V = Q + 2 * d;
  const int len = PADDED ? seq_len_of(lens, lens_period, b, S) : S;
  float* lse_row = lse != nullptr ? lse + ((int64_t)b * heads + h) * S : nullptr;
  stage_rows<256, S>(V, ld, Vs);
  f32x16 s[NT];
  float inv = 0.f;
  int qt = wave;
  if (qt < NT) attn_scores<NT>(Q, K, ld, qt, len, lane, s, inv, lse_row);   // overlaps the staging of V
  __syncthreads();                                                          // reached once by every wave
  while (qt < NT) {
    f32x16 o[2];
#pragma unroll
    for (int et = 0; et < 2; ++et) {
#pragma unroll
      for (int r = 0; r < 16; ++r) o[et][r] = 0.f;
#pragma unroll
      for (int kt = 0; kt < NT; ++kt)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const s16x4 pb = pack4(s[kt][4 * c] * inv, s[kt][4 * c + 1] * inv, s[kt][4 * c + 2] * inv, s[kt][4 * c + 3] * inv);
          const s16x4 va = ld_transposed(Vs, 32 * et, 32 * kt + 8 * c, lane);
          o[et] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(va, pb, o[et], 0, 0, 0);
        }
    }
    bf16_t* orow = out + ((int64_t)b * S + 32 * qt + (lane & 31)) * d + h * AD;
#pragma unroll
    for (int et = 0; et < 2; ++et)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        uint2 pk;
        pk.x = pack_bf16x2(o[et][4 * c], o[et][4 * c + 1]);
        pk.y = pack_bf16x2(o[et][4 * c + 2], o[et][4 * c + 3]);
        *reinterpret_cast<uint2*>(orow + 32 * et + 8 * c + 4 * (lane >> 5)) = pk;
      }
    qt += 4;
    if (qt < NT) attn_scores<NT>(Q, K, ld, qt, len, lane, s, inv, lse_row);
  }
}

// Backward.  Probabilities are recomputed from q, k and the saved log-sum-exp.
// Phase A (a wave owns 32 queries at a time): dS^T[key][q] -> dQ^T[e][q] = sum_key K^T[e][key] dS^T[key][q].
// Phase B (a wave owns 32 keys at a time):    P[q][key], dS[q][key] -> dV^T[e][key] = sum_q dO^T[e][q] P[q][key],
//                                                                      dK^T[e][key] = sum_q Q^T[e][q] dS[q][key].
// dS = P (dP - D) / 8 with D[q] = sum_e dO[q][e] O[q][e].
// The two phases only read what is staged and are independent: waves 0-3 run phase A while waves 4-7 run phase B, each
// over the tiles w, w + 4, ... of its phase.
template <int NT, bool PADDED>
__global__ __launch_bounds__(512) void k_attn_bwd(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ out,
                                                  const bf16_t* __restrict__ dout, const float* __restrict__ lse,
                                                  bf16_t* __restrict__ dqkv, int heads, int d, const int32_t* __restrict__ lens,
                                                  int lens_period) {
  constexpr int S = 32 * NT, TILE_UNROLL = NT <= 4 ? NT : 1;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[S * SLD];
  __shared__ __attribute__((aligned(16))) bf16_t Qs[S * SLD];
  __shared__ __attribute__((aligned(16))) bf16_t dOs[S * SLD];
  __shared__ float s_D[S], s_lse[S];
  const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x & 63, wave = (threadIdx.x >> 6) & 3;
  const bool phase_a = threadIdx.x < 256;
  const int len = PADDED ? seq_len_of(lens, lens_period, b, S) : S;
  const int64_t ld = 3 * (int64_t)d;
  const bf16_t* Q = qkv + (int64_t)b * S * ld + h * AD;
  const bf16_t* K = Q + d;
  const bf16_t* V = Q + 2 * d;
  const bf16_t* O = out + (int64_t)b * S * d + h * AD;
  const bf16_t* dO = dout + (int64_t)b * S * d + h * AD;
  stage_rows<512, S>(K, ld, Ks);
  stage_rows<512, S>(Q, ld, Qs);
  stage_rows<512, S>(dO, d, dOs);
  if (phase_a) {
    // two threads per query; 2 S and 256 are multiples of the wave size, so a wave is in or out of a trip as a whole
    for (int t = threadIdx.x; t < 2 * S; t += 256) {
      const int q = t >> 1, half = t & 1;
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint4 o4 = *reinterpret_cast<const uint4*>(O + (int64_t)q * d + half * 32 + 8 * i);
        const uint4 d4 = *reinterpret_cast<const uint4*>(dO + (int64_t)q * d + half * 32 + 8 * i);
        const uint32_t ow[4] = {o4.x, o4.y, o4.z, o4.w}, dw[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          acc = fmaf(bf16_to_f32((bf16_t)(ow[e >> 1] >> ((e & 1) * 16))), bf16_to_f32((bf16_t)(dw[e >> 1] >> ((e & 1) * 16))), acc);
      }
      acc += __shfl_xor(acc, 1, 64);
      if (half == 0) { s_D[q] = acc; s_lse[q] = lse[((int64_t)b * heads + h) * S + q]; }
    }
  }
  __syncthreads();

  // ---- phase A: dQ
  if (phase_a) {
    for (int qt = wave; qt < NT; qt += 4) {
      const int q = 32 * qt + (lane & 31);
      const float lq = s_lse[q], Dq = s_D[q];
      f32x16 dq[2];
#pragma unroll
      for (int et = 0; et < 2; ++et)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[et][r] = 0.f;
#pragma unroll TILE_UNROLL   // the long sequences keep one tile's operands in flight: unrolled they spill
      for (int kt = 0; kt < NT; ++kt) {
        f32x16 st = rows_dot_rows(K, Q, ld, 32 * kt, 32 * qt, lane);     // S^T[key][q]
        const bf16_t* vp = V + (int64_t)(32 * kt + (lane & 31)) * ld + 8 * (lane >> 5);
        const bf16_t* dop = dO + (int64_t)(32 * qt + (lane & 31)) * d + 8 * (lane >> 5);
        f32x16 dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) dp[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_bf16x8(vp + 16 * ks), ld_bf16x8(dop + 16 * ks), dp, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = 32 * kt + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          st[r] = key < len ? __expf(st[r] * 0.125f - lq) * (dp[r] - Dq) * 0.125f : 0.f;   // dS^T; a padded key has P = 0
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const s16x4 dsb = pack4(st[4 * c], st[4 * c + 1], st[4 * c + 2], st[4 * c + 3]);
#pragma unroll
          for (int et = 0; et < 2; ++et) {
            const s16x4 ka = ld_transposed(Ks, 32 * et, 32 * kt + 8 * c, lane);
            dq[et] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(ka, dsb, dq[et], 0, 0, 0);
          }
        }
      }
      bf16_t* dqrow = dqkv + ((int64_t)b * S + q) * ld + h * AD;
#pragma unroll
      for (int et = 0; et < 2; ++et)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint2 pk;
          pk.x = pack_bf16x2(dq[et][4 * c], dq[et][4 * c + 1]);
          pk.y = pack_bf16x2(dq[et][4 * c + 2], dq[et][4 * c + 3]);
          *reinterpret_cast<uint2*>(dqrow + 32 * et + 8 * c + 4 * (lane >> 5)) = pk;
        }
    }
  }

  // ---- phase B: dK, dV
  if (!phase_a) {
    for (int kt = wave; kt < NT; kt += 4) {
      const bool real_key = (32 * kt + (lane & 31)) < len;              // this lane's key
      f32x16 dk[2], dv[2];
#pragma unroll
      for (int et = 0; et < 2; ++et)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dk[et][r] = 0.f; dv[et][r] = 0.f; }
#pragma unroll TILE_UNROLL
      for (int qt = 0; qt < NT; ++qt) {
        f32x16 st = rows_dot_rows(Q, K, ld, 32 * qt, 32 * kt, lane);     // S[q][key]
        const bf16_t* dop = dO + (int64_t)(32 * qt + (lane & 31)) * d + 8 * (lane >> 5);
        const bf16_t* vp = V + (int64_t)(32 * kt + (lane & 31)) * ld + 8 * (lane >> 5);
        f32x16 dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) dp[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_bf16x8(dop + 16 * ks), ld_bf16x8(vp + 16 * ks), dp, 0, 0, 0);
        f32x16 ds;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int q = 32 * qt + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const float p = real_key ? __expf(st[r] * 0.125f - s_lse[q]) : 0.f;
          st[r] = p;
          ds[r] = p * (dp[r] - s_D[q]) * 0.125f;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const s16x4 pb = pack4(st[4 * c], st[4 * c + 1], st[4 * c + 2], st[4 * c + 3]);
          const s16x4 dsb = pack4(ds[4 * c], ds[4 * c + 1], ds[4 * c + 2], ds[4 * c + 3]);
#pragma unroll
          for (int et = 0; et < 2; ++et) {
            dv[et] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(ld_transposed(dOs, 32 * et, 32 * qt + 8 * c, lane), pb, dv[et], 0, 0, 0);
            dk[et] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(ld_transposed(Qs, 32 * et, 32 * qt + 8 * c, lane), dsb, dk[et], 0, 0, 0);
          }
        }
      }
      bf16_t* krow = dqkv + ((int64_t)b * S + 32 * kt + (lane & 31)) * ld + d + h * AD;
      bf16_t* vrow = krow + d;
#pragma unroll
      for (int et = 0; et < 2; ++et)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          uint2 pk;
          pk.x = pack_bf16x2(dk[et][4 * c], dk[et][4 * c + 1]);
          pk.y = pack_bf16x2(dk[et][4 * c + 2], dk[et][4 * c + 3]);
          *reinterpret_cast<uint2*>(krow + 32 * et + 8 * c + 4 * (lane >> 5)) = pk;
          pk.x = pack_bf16x2(dv[et][4 * c], dv[et][4 * c + 1]);
          pk.y = pack_bf16x2(dv[et][4 * c + 2], dv[et][4 * c + 3]);
          *reinterpret_cast<uint2*>(vrow + 32 * et + 8 * c + 4 * (lane >> 5)) = pk;
        }
    }
  }
}

// =========================================================================================== classifier head
__global__ __launch_bounds__(256) void k_head_fwd(const float* __restrict__ x, int S, int d, int B, int C, ParamView pv,
                                                  int64_t wc_off, int64_t bc_off, float* __restrict__ logits) {
  const int lane = threadIdx.x & 63, idx = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (idx >= B * C) return;
  const int b = idx / C, c = idx - b * C;
  const float sc = pv.scale_row(b);
  const float* xr = x + (int64_t)b * S * d;
  float acc = 0.f;
  for (int k = lane; k < d; k += 64) acc = fmaf(xr[k], pv.at(wc_off + (int64_t)c * d + k, sc), acc);
  acc = wave_sum(acc);
  if (lane == 0) logits[idx] = acc + pv.at(bc_off + c, sc);
}

__global__ __launch_bounds__(256) void k_head_bwd_w(const float* __restrict__ x, int S, int d, int B, int C,
                                                    const float* __restrict__ dlogits, float* __restrict__ gWc, float* __restrict__ gbc) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < C * d) {
    const int c = i / d, k = i - c * d;
    float s = 0.f;
    for (int b = 0; b < B; ++b) s = fmaf(dlogits[b * C + c], x[(int64_t)b * S * d + k], s);
    gWc[i] = s;
  }
  if (i < C) {
    float s = 0.f;
    for (int b = 0; b < B; ++b) s += dlogits[b * C + i];
    gbc[i] = s;
  }
}
__global__ __launch_bounds__(256) void k_head_bwd_x(int S, int d, int B, int C, const float* __restrict__ Wc,
                                                    const float* __restrict__ dlogits, float* __restrict__ dx) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= B * d) return;
  const int b = i / d, k = i - b * d;
  float s = 0.f;
  for (int c = 0; c < C; ++c) s = fmaf(dlogits[b * C + c], Wc[(int64_t)c * d + k], s);
  dx[(int64_t)b * S * d + k] = s;
}

// =========================================================================================== embedding gradients
__global__ __launch_bounds__(256) void k_pos_grad(const float* __restrict__ demb, int B, int S, int d, float* __restrict__ g_pos) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= S * d) return;
  float s = 0.f;
  for (int b = 0; b < B; ++b) s += demb[(int64_t)b * S * d + i];
  g_pos[i] = s;
}

// One block per position m.  The block lists, in ascending order, every position holding the same token id;
// only the block of the first occurrence goes on, and writes the ordered sum of those rows.
__global__ __launch_bounds__(256) void k_tok_grad(const float* __restrict__ demb, const int32_t* __restrict__ ids, int M, int d,
                                                  int V, float* __restrict__ g_tok) {
  __shared__ int s_list[MAX_TOKENS];
  __shared__ int s_cnt, s_wave[4];
  const int m = blockIdx.x, id = min(max(ids[m], 0), V - 1), lane = threadIdx.x & 63, wave = threadIdx.x >> 6;   // clamped as in the forward pass
  if (threadIdx.x == 0) s_cnt = 0;
  __syncthreads();
  for (int base = 0; base < M; base += 256) {
    const int mm = base + threadIdx.x;
    const bool hit = (mm < M) && (min(max(ids[mm], 0), V - 1) == id);
    const unsigned long long bal = __ballot(hit);
    if (lane == 0) s_wave[wave] = __popcll(bal);
    __syncthreads();
    int off = s_cnt;
    for (int w = 0; w < wave; ++w) off += s_wave[w];
    if (hit) {
      const int pos = off + __popcll(bal & ((1ull << lane) - 1ull));
      if (pos < MAX_TOKENS) s_list[pos] = mm;
    }
    __syncthreads();
    if (threadIdx.x == 0) s_cnt += s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
    __syncthreads();
    if (s_cnt > 0 && s_list[0] != m) return;   // an earlier position holds this id (the list is ascending)
  }
  const int cnt = s_cnt < MAX_TOKENS ? s_cnt : MAX_TOKENS;
  // a frequent id (position 0 of every sequence, the head of the Zipf law) has hundreds of rows: fetch them sixteen at
  // a time so that their latencies overlap, add them in list order
  for (int c = threadIdx.x; c < d; c += 256) {
    float s = 0.f;
    int i = 0;
    for (; i + 16 <= cnt; i += 16) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = demb[(int64_t)s_list[i + u] * d + c];
#pragma unroll
      for (int u = 0; u < 16; ++u) s += v[u];
    }
    for (; i < cnt; ++i) s += demb[(int64_t)s_list[i] * d + c];
    g_tok[(int64_t)id * d + c] = s;
  }
}
}  // namespace

void launch_ln_fwd(hipStream_t st, const LnFwdArgs& a) {
  ProfScope ps(st, F_LN_FWD, 6.0 * a.M * a.d);
  if (a.d <= 1024) launch_kernel(ps, k_ln_fwd<4>, (a.M + 3) / 4, 256, 0, st, a);
  else launch_kernel(ps, k_ln_fwd<8>, (a.M + 3) / 4, 256, 0, st, a);
}
void launch_ln_bwd(hipStream_t st, const LnBwdArgs& a) {
  ProfScope ps(st, F_LN_BWD, 14.0 * a.M * a.d);
  if (a.d <= 1024) launch_kernel(ps, k_ln_bwd<4>, (a.M + LN_BWD_ROWS - 1) / LN_BWD_ROWS, 256, 0, st, a);
  else launch_kernel(ps, k_ln_bwd<8>, (a.M + LN_BWD_ROWS - 1) / LN_BWD_ROWS, 256, 0, st, a);
}
void launch_reduce_rows_multi(hipStream_t st, const ReduceRowsJob* jobs, int count) {
  ReduceRowsMulti m{};
  m.count = count;
  int nb = 0;
  double bytes = 0.0;
  for (int k = 0; k < count; ++k) {
    m.j[k] = jobs[k];
    m.first_block[k] = nb;
    const int nv = jobs[k].out[2] ? 3 : (jobs[k].out[1] ? 2 : 1);
    nb += ((jobs[k].N + 31) / 32) * nv;
    bytes += 4.0 * jobs[k].nrows * jobs[k].N * nv;
  }
  for (int k = count; k <= REDUCE_MAX_JOBS; ++k) m.first_block[k] = nb;
  ProfScope ps(st, F_OTHER, bytes);
  launch_kernel(ps, k_reduce_rows, nb, 256, 0, st, m);
}
void launch_reduce_rows(hipStream_t st, const float* partial, int nrows, int64_t stride, int64_t vstride, int N, float* out0,
                        float* out1, float* out2) {
  const ReduceRowsJob j{partial, nrows, stride, vstride, N, {out0, out1, out2}};
  launch_reduce_rows_multi(st, &j, 1);
}
void launch_colsum_partial_multi(hipStream_t st, const ColsumJob* jobs, int count) {
  ColsumMulti m{};
  m.count = count;
  int nb = 0;
  double bytes = 0.0;
  for (int k = 0; k < count; ++k) {
    m.j[k] = jobs[k];
    m.first_block[k] = nb;
    nb += ((jobs[k].N + 2047) / 2048) * ((jobs[k].M + COLSUM_ROWS - 1) / COLSUM_ROWS);
    bytes += 2.0 * jobs[k].M * jobs[k].N;
  }
  for (int k = count; k < 3; ++k) m.first_block[k] = nb;
  ProfScope ps(st, F_OTHER, bytes);
  launch_kernel(ps, k_colsum_partial_bf16, nb, 256, 0, st, m);
}
void launch_colsum_bf16(hipStream_t st, const bf16_t* X, int M, int N, float* partial, float* out) {
  const int nrb = (M + COLSUM_ROWS - 1) / COLSUM_ROWS;
  const ColsumJob j{X, M, N, partial};
  launch_colsum_partial_multi(st, &j, 1);
  launch_reduce_rows(st, partial, nrb, N, 0, N, out, nullptr, nullptr);
}
// (S = 32 would fit the kernels, but the weight-gradient GEMMs contract over batch * S token rows in slabs of 64)
bool attention_supports(int S) { return S == 64 || S == 128 || S == 256; }
void launch_attention_fwd(hipStream_t st, const bf16_t* qkv, bf16_t* out, float* lse, int B, int S, int heads, int d,
                          const int32_t* lens, int lens_period) {
  ProfScope ps(st, F_ATTN_FWD, 4.0 * B * heads * (double)S * S * 64.0);
  const dim3 grid(heads, B);
  const int lp = lens_period > 0 ? lens_period : 1;
  switch (S) {
    case 64:
      if (lens) launch_kernel(ps, k_attn_fwd<2, true>, grid, 256, 0, st, qkv, out, lse, heads, d, lens, lp);
      else launch_kernel(ps, k_attn_fwd<2, false>, grid, 256, 0, st, qkv, out, lse, heads, d, lens, lp);
      break;
    case 128:
      if (lens) launch_kernel(ps, k_attn_fwd<4, true>, grid, 256, 0, st, qkv, out, lse, heads, d, lens, lp);
      else launch_kernel(ps, k_attn_fwd<4, false>, grid, 256, 0, st, qkv, out, lse, heads, d, lens, lp);
      break;
    case 256:
      if (lens) launch_kernel(ps, k_attn_fwd<8, true>, grid, 256, 0, st, qkv, out, lse, heads, d, lens, lp);
      else launch_kernel(ps, k_attn_fwd<8, false>, grid, 256, 0, st, qkv, out, lse, heads, d, lens, lp);
      break;
    default: break;   // make_encoder admits no other length
  }
}
void launch_attention_bwd(hipStream_t st, const bf16_t* qkv, const bf16_t* out, const bf16_t* dout, const float* lse,
                          bf16_t* dqkv, int B, int S, int heads, int d, const int32_t* lens, int lens_period) {
  ProfScope ps(st, F_ATTN_BWD, 10.0 * B * heads * (double)S * S * 64.0);
  const dim3 grid(heads, B);
  const int lp = lens_period > 0 ? lens_period : 1;
  switch (S) {
    case 64:
      if (lens) launch_kernel(ps, k_attn_bwd<2, true>, grid, 512, 0, st, qkv, out, dout, lse, dqkv, heads, d, lens, lp);
      else launch_kernel(ps, k_attn_bwd<2, false>, grid, 512, 0, st, qkv, out, dout, lse, dqkv, heads, d, lens, lp);
      break;
    case 128:
      if (lens) launch_kernel(ps, k_attn_bwd<4, true>, grid, 512, 0, st, qkv, out, dout, lse, dqkv, heads, d, lens, lp);
      else launch_kernel(ps, k_attn_bwd<4, false>, grid, 512, 0, st, qkv, out, dout, lse, dqkv, heads, d, lens, lp);
      break;
    case 256:
      if (lens) launch_kernel(ps, k_attn_bwd<8, true>, grid, 512, 0, st, qkv, out, dout, lse, dqkv, heads, d, lens, lp);
      else launch_kernel(ps, k_attn_bwd<8, false>, grid, 512, 0, st, qkv, out, dout, lse, dqkv, heads, d, lens, lp);
      break;
    default: break;
  }
}
void launch_head_fwd(hipStream_t st, const float* x, int S, int d, int B, int C, ParamView pv, int64_t wc_off, int64_t bc_off,
                     float* logits) {
  ProfScope ps(st, F_OTHER, 0.0);
  launch_kernel(ps, k_head_fwd, (B * C + 3) / 4, 256, 0, st, x, S, d, B, C, pv, wc_off, bc_off, logits);
}
void launch_head_bwd(hipStream_t st, const float* x, int S, int d, int B, int C, const float* theta, int64_t wc_off,
                     int64_t bc_off, const float* dlogits, float* grad, float* dx) {
  ProfScope ps(st, F_OTHER, 0.0);
  launch_kernel(ps, k_head_bwd_w, (C * d + 255) / 256, 256, 0, st, x, S, d, B, C, dlogits, grad + wc_off, grad + bc_off);
  launch_kernel(ps, k_head_bwd_x, (B * d + 255) / 256, 256, 0, st, S, d, B, C, theta + wc_off, dlogits, dx);
}
void launch_embedding_bwd(hipStream_t st, const float* demb, const int32_t* ids, int B, int S, int d, int V, float* g_tok, float* g_pos) {
  ProfScope ps(st, F_OTHER, 4.0 * B * S * d);
  launch_kernel(ps, k_pos_grad, (S * d + 255) / 256, 256, 0, st, demb, B, S, d, g_pos);
  launch_kernel(ps, k_tok_grad, B * S, 256, 0, st, demb, ids, B * S, d, V, g_tok);
}

}  // namespace sama
