// fp32 contraction for the fp32 base learners (logistic regression, small MLPs): forward, dgrad and wgrad of a
// linear layer are the same kernel with different strides.  The matrix cores are used in their fp32 form
// (v_mfma_f32_16x16x4_f32), so results carry plain fp32 rounding.  Shapes are arbitrary: every global access is
// bounds-checked, tiles are staged through LDS as [k][row].
//
// The +-eps v passes of Eq. 5 read the weight operand as B + s * Bv (s = +-eps from device memory), so no
// perturbed copy of theta is ever written.
#include "common.h"
#include "kernels.h"

namespace sama {
namespace {

typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int TM = 64, TN = 64, TK = 16, PAD = 4;

__global__ __launch_bounds__(256) void k_gemm_f32(GemmF32Args a) {
  __shared__ float As[TK][TM + PAD];
  __shared__ float Bs[TK][TN + PAD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i0 = blockIdx.y * TM, j0 = blockIdx.x * TN;
  const int wr = (wave >> 1) * 32, wc = (wave & 1) * 32;
  const float bscale = (a.Bv != nullptr && a.beps != nullptr) ? a.bsign * (*a.beps) : 0.f;

  float4v acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) acc[x][y] = (float4v){0.f, 0.f, 0.f, 0.f};

  const bool a_kfast = (a.sa_k == 1);
  const bool b_kfast = (a.sb_k == 1);
  for (int k0 = 0; k0 < a.K; k0 += TK) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int i, k;
      if (a_kfast) { k = tid & 15; i = (tid >> 4) + 16 * r; } else { i = tid & 63; k = (tid >> 6) + 4 * r; }
      const int gi = i0 + i, gk = k0 + k;
      As[k][i] = (gi < a.M && gk < a.K) ? a.A[(int64_t)gi * a.sa_i + (int64_t)gk * a.sa_k] : 0.f;
      int j, kb;
      if (b_kfast) { kb = tid & 15; j = (tid >> 4) + 16 * r; } else { j = tid & 63; kb = (tid >> 6) + 4 * r; }
      const int gj = j0 + j, gkb = k0 + kb;
      float bv = 0.f;
      if (gj < a.N && gkb < a.K) {
        const int64_t off = (int64_t)gkb * a.sb_k + (int64_t)gj * a.sb_j;
        bv = a.B[off];
        if (bscale != 0.f) bv = fmaf(bscale, a.Bv[off], bv);
      }
      Bs[kb][j] = bv;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; kk += 4) {
      const int kl = kk + (lane >> 4);
      float av[2], bv[2];
      av[0] = As[kl][wr + (lane & 15)];
      av[1] = As[kl][wr + 16 + (lane & 15)];
      bv[0] = Bs[kl][wc + (lane & 15)];
      bv[1] = Bs[kl][wc + 16 + (lane & 15)];
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[x], bv[y], acc[x][y], 0, 0, 0);
    }
    __syncthreads();
  }
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int gj = j0 + wc + 16 * y + (lane & 15);
      if (gj >= a.N) continue;
      float bias = 0.f;
      if (a.bias != nullptr) {
        bias = a.bias[gj];
        if (bscale != 0.f && a.bias_v != nullptr) bias = fmaf(bscale, a.bias_v[gj], bias);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int gi = i0 + wr + 16 * x + 4 * (lane >> 4) + r;
        if (gi >= a.M) continue;
        float c = acc[x][y][r] + bias;
        if (a.relu) c = fmaxf(c, 0.f);
        if (a.gate != nullptr) c = a.gate[(int64_t)gi * a.ldc + gj] > 0.f ? c : 0.f;
        a.C[(int64_t)gi * a.ldc + gj] = c;
      }
    }
}

// column sums, one thread per column, rows in order (deterministic); M is a batch size here
__global__ __launch_bounds__(256) void k_colsum_f32(const float* __restrict__ X, int64_t ld, int M, int N,
                                                    float* __restrict__ out) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= N) return;
  float s = 0.f;
  for (int i = 0; i < M; ++i) s += X[(int64_t)i * ld + j];
  out[j] = s;
}
}  // namespace

void launch_gemm_f32(hipStream_t st, const GemmF32Args& a) {
  if (a.M <= 0 || a.N <= 0) return;
  dim3 grid((a.N + TN - 1) / TN, (a.M + TM - 1) / TM);
  ProfScope ps(st, F_GEMM_F32, 2.0 * a.M * a.N * a.K);
  launch_kernel(ps, k_gemm_f32, grid, 256, 0, st, a);
}
void launch_colsum_f32(hipStream_t st, const float* X, int64_t ld, int M, int N, float* out) {
  if (N <= 0) return;
  k_colsum_f32<<<(N + 255) / 256, 256, 0, st>>>(X, ld, M, N, out);
}

}  // namespace sama
