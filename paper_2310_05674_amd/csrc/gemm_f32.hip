// fp32 contraction for the fp32 base learners (logistic regression, small MLPs): forward, dgrad and wgrad of a
// linear layer are the same kernel with different strides.  The matrix cores are used in their fp32 form
// (v_mfma_f32_16x16x4_f32), so results carry plain fp32 rounding.  Shapes are arbitrary: every global access is
// bounds-checked.
//
// These problems are tiny (a batch of 128 rows, a few hundred columns) and latency-bound, so the kernel is built for
// short dependency chains rather than for reuse: a workgroup owns a 32 x 32 output tile, its four waves split the
// contraction between them in interleaved chunks of 16 and fetch their operands from global memory straight into the
// MFMA operand layout (lane (r, q) holds row r and the four contraction indices 4q .. 4q+3 of a chunk: one 16-byte
// load where the contraction index is the contiguous one) -- no LDS staging, no barrier inside the loop, the next
// chunk's loads in flight behind the current chunk's MFMAs.  The four partial tiles are added in wave order through
// LDS, so the result does not depend on timing.
//
// The +-eps v passes of Eq. 5 read the weight operand as B + s * Bv (s = +-eps from device memory), so no
// perturbed copy of theta is ever written.
#include "common.h"
#include "kernels.h"

namespace sama {
namespace {

typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int FT = 32;        // output tile edge
constexpr int FCH = 16;       // contraction indices per chunk (one wave, four MFMAs deep)

// four consecutive contraction indices k .. k+3 of row `row` of an operand with element (row, k) at p[row * s_row + k * s_k];
// out-of-range rows / indices read as 0
__device__ __forceinline__ float4v load_k4(const float* __restrict__ p, int64_t s_row, int64_t s_k, int row, int nrows, int k, int K,
                                            bool vec_ok) {
  float4v v = {0.f, 0.f, 0.f, 0.f};
  if (row >= nrows) return v;
  const float* q = p + (int64_t)row * s_row + (int64_t)k * s_k;
  if (vec_ok && k + 3 < K) return *reinterpret_cast<const float4v*>(q);
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if (k + c < K) v[c] = q[(int64_t)c * s_k];
  return v;
}

__global__ __launch_bounds__(256) void k_gemm_f32(GemmF32Args a) {
  __shared__ float red[3][FT][FT + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int i0 = blockIdx.y * FT, j0 = blockIdx.x * FT;
  const float bscale = (a.Bv != nullptr && a.beps != nullptr) ? a.bsign * (*a.beps) : 0.f;
  // 16-byte loads along the contraction index need it contiguous and every row start aligned
  const bool a_vec = a.sa_k == 1 && (a.sa_i & 3) == 0 && ((uintptr_t)a.A & 15) == 0;
  const bool b_vec = a.sb_k == 1 && (a.sb_j & 3) == 0 && ((uintptr_t)a.B & 15) == 0 && (a.Bv == nullptr || ((uintptr_t)a.Bv & 15) == 0);

  float4v acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) acc[x][y] = (float4v){0.f, 0.f, 0.f, 0.f};

  auto fetch = [&](int k0, float4v (&av)[2], float4v (&bv)[2]) {
    const int k = k0 + 4 * q;
#pragma unroll
    for (int x = 0; x < 2; ++x) av[x] = load_k4(a.A, a.sa_i, a.sa_k, i0 + 16 * x + r, a.M, k, a.K, a_vec);
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      bv[y] = load_k4(a.B, a.sb_j, a.sb_k, j0 + 16 * y + r, a.N, k, a.K, b_vec);
      if (bscale != 0.f) {
        const float4v pv = load_k4(a.Bv, a.sb_j, a.sb_k, j0 + 16 * y + r, a.N, k, a.K, b_vec);
#pragma unroll
        for (int c = 0; c < 4; ++c) bv[y][c] = fmaf(bscale, pv[c], bv[y][c]);
      }
    }
  };
  float4v av[2][2], bv[2][2];   // [buffer][tile]
  int k0 = wave * FCH, buf = 0;
  if (k0 < a.K) fetch(k0, av[0], bv[0]);
  for (; k0 < a.K; k0 += 4 * FCH, buf ^= 1) {
    if (k0 + 4 * FCH < a.K) fetch(k0 + 4 * FCH, av[buf ^ 1], bv[buf ^ 1]);
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[buf][x][c], bv[buf][y][c], acc[x][y], 0, 0, 0);
  }
  // partial tiles of waves 1..3 -> LDS; wave 0 adds them in wave order and finishes the tile
  if (wave > 0) {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave - 1][16 * x + 4 * q + e][16 * y + r] = acc[x][y][e];
  }
  __syncthreads();
  if (wave > 0) return;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int gj = j0 + 16 * y + r;
      if (gj >= a.N) continue;
      float bias = 0.f;
      if (a.bias != nullptr) {
        bias = a.bias[gj];
        if (bscale != 0.f && a.bias_v != nullptr) bias = fmaf(bscale, a.bias_v[gj], bias);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int li = 16 * x + 4 * q + e, gi = i0 + li;
        if (gi >= a.M) continue;
        float c = ((acc[x][y][e] + red[0][li][16 * y + r]) + red[1][li][16 * y + r]) + red[2][li][16 * y + r];
        c += bias;
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
  dim3 grid((a.N + FT - 1) / FT, (a.M + FT - 1) / FT);
  ProfScope ps(st, F_GEMM_F32, 2.0 * a.M * a.N * a.K);
  launch_kernel(ps, k_gemm_f32, grid, 256, 0, st, a);
}
void launch_colsum_f32(hipStream_t st, const float* X, int64_t ld, int M, int N, float* out) {
  if (N <= 0) return;
  k_colsum_f32<<<(N + 255) / 256, 256, 0, st>>>(X, ld, M, N, out);
}

}  // namespace sama
