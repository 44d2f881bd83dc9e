// bf16 x bf16 -> fp32 contraction on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16) for the encoder's
// linear layers: forward (X W^T), dgrad (dY W) and wgrad (dY^T X) are the same kernel with different operand
// storage flags.  128x128 block tile, 64-deep k slab staged through LDS, four waves in a 2x2 arrangement each
// owning a 64x64 accumulator (2x2 MFMA tiles), global loads of the next slab issued before the current slab's
// MFMAs.  Operands whose contraction index is not the contiguous one are transposed on their way into LDS.
//
// For the theta +- eps v passes of Eq. 5 the weight operand is hi + lo (two bf16 halves): the k loop simply runs
// twice, the second time over `B2`, into the same accumulators.
//
// Fused epilogues: + bias (fp32, optionally perturbed), + residual (bf16 or fp32), GELU forward (writes both
// the pre-activation and the activation), GELU backward (multiplies by gelu'(pre)), fp32 and/or bf16 stores.
#include "common.h"
#include "kernels.h"

namespace sama {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 64, LDS_LD = BK + 8;  // row stride 144 B: conflict-free 16-byte reads

__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float dgelu_f(float x) {
  return 0.5f * (1.f + erff(x * 0.70710678118654752f)) + x * 0.39894228040143268f * __expf(-0.5f * x * x);
}

// Loads one 128 x 64 operand slab into registers (4 x 16 B per thread).  TRANS = false: storage [rows][k]
// (k contiguous); TRANS = true: storage [k][rows] (rows contiguous).  Rows past `nrows` read as zero.
template <bool TRANS>
__device__ __forceinline__ void load_slab(const bf16_t* __restrict__ P, int64_t ld, int row0, int nrows, int k0, uint4 (&r)[4]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = t + 256 * i;
    if (!TRANS) {
      const int row = c >> 3, kc = c & 7;
      r[i] = (row0 + row < nrows) ? *reinterpret_cast<const uint4*>(P + (int64_t)(row0 + row) * ld + k0 + kc * 8) : make_uint4(0, 0, 0, 0);
    } else {
      const int k = c >> 4, rc = c & 15;
      r[i] = (row0 + rc * 8 < nrows) ? *reinterpret_cast<const uint4*>(P + (int64_t)(k0 + k) * ld + row0 + rc * 8) : make_uint4(0, 0, 0, 0);
    }
  }
}
template <bool TRANS>
__device__ __forceinline__ void store_slab(bf16_t* __restrict__ S, const uint4 (&r)[4]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = t + 256 * i;
    if (!TRANS) {
      const int row = c >> 3, kc = c & 7;
      *reinterpret_cast<uint4*>(S + row * LDS_LD + kc * 8) = r[i];
    } else {
      const int k = c >> 4, rc = c & 15;
      const uint32_t w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
#pragma unroll
      for (int e = 0; e < 8; ++e) S[(rc * 8 + e) * LDS_LD + k] = (bf16_t)(w[e >> 1] >> ((e & 1) * 16));
    }
  }
}

template <bool A_TRANS, bool B_TRANS>
__global__ __launch_bounds__(256) void k_gemm_bf16(GemmBf16Args a) {
  __shared__ __attribute__((aligned(16))) bf16_t As[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * LDS_LD];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wr = (wave >> 1) * 64, wc = (wave & 1) * 64;
  const int i0 = blockIdx.y * BM, j0 = blockIdx.x * BN;

  f32x16 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  const int nk = a.K / BK;
  const int iters = (a.B2 != nullptr) ? 2 * nk : nk;
  uint4 ra[4], rb[4];
  load_slab<A_TRANS>(a.A, a.lda, i0, a.M, 0, ra);
  load_slab<!B_TRANS>(a.B, a.ldb, j0, a.N, 0, rb);   // B_TRANS = true means storage [N][K] = rows-major for this loader
  for (int it = 0; it < iters; ++it) {
    __syncthreads();
    store_slab<A_TRANS>(As, ra);
    store_slab<!B_TRANS>(Bs, rb);
    __syncthreads();
    if (it + 1 < iters) {
      const int nx = it + 1;
      const int kk = (nx >= nk ? nx - nk : nx) * BK;
      load_slab<A_TRANS>(a.A, a.lda, i0, a.M, kk, ra);
      load_slab<!B_TRANS>(nx >= nk ? a.B2 : a.B, a.ldb, j0, a.N, kk, rb);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 av[2], bv[2];
      const int kof = ks * 16 + 8 * (lane >> 5);
#pragma unroll
      for (int x = 0; x < 2; ++x) av[x] = *reinterpret_cast<const bf16x8*>(As + (wr + x * 32 + (lane & 31)) * LDS_LD + kof);
#pragma unroll
      for (int y = 0; y < 2; ++y) bv[y] = *reinterpret_cast<const bf16x8*>(Bs + (wc + y * 32 + (lane & 31)) * LDS_LD + kof);
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[x], bv[y], acc[x][y], 0, 0, 0);
    }
  }

  const float bscale = (a.bias_v != nullptr && a.beps != nullptr && a.bsign != 0.f) ? a.bsign * (*a.beps) : 0.f;
#pragma unroll
  for (int y = 0; y < 2; ++y) {
    const int gj = j0 + wc + y * 32 + (lane & 31);
    if (gj >= a.N) continue;
    float bias = 0.f;
    if (a.bias != nullptr) {
      bias = a.bias[gj];
      if (bscale != 0.f) bias = fmaf(bscale, a.bias_v[gj], bias);
    }
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int gi = i0 + wr + x * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (gi >= a.M) continue;
        const int64_t o = (int64_t)gi * a.ldc + gj;
        float c = acc[x][y][r] + bias;
        if (a.res16 != nullptr) c += bf16_to_f32(a.res16[o]);
        if (a.res32 != nullptr) c += a.res32[o];
        if (a.act == GEMM_ACT_GELU_FWD) {
          a.C16_pre[o] = f32_to_bf16(c);
          c = gelu_f(bf16_to_f32(f32_to_bf16(c)));   // the backward pass sees the rounded pre-activation
        } else if (a.act == GEMM_ACT_GELU_BWD) {
          c *= dgelu_f(bf16_to_f32(a.aux16[o]));
        }
        if (a.C32 != nullptr) a.C32[o] = c;
        if (a.C16 != nullptr) a.C16[o] = f32_to_bf16(c);
      }
  }
}
}  // namespace

const char* check_gemm_bf16(const GemmBf16Args& a) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return "empty GEMM";
  if (a.K % BK != 0) return "K must be a multiple of 64";
  if (a.M % 8 != 0 || a.N % 8 != 0) return "M and N must be multiples of 8";
  if (a.lda % 8 != 0 || a.ldb % 8 != 0) return "leading dimensions must be multiples of 8";
  if (((uintptr_t)a.A | (uintptr_t)a.B | (uintptr_t)a.B2) & 15) return "operands must be 16-byte aligned";
  if (a.lda < (a.a_trans ? a.M : a.K) || a.ldb < (a.b_trans ? a.K : a.N) || a.ldc < a.N) return "leading dimension too small";
  return nullptr;
}

void launch_gemm_bf16(hipStream_t st, const GemmBf16Args& a) {
  dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM);
  const double flops = 2.0 * a.M * a.N * a.K * (a.B2 ? 2.0 : 1.0);   // hi + lo contracts over 2K
  ProfScope ps(st, a.a_trans ? F_GEMM_TN : (a.b_trans ? F_GEMM_NT : F_GEMM_NN), flops);
  if (!a.a_trans && a.b_trans) k_gemm_bf16<false, true><<<grid, 256, 0, st>>>(a);
  else if (!a.a_trans && !a.b_trans) k_gemm_bf16<false, false><<<grid, 256, 0, st>>>(a);
  else if (a.a_trans && !a.b_trans) k_gemm_bf16<true, false><<<grid, 256, 0, st>>>(a);
  else k_gemm_bf16<true, true><<<grid, 256, 0, st>>>(a);
}

}  // namespace sama
