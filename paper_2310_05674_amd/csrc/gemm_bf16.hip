// bf16 x bf16 -> fp32 contraction on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16) for the encoder's
// linear layers: forward (X W^T), dgrad (dY W) and wgrad (dY^T X) are one kernel template over the storage of its
// two operands.
//
//   block tile 128 x 128, k slab 64, four waves (2 x 2), each owning a 64 x 64 accumulator (2 x 2 MFMA tiles)
//   LDS double buffer (one barrier per slab); the global loads of slab i+1 are in flight during slab i's MFMAs
//   an operand whose contraction index is contiguous in memory is staged as [row][k] and fetched with 16-byte reads;
//   an operand whose contraction index is the strided one (dgrad's W, both operands of wgrad) is staged as it lies
//   in memory, [k][row], and fetched with the transposing LDS read (ds_read_b64_tr_b16), so nothing is ever
//   transposed through registers or scattered into LDS
//   the accumulators leave through LDS so that every global access of the epilogue is a full row segment
//
// For the theta +- eps v passes of Eq. 5 and the direct-gradient pass the weight operand is hi + lo (two bf16
// halves): the k loop simply runs twice, the second time over `B2`, into the same accumulators.
//
// Fused epilogues: + bias (fp32, optionally perturbed), + residual (bf16 or fp32), GELU forward (writes both the
// pre-activation and the activation), GELU backward (multiplies by gelu'(pre)), fp32 and/or bf16 stores.
#include "common.h"
#include "kernels.h"

namespace sama {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDK = BK + 8;        // [row][k] staging: 144-byte rows, conflict-free 16-byte reads
constexpr int LDR = 128 + 32;      // [k][row] staging: 320-byte rows, conflict-free transposing reads
constexpr int TILE_ELEMS = BK * LDR;                 // 10240 bf16 = 20480 B (>= 128 * LDK = 9216)
constexpr int STAGE_ELEMS = 2 * TILE_ELEMS;          // A tile + B tile
constexpr int LDS_BYTES = 2 * STAGE_ELEMS * 2;       // two stages: 81920 B
constexpr int EPI_LD = 64 + 4;                       // fp32 row stride of a wave's 64 x 64 epilogue tile

// erf by Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7), sharing exp(-x^2) with the Gaussian density
__device__ __forceinline__ void erf_and_gauss(float z, float& erfz, float& ez2) {
  const float az = fabsf(z);
  const float t = __frcp_rn(fmaf(0.3275911f, az, 1.f));
  ez2 = __expf(-az * az);
  const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f), 0.254829592f);
  const float e = 1.f - poly * ez2;
  erfz = z < 0.f ? -e : e;
}
__device__ __forceinline__ float gelu_f(float x) {
  float e, g;
  erf_and_gauss(x * 0.70710678118654752f, e, g);
  return 0.5f * x * (1.f + e);
}
__device__ __forceinline__ float dgelu_f(float x) {
  float e, g;
  erf_and_gauss(x * 0.70710678118654752f, e, g);   // g = exp(-x^2 / 2)
  return fmaf(x * 0.39894228040143268f, g, 0.5f * (1.f + e));
}

// One 128-row x 64-k operand slab, global -> registers (4 x 16 B per thread).  KC = true: storage [rows][k];
// false: storage [k][rows].  Rows past `nrows` read as zero.
template <bool KC>
__device__ __forceinline__ void load_slab(const bf16_t* __restrict__ P, int64_t ld, int row0, int nrows, int k0, uint4 (&r)[4]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = t + 256 * i;
    if (KC) {
      const int row = c >> 3, kc = c & 7;
      r[i] = (row0 + row < nrows) ? *reinterpret_cast<const uint4*>(P + (int64_t)(row0 + row) * ld + k0 + kc * 8) : make_uint4(0, 0, 0, 0);
    } else {
      const int k = c >> 4, rc = c & 15;
      r[i] = (row0 + rc * 8 < nrows) ? *reinterpret_cast<const uint4*>(P + (int64_t)(k0 + k) * ld + row0 + rc * 8) : make_uint4(0, 0, 0, 0);
    }
  }
}
template <bool KC>
__device__ __forceinline__ void store_slab(bf16_t* __restrict__ S, const uint4 (&r)[4]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = t + 256 * i;
    if (KC) *reinterpret_cast<uint4*>(S + (c >> 3) * LDK + (c & 7) * 8) = r[i];
    else *reinterpret_cast<uint4*>(S + (c >> 4) * LDR + (c & 15) * 8) = r[i];
  }
}

// The 8 contraction values k = ks*16 + 8*(lane/32) + 0..7 of tile row (rbase + lane%32), as an MFMA operand.
template <bool KC>
__device__ __forceinline__ bf16x8 fetch_operand(const bf16_t* __restrict__ S, int rbase, int ks, int lane) {
  if (KC) {
    return *reinterpret_cast<const bf16x8*>(S + (rbase + (lane & 31)) * LDK + ks * 16 + 8 * (lane >> 5));
  } else {
    // Transposing read: in every group of 16 lanes, lane j addresses 4 consecutive elements of k-row (j/4) at
    // column 4*(j%4); lane i of the group receives column i of those four k-rows.
    const int g = lane >> 4, j = lane & 15;
    const bf16_t* p = S + (ks * 16 + 8 * (g >> 1) + (j >> 2)) * LDR + rbase + 16 * (g & 1) + 4 * (j & 3);
    union { bf16x8 v; s16x4 h[2]; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * LDR));
    return u.v;
  }
}

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(256, 2) void k_gemm_bf16(GemmBf16Args a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
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
  load_slab<A_KC>(a.A, a.lda, i0, a.M, 0, ra);
  load_slab<B_KC>(a.B, a.ldb, j0, a.N, 0, rb);
  store_slab<A_KC>(smem, ra);
  store_slab<B_KC>(smem + TILE_ELEMS, rb);
  __syncthreads();
  for (int it = 0; it < iters; ++it) {
    const bf16_t* As = smem + (it & 1) * STAGE_ELEMS;
    const bf16_t* Bs = As + TILE_ELEMS;
    const bool more = it + 1 < iters;
    if (more) {
      const int nx = it + 1;
      const int kk = (nx >= nk ? nx - nk : nx) * BK;
      load_slab<A_KC>(a.A, a.lda, i0, a.M, kk, ra);
      load_slab<B_KC>(nx >= nk ? a.B2 : a.B, a.ldb, j0, a.N, kk, rb);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 av[2], bv[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) av[x] = fetch_operand<A_KC>(As, wr + x * 32, ks, lane);
#pragma unroll
      for (int y = 0; y < 2; ++y) bv[y] = fetch_operand<B_KC>(Bs, wc + y * 32, ks, lane);
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[x], bv[y], acc[x][y], 0, 0, 0);
    }
    if (more) {
      bf16_t* nxt = smem + ((it + 1) & 1) * STAGE_ELEMS;   // last read two iterations ago, before the previous barrier
      store_slab<A_KC>(nxt, ra);
      store_slab<B_KC>(nxt + TILE_ELEMS, rb);
    }
    __syncthreads();
  }

  // ---- epilogue: accumulators -> LDS (per-wave 64 x 64 fp32 tile) -> row-contiguous global accesses
  float* epi = reinterpret_cast<float*>(smem_raw) + wave * 64 * EPI_LD;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        epi[(x * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * EPI_LD + y * 32 + (lane & 31)] = acc[x][y][r];
  __syncthreads();
  const int cg = lane & 15, rq = lane >> 4;          // this lane: columns 4*cg .. 4*cg+3, rows rq, rq+4, ...
  const int gj = j0 + wc + 4 * cg;
  if (gj >= a.N) return;
  float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
  if (a.bias != nullptr) {
    bias = *reinterpret_cast<const float4*>(a.bias + gj);
    if (a.bias_v != nullptr && a.beps != nullptr && a.bsign != 0.f) {
      const float s = a.bsign * (*a.beps);
      const float4 bv = *reinterpret_cast<const float4*>(a.bias_v + gj);
      bias.x = fmaf(s, bv.x, bias.x); bias.y = fmaf(s, bv.y, bias.y); bias.z = fmaf(s, bv.z, bias.z); bias.w = fmaf(s, bv.w, bias.w);
    }
  }
#pragma unroll 4
  for (int itr = 0; itr < 16; ++itr) {
    const int row = rq + 4 * itr, gi = i0 + wr + row;
    if (gi >= a.M) break;
    const float4 v = *reinterpret_cast<const float4*>(epi + row * EPI_LD + 4 * cg);
    const int64_t o = (int64_t)gi * a.ldc + gj;
    float c[4] = {v.x + bias.x, v.y + bias.y, v.z + bias.z, v.w + bias.w};
    if (a.res16 != nullptr) {
      const uint2 rr = *reinterpret_cast<const uint2*>(a.res16 + o);
      c[0] += bf16_to_f32((bf16_t)rr.x); c[1] += bf16_to_f32((bf16_t)(rr.x >> 16));
      c[2] += bf16_to_f32((bf16_t)rr.y); c[3] += bf16_to_f32((bf16_t)(rr.y >> 16));
    }
    if (a.res32 != nullptr) {
      const float4 rr = *reinterpret_cast<const float4*>(a.res32 + o);
      c[0] += rr.x; c[1] += rr.y; c[2] += rr.z; c[3] += rr.w;
    }
    if (a.act == GEMM_ACT_GELU_FWD) {
      uint2 pk;
      pk.x = (uint32_t)f32_to_bf16(c[0]) | ((uint32_t)f32_to_bf16(c[1]) << 16);
      pk.y = (uint32_t)f32_to_bf16(c[2]) | ((uint32_t)f32_to_bf16(c[3]) << 16);
      *reinterpret_cast<uint2*>(a.C16_pre + o) = pk;
      // the backward pass sees the rounded pre-activation, so the activation is taken from it too
      c[0] = gelu_f(bf16_to_f32((bf16_t)pk.x)); c[1] = gelu_f(bf16_to_f32((bf16_t)(pk.x >> 16)));
      c[2] = gelu_f(bf16_to_f32((bf16_t)pk.y)); c[3] = gelu_f(bf16_to_f32((bf16_t)(pk.y >> 16)));
    } else if (a.act == GEMM_ACT_GELU_BWD) {
      const uint2 ax = *reinterpret_cast<const uint2*>(a.aux16 + o);
      c[0] *= dgelu_f(bf16_to_f32((bf16_t)ax.x)); c[1] *= dgelu_f(bf16_to_f32((bf16_t)(ax.x >> 16)));
      c[2] *= dgelu_f(bf16_to_f32((bf16_t)ax.y)); c[3] *= dgelu_f(bf16_to_f32((bf16_t)(ax.y >> 16)));
    }
    if (a.C32 != nullptr) *reinterpret_cast<float4*>(a.C32 + o) = make_float4(c[0], c[1], c[2], c[3]);
    if (a.C16 != nullptr) {
      uint2 pk;
      pk.x = (uint32_t)f32_to_bf16(c[0]) | ((uint32_t)f32_to_bf16(c[1]) << 16);
      pk.y = (uint32_t)f32_to_bf16(c[2]) | ((uint32_t)f32_to_bf16(c[3]) << 16);
      *reinterpret_cast<uint2*>(a.C16 + o) = pk;
    }
  }
}

template <bool A_KC, bool B_KC>
void launch_one(hipStream_t st, dim3 grid, const GemmBf16Args& a) {
  static bool configured = false;      // per instantiation: raise the dynamic LDS limit once
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16<A_KC, B_KC>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    configured = true;
  }
  k_gemm_bf16<A_KC, B_KC><<<grid, 256, LDS_BYTES, st>>>(a);
}
}  // namespace

const char* check_gemm_bf16(const GemmBf16Args& a) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return "empty GEMM";
  if (a.K % BK != 0) return "K must be a multiple of 64";
  if (a.M % 8 != 0 || a.N % 8 != 0) return "M and N must be multiples of 8";
  if (a.lda % 8 != 0 || a.ldb % 8 != 0 || a.ldc % 4 != 0) return "leading dimensions must be multiples of 8 (A, B) and 4 (C)";
  if (((uintptr_t)a.A | (uintptr_t)a.B | (uintptr_t)a.B2 | (uintptr_t)a.bias | (uintptr_t)a.bias_v | (uintptr_t)a.C32 |
       (uintptr_t)a.res32) & 15) return "operands, bias, fp32 residual and fp32 output must be 16-byte aligned";
  if (((uintptr_t)a.C16 | (uintptr_t)a.C16_pre | (uintptr_t)a.aux16 | (uintptr_t)a.res16) & 7) return "bf16 epilogue tensors must be 8-byte aligned";
  if (a.lda < (a.a_trans ? a.M : a.K) || a.ldb < (a.b_trans ? a.K : a.N) || a.ldc < a.N) return "leading dimension too small";
  return nullptr;
}

void launch_gemm_bf16(hipStream_t st, const GemmBf16Args& a) {
  dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM);
  const double flops = 2.0 * a.M * a.N * a.K * (a.B2 ? 2.0 : 1.0);   // hi + lo contracts over 2K
  ProfScope ps(st, a.a_trans ? F_GEMM_TN : (a.b_trans ? F_GEMM_NT : F_GEMM_NN), flops);
  // a_trans = 0: A is [M][K], contraction contiguous.  b_trans = 1: B is [N][K], contraction contiguous.
  if (!a.a_trans && a.b_trans) launch_one<true, true>(st, grid, a);
  else if (!a.a_trans && !a.b_trans) launch_one<true, false>(st, grid, a);
  else if (a.a_trans && !a.b_trans) launch_one<false, false>(st, grid, a);
  else launch_one<false, true>(st, grid, a);
}

}  // namespace sama
