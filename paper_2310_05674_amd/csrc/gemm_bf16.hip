// bf16 x bf16 -> fp32 contraction on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16) for the encoder's
// linear layers: forward (X W^T), dgrad (dY W) and wgrad (dY^T X) are one kernel template over the storage of its
// two operands.
//
//   block tile 128 x 128 (4 waves) or 256 x 128 (8 waves), k slab 64, each wave owning a 64 x 64 accumulator
//   LDS double buffer (one barrier per slab); three register sets keep the global loads of the next three slabs in
//   flight behind the MFMAs of the current one
//   an operand whose contraction index is contiguous in memory is staged as [row][k] and fetched with 16-byte reads;
//   an operand whose contraction index is the strided one (dgrad's W, both operands of wgrad) is staged as it lies
//   in memory, [k][row], and fetched with the transposing LDS read (ds_read_b64_tr_b16), so nothing is ever
//   transposed through registers or scattered into LDS
//   workgroup ids are remapped so that each XCD (own L2) works on a contiguous run of tiles
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

constexpr int BN = 128, BK = 64;
constexpr int LDK = BK + 8;        // [row][k] staging: 144-byte rows, conflict-free 16-byte reads
constexpr int EPI_LD = 64 + 4;     // fp32 row stride of a wave's 32 x 64 epilogue tile

// Block shapes: WROWS x 2 waves, each wave owning XT x 2 MFMA tiles of 32 x 32:
//   <2,2> 128 x 128, 4 waves of 64 x 64, two blocks per CU: keeps every CU busy on small problems
//   <4,2> 256 x 128, 8 waves of 64 x 64, one block per CU
//   <2,4> 256 x 128, 4 waves of 128 x 64, one block per CU: fewest LDS operand reads per MFMA
// The 256-row tiles move 25% fewer operand bytes per flop through L2 and the vector memory path.
template <int WROWS, int XT>
struct Shape {
  static constexpr int THREADS = WROWS * 128;
  static constexpr int WM = 32 * XT;         // rows of a wave tile
  static constexpr int BM = WROWS * WM;
  static constexpr int LDRA = BM + 32;       // [k][row] staging of A: 320 / 576-byte rows, conflict-free transposing reads
  static constexpr int LDRB = BN + 32;
  static constexpr int TILE_A = (BM * LDK > BK * LDRA) ? BM * LDK : BK * LDRA;
  static constexpr int TILE_B = BK * LDRB;   // >= BN * LDK
  static constexpr int STAGE = TILE_A + TILE_B;
  static constexpr int LDS_BYTES = 2 * STAGE * 2;
  static constexpr int NA = BM * 8 / THREADS;   // 16-byte pieces of the A slab per thread (4 or 8)
  static constexpr int NB = 1024 / THREADS;     // of the B slab (4 or 2)
};

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

// One 16-byte piece (i-th of this thread) of a ROWS-row x 64-k operand slab, global -> register.  KC = true:
// storage [rows][k]; false: storage [k][rows].  Rows past `nrows` are clamped to the last valid row (their
// products land in output rows / columns that the epilogue never stores), so every load is unconditional and in
// bounds.
template <bool KC, int ROWS, int THREADS>
__device__ __forceinline__ uint4 load_piece(const bf16_t* __restrict__ P, int64_t ld, int row0, int nrows, int k0, int i) {
  const int c = threadIdx.x + THREADS * i;
  if (KC) {
    const int row = min(row0 + (c >> 3), nrows - 1), kc = c & 7;
    return *reinterpret_cast<const uint4*>(P + (int64_t)row * ld + k0 + kc * 8);
  } else {
    constexpr int CPR = ROWS / 8;    // 16-byte chunks per k-row
    const int k = c / CPR, rs = min(row0 + (c % CPR) * 8, nrows - 8);
    return *reinterpret_cast<const uint4*>(P + (int64_t)(k0 + k) * ld + rs);
  }
}
template <bool KC, int ROWS, int THREADS>
__device__ __forceinline__ void store_piece(bf16_t* __restrict__ S, int i, const uint4& v) {
  const int c = threadIdx.x + THREADS * i;
  if (KC) *reinterpret_cast<uint4*>(S + (c >> 3) * LDK + (c & 7) * 8) = v;
  else {
    constexpr int CPR = ROWS / 8;
    *reinterpret_cast<uint4*>(S + (c / CPR) * (ROWS + 32) + (c % CPR) * 8) = v;
  }
}

// The 8 contraction values k = ks*16 + 8*(lane/32) + 0..7 of tile row (rbase + lane%32), as an MFMA operand.
template <bool KC, int LDR>
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

template <typename SH, int XT, bool A_KC, bool B_KC>
__device__ __forceinline__ void compute_slab(const bf16_t* __restrict__ As, const bf16_t* __restrict__ Bs, int wr, int wc, int lane,
                                             f32x16 (&acc)[XT][2]) {
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) {
    bf16x8 av[XT], bv[2];
#pragma unroll
    for (int x = 0; x < XT; ++x) av[x] = fetch_operand<A_KC, SH::LDRA>(As, wr + x * 32, ks, lane);
#pragma unroll
    for (int y = 0; y < 2; ++y) bv[y] = fetch_operand<B_KC, SH::LDRB>(Bs, wc + y * 32, ks, lane);
#pragma unroll
    for (int x = 0; x < XT; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[x], bv[y], acc[x][y], 0, 0, 0);
  }
}

template <int WROWS, int XT, bool A_KC, bool B_KC>
__global__ __launch_bounds__(WROWS * 128) void k_gemm_bf16(GemmBf16Args a, int gx, int ntiles, int tiles_per_xcd) {
  typedef Shape<WROWS, XT> SH;
  constexpr int BM = SH::BM, NT = SH::THREADS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wr = (wave >> 1) * SH::WM, wc = (wave & 1) * 64;
  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD one contiguous run of row-major tiles so that
  // the A row panels and B column panels it touches stay in its own L2.
  const int tile = (blockIdx.x & 7) * tiles_per_xcd + (blockIdx.x >> 3);
  if (tile >= ntiles) return;
  const int i0 = (tile / gx) * BM, j0 = (tile % gx) * BN;

  f32x16 acc[XT][2];
#pragma unroll
  for (int x = 0; x < XT; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  const int nk = a.K / BK;
  const int iters = (a.B2 != nullptr) ? 2 * nk : nk;
  // Three register sets rotate through the slabs: while slab i is multiplied out of LDS, slabs i+1 .. i+3 are in
  // registers or still in flight, so a slab's global loads have two to three slab-times to land.  (Named scalars
  // and branch-free steady state: the sets must stay in registers and the wait counters exact.)
  uint4 a00, a01, a02, a03, a04, a05, a06, a07, b00, b01, b02, b03, a10, a11, a12, a13, a14, a15, a16, a17, b10, b11, b12, b13,
      a20, a21, a22, a23, a24, a25, a26, a27, b20, b21, b22, b23;
#define SAMA_LOAD(SL, S)                                                                          \
  {                                                                                               \
    const int sl_ = (SL);                                                                         \
    const int kk_ = (sl_ >= nk ? sl_ - nk : sl_) * BK;                                            \
    const bf16_t* bp_ = sl_ >= nk ? a.B2 : a.B;                                                   \
    a##S##0 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 0);                              \
    a##S##1 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 1);                              \
    a##S##2 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 2);                              \
    a##S##3 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 3);                              \
    if (SH::NA > 4) {                                                                             \
      a##S##4 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 4);                            \
      a##S##5 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 5);                            \
      a##S##6 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 6);                            \
      a##S##7 = load_piece<A_KC, BM, NT>(a.A, a.lda, i0, a.M, kk_, 7);                            \
    }                                                                                             \
    b##S##0 = load_piece<B_KC, BN, NT>(bp_, a.ldb, j0, a.N, kk_, 0);                              \
    b##S##1 = load_piece<B_KC, BN, NT>(bp_, a.ldb, j0, a.N, kk_, 1);                              \
    if (SH::NB > 2) {                                                                             \
      b##S##2 = load_piece<B_KC, BN, NT>(bp_, a.ldb, j0, a.N, kk_, 2);                            \
      b##S##3 = load_piece<B_KC, BN, NT>(bp_, a.ldb, j0, a.N, kk_, 3);                            \
    }                                                                                             \
  }
#define SAMA_STORE(STG, S)                                                                        \
  {                                                                                               \
    bf16_t* sa_ = smem + (STG) * SH::STAGE;                                                       \
    bf16_t* sb_ = sa_ + SH::TILE_A;                                                               \
    store_piece<A_KC, BM, NT>(sa_, 0, a##S##0); store_piece<A_KC, BM, NT>(sa_, 1, a##S##1);       \
    store_piece<A_KC, BM, NT>(sa_, 2, a##S##2); store_piece<A_KC, BM, NT>(sa_, 3, a##S##3);       \
    if (SH::NA > 4) {                                                                             \
      store_piece<A_KC, BM, NT>(sa_, 4, a##S##4); store_piece<A_KC, BM, NT>(sa_, 5, a##S##5);     \
      store_piece<A_KC, BM, NT>(sa_, 6, a##S##6); store_piece<A_KC, BM, NT>(sa_, 7, a##S##7);     \
    }                                                                                             \
    store_piece<B_KC, BN, NT>(sb_, 0, b##S##0); store_piece<B_KC, BN, NT>(sb_, 1, b##S##1);       \
    if (SH::NB > 2) {                                                                             \
      store_piece<B_KC, BN, NT>(sb_, 2, b##S##2); store_piece<B_KC, BN, NT>(sb_, 3, b##S##3);     \
    }                                                                                             \
  }
#define SAMA_COMPUTE(I)                                                                           \
  {                                                                                               \
    const bf16_t* As_ = smem + ((I) & 1) * SH::STAGE;                                             \
    compute_slab<SH, XT, A_KC, B_KC>(As_, As_ + SH::TILE_A, wr, wc, lane, acc);                   \
  }
  // slab I: start the loads of slab I+3 into set L (the set slab I came from); multiply slab I out of its LDS
  // stage; move slab I+1 from set T into the other stage (last read during slab I-1, before the previous barrier)
#define SAMA_PHASE_FULL(I, L, T)                                                                  \
  {                                                                                               \
    SAMA_LOAD((I) + 3, L)                                                                         \
    SAMA_COMPUTE(I)                                                                               \
    SAMA_STORE(((I) + 1) & 1, T)                                                                  \
    __syncthreads();                                                                              \
  }
#define SAMA_PHASE(I, L, T)                                                                       \
  {                                                                                               \
    if ((I) + 3 < iters) SAMA_LOAD((I) + 3, L)                                                    \
    SAMA_COMPUTE(I)                                                                               \
    if ((I) + 1 < iters) SAMA_STORE(((I) + 1) & 1, T)                                             \
    __syncthreads();                                                                              \
  }
  SAMA_LOAD(0, 0)
  if (iters > 1) SAMA_LOAD(1, 1)
  if (iters > 2) SAMA_LOAD(2, 2)
  SAMA_STORE(0, 0)
  __syncthreads();
  int it = 0;
  for (; it + 5 < iters; it += 3) {
    SAMA_PHASE_FULL(it, 0, 1)
    SAMA_PHASE_FULL(it + 1, 1, 2)
    SAMA_PHASE_FULL(it + 2, 2, 0)
  }
  for (; it < iters; it += 3) {
    SAMA_PHASE(it, 0, 1)
    if (it + 1 < iters) SAMA_PHASE(it + 1, 1, 2)
    if (it + 2 < iters) SAMA_PHASE(it + 2, 2, 0)
  }
#undef SAMA_PHASE
#undef SAMA_PHASE_FULL
#undef SAMA_COMPUTE
#undef SAMA_STORE
#undef SAMA_LOAD

  // ---- epilogue: accumulators -> LDS (per wave, 32 x 64 fp32 at a time) -> row-contiguous global accesses
  float* epi = reinterpret_cast<float*>(smem_raw) + wave * 32 * EPI_LD;
  const int cg = lane & 15, rq = lane >> 4;          // this lane: columns 4*cg .. 4*cg+3, rows rq, rq+4, ...
  const int gj = j0 + wc + 4 * cg;
  const bool col_ok = gj < a.N;
  float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
  if (col_ok && a.bias != nullptr) {
    bias = *reinterpret_cast<const float4*>(a.bias + gj);
    if (a.bias_v != nullptr && a.beps != nullptr && a.bsign != 0.f) {
      const float s = a.bsign * (*a.beps);
      const float4 bv = *reinterpret_cast<const float4*>(a.bias_v + gj);
      bias.x = fmaf(s, bv.x, bias.x); bias.y = fmaf(s, bv.y, bias.y); bias.z = fmaf(s, bv.z, bias.z); bias.w = fmaf(s, bv.w, bias.w);
    }
  }
#pragma unroll
  for (int x = 0; x < XT; ++x) {
    if (x > 0) __syncthreads();
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        epi[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * EPI_LD + y * 32 + (lane & 31)] = acc[x][y][r];
    __syncthreads();
    if (!col_ok) continue;
#pragma unroll 4
    for (int itr = 0; itr < 8; ++itr) {
      const int row = rq + 4 * itr, gi = i0 + wr + x * 32 + row;
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
}

template <int WROWS, int XT, bool A_KC, bool B_KC>
void launch_shape(hipStream_t st, const GemmBf16Args& a) {
  typedef Shape<WROWS, XT> SH;
  static bool configured = false;      // per instantiation: raise the dynamic LDS limit once
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16<WROWS, XT, A_KC, B_KC>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, SH::LDS_BYTES);
    configured = true;
  }
  const int gx = (a.N + BN - 1) / BN, gy = (a.M + SH::BM - 1) / SH::BM, ntiles = gx * gy, per_xcd = (ntiles + 7) / 8;
  k_gemm_bf16<WROWS, XT, A_KC, B_KC><<<8 * per_xcd, SH::THREADS, SH::LDS_BYTES, st>>>(a, gx, ntiles, per_xcd);
}
int g_force_shape = 0;   // 0 = heuristic; 1, 2, 3 = force <2,2>, <4,2>, <2,4> (tuning hook)
template <bool A_KC, bool B_KC>
void launch_one(hipStream_t st, const GemmBf16Args& a) {
  // 256 x 128 tiles when they still give (nearly) every CU a block, else 128 x 128
  const int64_t big_tiles = (int64_t)((a.M + 255) / 256) * ((a.N + BN - 1) / BN);
  int shape = g_force_shape ? g_force_shape : (big_tiles >= 192 ? 2 : 1);
  if (shape == 3) launch_shape<2, 4, A_KC, B_KC>(st, a);
  else if (shape == 2) launch_shape<4, 2, A_KC, B_KC>(st, a);
  else launch_shape<2, 2, A_KC, B_KC>(st, a);
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

void gemm_bf16_force_shape(int s) { g_force_shape = s; }

void launch_gemm_bf16(hipStream_t st, const GemmBf16Args& a) {
  const double flops = 2.0 * a.M * a.N * a.K * (a.B2 ? 2.0 : 1.0);   // hi + lo contracts over 2K
  ProfScope ps(st, a.a_trans ? F_GEMM_TN : (a.b_trans ? F_GEMM_NT : F_GEMM_NN), flops);
  // a_trans = 0: A is [M][K], contraction contiguous.  b_trans = 1: B is [N][K], contraction contiguous.
  if (!a.a_trans && a.b_trans) launch_one<true, true>(st, a);
  else if (!a.a_trans && !a.b_trans) launch_one<true, false>(st, a);
  else if (a.a_trans && !a.b_trans) launch_one<false, false>(st, a);
  else launch_one<false, true>(st, a);
}

}  // namespace sama
