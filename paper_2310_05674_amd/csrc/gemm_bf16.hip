// bf16 x bf16 -> fp32 contraction on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16) for the encoder's linear
// layers: forward (X W^T), dgrad (dY W) and wgrad (dY^T X) are one kernel template over the storage of its two
// operands.
//
//   operand slabs go global -> LDS directly (global_load_lds_dwordx4, 1 KB per wave instruction) into dense,
//   XOR-swizzled stages, NSTAGE - 1 slabs in flight, one barrier per slab; no staging registers
//   an operand whose contraction index is contiguous in memory is staged [row][k] and fetched with 16-byte reads;
//   one whose contraction index is the strided one (dgrad's W, both operands of wgrad) is staged as it lies in
//   memory, [k][row], and fetched with the transposing LDS read (ds_read_b64_tr_b16)
//   the MFMA operands of k-step t + 1 are fetched while the MFMAs of step t issue, also across the slab boundary
//   measured on MI355X: a CU ingests at most ~25-30 B/clk from L2 (about 100-128 outstanding 128-byte requests
//   times the loaded L2 latency), so the block tile, not the MFMA rate, bounds the kernel: 256 x 256 tiles need
//   32 B/clk per CU at the MFMA peak, 256 x 128 need 48, 128 x 128 need 64
//   workgroup ids are remapped so that each XCD (own L2) works on a compact patch of tiles
//   the accumulators leave through LDS so that every global access of the epilogue is a full row segment
//
// For the theta +- eps v passes of Eq. 5 and the direct-gradient pass the weight operand is hi + lo (two bf16
// halves).  DUAL tiles stage the A slab once together with the hi and the lo slab of B and issue two MFMAs per A
// operand, so A is neither loaded nor fetched twice.
//
// Several independent problems of one storage class can share a launch (the + and - pass of Eq. 5, the four weight
// gradients of a layer): more tiles per launch for the small per-layer shapes.
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
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gvoid;
constexpr int LDS_MAX = 160 * 1024;

template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int NSTAGE_, bool DUAL_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, NSTAGE = NSTAGE_;
  static constexpr bool DUAL = DUAL_;
  static constexpr int WAVES = WGM * WGN, THREADS = WAVES * 64;
  static constexpr int WM = BM / WGM, WN = BN / WGN, XT = WM / 32, YT = WN / 32;
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + (DUAL ? 2 : 1) * B_BYTES;
  static constexpr int NLA = A_BYTES / 1024 / WAVES, NLB = B_BYTES / 1024 / WAVES;   // wave-level 1 KB loads per slab
  static constexpr int NL = NLA + (DUAL ? 2 : 1) * NLB;
  static_assert(LDS_MAX >= NSTAGE * STAGE_BYTES, "stages exceed the 160 KB of LDS");
  static constexpr int LDS_MAIN = NSTAGE * STAGE_BYTES;
  static constexpr int EPI_LD = WN + 8;   // 4 rows apart = 32 banks apart: the two lane halves of a staging write do not collide
  static constexpr int LDS_EPI = WAVES * 32 * EPI_LD * 4;
  static constexpr int LDS_BYTES = LDS_MAIN > LDS_EPI ? LDS_MAIN : LDS_EPI;
  static_assert(A_BYTES % (1024 * WAVES) == 0 && B_BYTES % (1024 * WAVES) == 0, "slab must split into whole wave loads");
  static_assert(NL * (NSTAGE - 2) <= 63, "vmcnt range");
};

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
  erf_and_gauss(x * 0.70710678118654752f, e, g);
  return fmaf(x * 0.39894228040143268f, g, 0.5f * (1.f + e));
}

// Byte offset (relative to the slab's first element in global memory) of the 16-byte piece that belongs at byte
// `ldsoff` of an operand's dense LDS stage.
//   KC (contraction contiguous, storage [rows][k]): stage [R][BK]; the 16-byte chunk index within a row is XORed
//     with (row / RP) % NCH so that 16 consecutive rows at one logical chunk fill all 64 banks.
//   KS (contraction strided, storage [k][rows]): stage [BK][R]; the 64-byte chunk index within a k-row is XORed with
//     (k-row / RP) % W (RP = k-rows per 256 bytes, W = min(chunks per k-row, 4)) so that the four k-rows one
//     transposing read touches fill all 64 banks.
// Rows past `nrows` are clamped (their products land in outputs the epilogue never stores).
template <bool KC, int R, int BK>
__device__ __forceinline__ uint32_t piece_offset(int ldsoff, int row0, int nrows, int64_t ld) {
  if (KC) {
    constexpr int RB = BK * 2, RP = 256 / RB, NCH = RB / 16;
    const int r = ldsoff / RB, p = (ldsoff % RB) / 16;
    const int c = p ^ ((r / RP) % NCH);
    return (uint32_t)(((int64_t)min(row0 + r, nrows - 1) * ld + c * 8) * 2);
  } else {
    constexpr int RBS = R * 2, RP = RBS >= 256 ? 1 : 256 / RBS, W = RBS / 64 < 4 ? RBS / 64 : 4;
    const int kr = ldsoff / RBS, q16 = (ldsoff % RBS) / 16;
    const int ql = (((q16 >> 2) ^ ((kr / RP) % W)) << 2) | (q16 & 3);
    return (uint32_t)(((int64_t)kr * ld + min(row0 + ql * 8, nrows - 8)) * 2);
  }
}

// MFMA operand (8 contraction values k = ks*16 + 8*(lane/32) + 0..7 of tile row tb + lane%32) out of a swizzled stage.
// `lo` is the lane-dependent part precomputed by fetch_lane_offset, `tb` the first row of the 32-row tile.
template <bool KC, int R, int BK>
__device__ __forceinline__ int fetch_lane_offset(int lane, int ks_or_tile) {
  if (KC) {
    constexpr int RB = BK * 2, RP = 256 / RB, NCH = RB / 16;
    const int rl = lane & 31, hi = lane >> 5;
    const int s = (rl / RP) % NCH;
    return rl * RB + (((2 * ks_or_tile + hi) ^ s) * 16);                  // per ks
  } else {
    constexpr int RBS = R * 2, RP = RBS >= 256 ? 1 : 256 / RBS, W = RBS / 64 < 4 ? RBS / 64 : 4;
    const int g = lane >> 4, j = lane & 15;
    const int cc = ks_or_tile;                                            // 64-byte chunk of the tile = tile_row0 / 32
    const int kr = 8 * (g >> 1) + (j >> 2);                               // (kr / RP) % W is the same for kr + 4 and kr + 16
    return kr * RBS + ((cc ^ ((kr / RP) % W)) * 64) + (16 * (g & 1) + 4 * (j & 3)) * 2;   // per tile
  }
}

struct GemmBatch {
  GemmBf16Args p[GEMM_MAX_BATCH];
  int first_tile[GEMM_MAX_BATCH + 1];   // tile ids [first_tile[k], first_tile[k + 1]) belong to problem k
  int count, group;
};

template <typename T, bool A_KC, bool B_KC>
__global__ __launch_bounds__(T::THREADS) void k_gemm_bf16(GemmBatch batch, int ntiles, int tiles_per_xcd) {
  constexpr int BM = T::BM, BN = T::BN, BK = T::BK, XT = T::XT, YT = T::YT, NSTAGE = T::NSTAGE, WAVES = T::WAVES;
  constexpr bool DUAL = T::DUAL;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wr = (wave / T::WGN) * T::WM, wc = (wave % T::WGN) * T::WN;
  // XCD-aware order: workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous run of tile ids, and
  // tile ids walk down `group` tile rows before moving one tile column to the right, so that the tiles in flight on
  // one XCD form a compact patch (few distinct A and B panels in its L2).
  int pid = (blockIdx.x & 7) * tiles_per_xcd + (blockIdx.x >> 3);
  if (pid >= ntiles) return;
  int prob = 0;
#pragma unroll
  for (int k = 1; k < GEMM_MAX_BATCH; ++k)
    if (k < batch.count && pid >= batch.first_tile[k]) prob = k;
  pid -= batch.first_tile[prob];
  const GemmBf16Args& a = batch.p[prob];
  const int group = batch.group;
  const int gx = (a.N + BN - 1) / BN, gy = (a.M + BM - 1) / BM;
  const int width = group * gx, grp = pid / width, first = grp * group;
  const int gsz = min(gy - first, group);
  const int ti = first + (pid % width) % gsz, tj = (pid % width) / gsz;
  const int i0 = ti * BM, j0 = tj * BN;

  f32x16 acc[XT][YT];
#pragma unroll
  for (int x = 0; x < XT; ++x)
#pragma unroll
    for (int y = 0; y < YT; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  const int nk = a.K / BK;
  // The operand pointers live in registers for the whole k loop (read through `a` they would be re-fetched from the
  // kernel-argument segment after every inline-assembly load, a scalar-memory round trip per slab).
  const char* const pA = reinterpret_cast<const char*>(a.A);
  const char* const pB = reinterpret_cast<const char*>(a.B);
  const char* const pB2 = reinterpret_cast<const char*>(a.B2);
  const int iters = (!DUAL && pB2 != nullptr) ? 2 * nk : nk;   // non-DUAL tiles contract with hi, then with lo

  // per-lane global offsets of this wave's loads
  uint32_t offA[T::NLA], offB[T::NLB];
#pragma unroll
  for (int q = 0; q < T::NLA; ++q) offA[q] = piece_offset<A_KC, BM, BK>((q * WAVES + wave) * 1024 + lane * 16, i0, a.M, a.lda);
#pragma unroll
  for (int q = 0; q < T::NLB; ++q) offB[q] = piece_offset<B_KC, BN, BK>((q * WAVES + wave) * 1024 + lane * 16, j0, a.N, a.ldb);
  const int64_t stepA = A_KC ? (int64_t)BK * 2 : (int64_t)BK * a.lda * 2;   // bytes per slab
  const int64_t stepB = B_KC ? (int64_t)BK * 2 : (int64_t)BK * a.ldb * 2;

  // Direct global -> LDS loads: lane l of a wave-level load lands at (m0) + 16 l.  Written as inline assembly so
  // that the only waits on them are the explicit vmcnt waits below.
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void*)smem_raw;
  // All NL wave-level loads of a slab are issued together right after the barrier that frees their stage (spreading
  // them over the k-steps of the slab computed meanwhile measured 3-8% slower: it shortens the prefetch distance).
  constexpr int KS = BK / 16;
  auto issue = [&](int sl) {
    if (sl >= iters) return;
    const int stage = sl % NSTAGE;
    const int kq = sl >= nk ? sl - nk : sl;
    const char* ap = pA + kq * stepA;
    const char* bp = (sl >= nk ? pB2 : pB) + kq * stepB;
    const char* b2p = pB2 + kq * stepB;
    const uint32_t sa = lds0 + stage * T::STAGE_BYTES + wave * 1024;
    const uint32_t sb = sa + T::A_BYTES;
#pragma unroll
    for (int t = 0; t < T::NL; ++t) {
      if (t < T::NLA) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(sa + t * WAVES * 1024), "v"(offA[t]), "s"(ap) : "memory", "m0");
      } else if (t < T::NLA + T::NLB) {
        const int q = t - T::NLA;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(sb + q * WAVES * 1024), "v"(offB[q]), "s"(bp) : "memory", "m0");
      } else {
        const int q = t - T::NLA - T::NLB;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(sb + T::B_BYTES + q * WAVES * 1024), "v"(offB[q]), "s"(b2p) : "memory", "m0");
      }
    }
  };

  // lane-dependent parts of the operand fetch addresses
  int fa[A_KC ? BK / 16 : XT], fb[B_KC ? BK / 16 : YT];
  if (A_KC) {
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) fa[ks] = fetch_lane_offset<true, BM, BK>(lane, ks) + wr * BK * 2;
  } else {
#pragma unroll
    for (int x = 0; x < XT; ++x) fa[x] = fetch_lane_offset<false, BM, BK>(lane, (wr >> 5) + x);
  }
  if (B_KC) {
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) fb[ks] = fetch_lane_offset<true, BN, BK>(lane, ks) + wc * BK * 2;
  } else {
#pragma unroll
    for (int y = 0; y < YT; ++y) fb[y] = fetch_lane_offset<false, BN, BK>(lane, (wc >> 5) + y);
  }

  auto fetchA = [&](const unsigned char* sa, int x, int ks) -> bf16x8 {
    if (A_KC) return *reinterpret_cast<const bf16x8*>(sa + fa[ks] + x * 32 * BK * 2);
    const unsigned char* p = sa + fa[x] + ks * 16 * BM * 2;
    union { bf16x8 v; s16x4 h[2]; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * BM * 2));
    return u.v;
  };
  auto fetchB = [&](const unsigned char* sb, int y, int ks) -> bf16x8 {
    if (B_KC) return *reinterpret_cast<const bf16x8*>(sb + fb[ks] + y * 32 * BK * 2);
    const unsigned char* p = sb + fb[y] + ks * 16 * BN * 2;
    union { bf16x8 v; s16x4 h[2]; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * BN * 2));
    return u.v;
  };

  // ---- pipeline: NSTAGE - 1 slabs in flight; the k-steps of all slabs form one stream in which the operands of
  // step t + 1 are fetched from LDS before the MFMAs of step t are issued (also across the slab boundary, so the
  // LDS latency after a barrier hides behind the last MFMAs of the previous slab)
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s) issue(s);

  static_assert(KS % 2 == 0, "operand double buffer parity");
  bf16x8 av[2][XT], bv[2][YT], bw[2][DUAL ? YT : 1];
  // make slab `sl` visible: own loads landed, then everyone's; afterwards the stage of slab sl - 1 is free
  auto arrive = [&](int sl) {
    const int younger = iters - 1 - sl;
    if (younger >= NSTAGE - 2) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(T::NL * (NSTAGE - 2)) : "memory");
    } else if (NSTAGE >= 4 && younger == NSTAGE - 3) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(T::NL * (NSTAGE >= 4 ? NSTAGE - 3 : 0)) : "memory");
    } else if (NSTAGE >= 5 && younger == NSTAGE - 4) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(T::NL * (NSTAGE >= 5 ? NSTAGE - 4 : 0)) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    issue(sl + NSTAGE - 1);
  };
  auto fetch = [&](int sl, int ks, int buf) {
    const unsigned char* sa = smem_raw + (sl % NSTAGE) * T::STAGE_BYTES;
    const unsigned char* sb = sa + T::A_BYTES;
#pragma unroll
    for (int x = 0; x < XT; ++x) av[buf][x] = fetchA(sa, x, ks);
#pragma unroll
    for (int y = 0; y < YT; ++y) bv[buf][y] = fetchB(sb, y, ks);
    if (DUAL) {
#pragma unroll
      for (int y = 0; y < YT; ++y) bw[buf][y] = fetchB(sb + T::B_BYTES, y, ks);
    }
  };
  arrive(0);
  fetch(0, 0, 0);
  auto mfma_step = [&](int cur) {
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int x = 0; x < XT; ++x)
#pragma unroll
      for (int y = 0; y < YT; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[cur][x], bv[cur][y], acc[x][y], 0, 0, 0);
    if (DUAL) {
#pragma unroll
      for (int x = 0; x < XT; ++x)
#pragma unroll
        for (int y = 0; y < YT; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[cur][x], bw[cur][y], acc[x][y], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  for (int i = 0; i + 1 < iters; ++i) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = ks & 1;
      if (ks + 1 < KS) {
        fetch(i, ks + 1, cur ^ 1);
      } else {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's reads of slab i are complete
        arrive(i + 1);
        fetch(i + 1, 0, cur ^ 1);
      }
      mfma_step(cur);
    }
  }
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {   // last slab
    if (ks + 1 < KS) fetch(iters - 1, ks + 1, (ks & 1) ^ 1);
    mfma_step(ks & 1);
  }
  __syncthreads();

  // ---- epilogue: accumulators -> LDS (per wave, 32 x WN fp32 at a time) -> row-contiguous global accesses
  constexpr int EPI_LD = T::EPI_LD, LPR = T::WN / 4, RPP = 64 / LPR;   // lanes per row, rows per pass
  float* epi = reinterpret_cast<float*>(smem_raw) + wave * 32 * EPI_LD;
  const int cg = lane % LPR, rq = lane / LPR;
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
  const bf16_t* const res16 = a.res16; const float* const res32 = a.res32; const bf16_t* const aux16 = a.aux16;
  bf16_t* const C16_pre = a.C16_pre; bf16_t* const C16 = a.C16; float* const C32 = a.C32;
  const int act = a.act, Mrows = a.M;
  const int64_t ldc = a.ldc;
  constexpr int NIT = 32 / RPP;
  // one output vector: bias, residual, activation, stores
  auto finish = [&](const float4& v, int64_t o, const float4& rr32, const uint2& rr16, const uint2& axv) {
    float c[4] = {v.x + bias.x, v.y + bias.y, v.z + bias.z, v.w + bias.w};
    if (res16 != nullptr) {
      c[0] += bf16_to_f32((bf16_t)rr16.x); c[1] += bf16_to_f32((bf16_t)(rr16.x >> 16));
      c[2] += bf16_to_f32((bf16_t)rr16.y); c[3] += bf16_to_f32((bf16_t)(rr16.y >> 16));
    }
    if (res32 != nullptr) { c[0] += rr32.x; c[1] += rr32.y; c[2] += rr32.z; c[3] += rr32.w; }
    if (act == GEMM_ACT_GELU_FWD) {
      uint2 pk;
      pk.x = pack_bf16x2(c[0], c[1]);
      pk.y = pack_bf16x2(c[2], c[3]);
      if (C16_pre != nullptr) *reinterpret_cast<uint2*>(C16_pre + o) = pk;   // forward-only passes do not keep it
      // the backward pass sees the rounded pre-activation, so the activation is taken from it too
      c[0] = gelu_f(bf16_to_f32((bf16_t)pk.x)); c[1] = gelu_f(bf16_to_f32((bf16_t)(pk.x >> 16)));
      c[2] = gelu_f(bf16_to_f32((bf16_t)pk.y)); c[3] = gelu_f(bf16_to_f32((bf16_t)(pk.y >> 16)));
    } else if (act == GEMM_ACT_GELU_BWD) {
      c[0] *= dgelu_f(bf16_to_f32((bf16_t)axv.x)); c[1] *= dgelu_f(bf16_to_f32((bf16_t)(axv.x >> 16)));
      c[2] *= dgelu_f(bf16_to_f32((bf16_t)axv.y)); c[3] *= dgelu_f(bf16_to_f32((bf16_t)(axv.y >> 16)));
    }
    if (C32 != nullptr) *reinterpret_cast<float4*>(C32 + o) = make_float4(c[0], c[1], c[2], c[3]);
    if (C16 != nullptr) {
      uint2 pk;
      pk.x = pack_bf16x2(c[0], c[1]);
      pk.y = pack_bf16x2(c[2], c[3]);
      *reinterpret_cast<uint2*>(C16 + o) = pk;
    }
  };
  const bool side = res32 != nullptr || res16 != nullptr || act == GEMM_ACT_GELU_BWD;
  constexpr bool PREFETCH = NIT <= 8;   // wider wave tiles have no registers to spare for the side inputs of a whole slice
#pragma unroll
  for (int x = 0; x < XT; ++x) {
    // Side inputs of this 32-row slice (residual, saved pre-activation) are requested before the accumulators go
    // through LDS, so that their latency hides behind the staging.  Launches without side inputs skip this path.
    float4 r32[PREFETCH ? NIT : 1];
    uint2 r16[PREFETCH ? NIT : 1], ax[PREFETCH ? NIT : 1];
    if (PREFETCH && side && col_ok) {
#pragma unroll
      for (int itr = 0; itr < (PREFETCH ? NIT : 1); ++itr) {
        const int gi = i0 + wr + x * 32 + rq + RPP * itr;
        r32[itr] = make_float4(0.f, 0.f, 0.f, 0.f); r16[itr] = make_uint2(0u, 0u); ax[itr] = make_uint2(0u, 0u);
        if (gi < Mrows) {
          const int64_t o = (int64_t)gi * ldc + gj;
          if (res32 != nullptr) r32[itr] = *reinterpret_cast<const float4*>(res32 + o);
          if (res16 != nullptr) r16[itr] = *reinterpret_cast<const uint2*>(res16 + o);
          if (act == GEMM_ACT_GELU_BWD) ax[itr] = *reinterpret_cast<const uint2*>(aux16 + o);
        }
      }
    }
    // the staging region is private to the wave: LDS operations of one wave complete in order, no block barrier
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
#pragma unroll
    for (int y = 0; y < YT; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        epi[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * EPI_LD + y * 32 + (lane & 31)] = acc[x][y][r];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (!col_ok) continue;
    if (side && PREFETCH) {
#pragma unroll
      for (int itr = 0; itr < (PREFETCH ? NIT : 1); ++itr) {
        const int row = rq + RPP * itr, gi = i0 + wr + x * 32 + row;
        if (gi >= Mrows) break;
        finish(*reinterpret_cast<const float4*>(epi + row * EPI_LD + 4 * cg), (int64_t)gi * ldc + gj, r32[itr], r16[itr], ax[itr]);
      }
    } else if (side) {
#pragma unroll 4
      for (int itr = 0; itr < NIT; ++itr) {
        const int row = rq + RPP * itr, gi = i0 + wr + x * 32 + row;
        if (gi >= Mrows) break;
        const int64_t o = (int64_t)gi * ldc + gj;
        float4 q32 = make_float4(0.f, 0.f, 0.f, 0.f);
        uint2 q16 = make_uint2(0u, 0u), qa = make_uint2(0u, 0u);
        if (res32 != nullptr) q32 = *reinterpret_cast<const float4*>(res32 + o);
        if (res16 != nullptr) q16 = *reinterpret_cast<const uint2*>(res16 + o);
        if (act == GEMM_ACT_GELU_BWD) qa = *reinterpret_cast<const uint2*>(aux16 + o);
        finish(*reinterpret_cast<const float4*>(epi + row * EPI_LD + 4 * cg), o, q32, q16, qa);
      }
    } else {
      const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
      const uint2 z2 = make_uint2(0u, 0u);
#pragma unroll 4
      for (int itr = 0; itr < NIT; ++itr) {
        const int row = rq + RPP * itr, gi = i0 + wr + x * 32 + row;
        if (gi >= Mrows) break;
        finish(*reinterpret_cast<const float4*>(epi + row * EPI_LD + 4 * cg), (int64_t)gi * ldc + gj, z4, z2, z2);
      }
    }
  }
}

template <typename T, bool A_KC, bool B_KC>
void launch_tile(ProfScope& ps, hipStream_t st, const GemmBf16Args* p, int count, int group) {
  static bool configured = false;      // per instantiation: raise the dynamic LDS limit once
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16<T, A_KC, B_KC>), hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    configured = true;
  }
  GemmBatch b{};
  b.count = count; b.group = group;
  int nt = 0;
  for (int k = 0; k < count; ++k) {
    b.p[k] = p[k];
    b.first_tile[k] = nt;
    nt += ((p[k].N + T::BN - 1) / T::BN) * ((p[k].M + T::BM - 1) / T::BM);
  }
  for (int k = count; k <= GEMM_MAX_BATCH; ++k) b.first_tile[k] = nt;
  const int per_xcd = (nt + 7) / 8;
  launch_kernel(ps, k_gemm_bf16<T, A_KC, B_KC>, 8 * per_xcd, T::THREADS, T::LDS_BYTES, st, b, nt, per_xcd);
}

// Tile configurations <BM, BN, BK, waves in M, waves in N, stages, DUAL>
typedef Tile<256, 256, 64, 2, 4, 2, false> TL;    // 8 waves of 128 x 64, 2 stages of 64 KB
typedef Tile<256, 128, 64, 4, 2, 3, false> TM;    // 8 waves of 64 x 64, 3 stages of 48 KB
typedef Tile<128, 128, 64, 2, 2, 2, false> TS;    // 4 waves of 64 x 64, 2 stages of 32 KB: two blocks per CU
typedef Tile<128, 64, 64, 2, 2, 3, false> TX;     // 4 waves of 64 x 32, 3 stages of 24 KB: two blocks per CU
typedef Tile<128, 64, 64, 2, 2, 4, false> TX4;    // 4 stages: one block per CU, deeper prefetch
typedef Tile<128, 64, 64, 4, 2, 4, false> TX8;    // 8 waves of 32 x 32: the small tile when one block per CU is all there is
typedef Tile<128, 128, 64, 4, 2, 3, false> TS8;   // 8 waves of 32 x 64
typedef Tile<256, 256, 32, 2, 4, 3, true> DL;     // DUAL: 3 stages of 48 KB
typedef Tile<256, 128, 64, 4, 2, 2, true> DM;     // 2 stages of 64 KB
typedef Tile<128, 128, 64, 2, 2, 3, true> DS;     // 3 stages of 48 KB
typedef Tile<128, 64, 64, 2, 2, 2, true> DX;      // 2 stages of 32 KB: two blocks per CU
typedef Tile<128, 64, 64, 2, 2, 4, true> DX4;     // 4 stages of 32 KB

int g_force_shape = 0, g_group = 8;

// Which block tile: estimated cycles per 64-deep k-slab on the busiest CU.  A CU ingests ~25 B/clk from L2 (measured),
// i.e. 5.12 clk per 128-byte operand row, and sustains ~70% of its 4096 flop/clk MFMA rate; rounds = how many tiles
// the busiest of the 256 CUs works through.  The two smaller tiles exist in a form of which two blocks fit a CU side
// by side (measured: two co-resident blocks take 1.3 times one) and, for single-term problems, in an 8-wave form that
// is the fastest when one block per CU is all the problem gives.  Near-ties go to the larger tile.
int pick_tile(const GemmBf16Args* p, int count, bool dual) {
  static const int dims[4][2] = {{256, 256}, {256, 128}, {128, 128}, {128, 64}};
  const double nb = dual ? 2.0 : 1.0;
  int best = 0;
  int64_t best_tiles = 0;
  double best_cost = 0.0;
  for (int c = 0; c < 4; ++c) {
    const int bm = dims[c][0], bn = dims[c][1];
    int64_t tiles = 0;
    for (int k = 0; k < count; ++k) tiles += (int64_t)((p[k].M + bm - 1) / bm) * ((p[k].N + bn - 1) / bn);
    const bool pairs = c == 3 || (c == 2 && !dual);   // a form with two blocks per CU exists
    const double rounds = (pairs && tiles > 256) ? 1.3 * (double)((tiles + 511) / 512) : (double)((tiles + 255) / 256);
    const double ingest = 5.12 * (bm + nb * bn), mfma = bm * bn * nb / 22.0;
    const double cost = rounds * (ingest > mfma ? ingest : mfma) * (1.0 + 0.05 * c);
    if (c == 0 || cost < best_cost) { best = c; best_cost = cost; best_tiles = tiles; }
  }
  if (dual) return best == 3 ? (best_tiles <= 256 ? 15 : 14) : 11 + best;
  if (best == 2) return best_tiles <= 256 ? 7 : 3;
  if (best == 3) return best_tiles <= 256 ? 6 : 4;
  return 1 + best;
}

template <bool A_KC, bool B_KC>
void launch_class(ProfScope& ps, hipStream_t st, const GemmBf16Args* p, int count) {
  const bool dual = p[0].B2 != nullptr;
  int shape = g_force_shape;
  if (shape >= 11 && !dual) shape = 0;   // DUAL tiles read B2
  if (shape == 0) shape = pick_tile(p, count, dual);
  switch (shape) {
    case 1: launch_tile<TL, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 2: launch_tile<TM, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 4: launch_tile<TX, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 5: launch_tile<TX4, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 6: launch_tile<TX8, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 7: launch_tile<TS8, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 11: launch_tile<DL, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 12: launch_tile<DM, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 13: launch_tile<DS, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 14: launch_tile<DX, A_KC, B_KC>(ps, st, p, count, g_group); break;
    case 15: launch_tile<DX4, A_KC, B_KC>(ps, st, p, count, g_group); break;
    default: launch_tile<TS, A_KC, B_KC>(ps, st, p, count, g_group); break;
  }
}
}  // namespace

const char* check_gemm_bf16(const GemmBf16Args& a) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return "empty GEMM";
  if (a.K % 64 != 0) return "K must be a multiple of 64";
  if (a.M % 8 != 0 || a.N % 8 != 0) return "M and N must be multiples of 8";
  if (a.lda % 8 != 0 || a.ldb % 8 != 0 || a.ldc % 4 != 0) return "leading dimensions must be multiples of 8 (A, B) and 4 (C)";
  if (((uintptr_t)a.A | (uintptr_t)a.B | (uintptr_t)a.B2 | (uintptr_t)a.bias | (uintptr_t)a.bias_v | (uintptr_t)a.C32 |
       (uintptr_t)a.res32) & 15) return "operands, bias, fp32 residual and fp32 output must be 16-byte aligned";
  if (((uintptr_t)a.C16 | (uintptr_t)a.C16_pre | (uintptr_t)a.aux16 | (uintptr_t)a.res16) & 7) return "bf16 epilogue tensors must be 8-byte aligned";
  if (a.lda < (a.a_trans ? a.M : a.K) || a.ldb < (a.b_trans ? a.K : a.N) || a.ldc < a.N) return "leading dimension too small";
  const int64_t abytes = (int64_t)(a.a_trans ? a.K : a.M) * a.lda * 2, bbytes = (int64_t)(a.b_trans ? a.N : a.K) * a.ldb * 2;
  if (abytes >= ((int64_t)1 << 31) || bbytes >= ((int64_t)1 << 31)) return "operands must be smaller than 2 GiB";
  return nullptr;
}

void gemm_bf16_force_shape(int s) { g_force_shape = s % 100; g_group = s >= 100 ? s / 100 : 8; }

const char* check_gemm_bf16_batch(const GemmBf16Args* p, int count) {
  if (count < 1 || count > GEMM_MAX_BATCH) return "batch of 1 to 4 problems";
  for (int k = 0; k < count; ++k) {
    if (const char* e = check_gemm_bf16(p[k])) return e;
    if (p[k].a_trans != p[0].a_trans || p[k].b_trans != p[0].b_trans || (p[k].B2 != nullptr) != (p[0].B2 != nullptr))
      return "the problems of a batch must share operand storage and the hi + lo form";
  }
  return nullptr;
}

static const char* g_launch_error = nullptr;
void note_launch_error(const char* what) { if (g_launch_error == nullptr) g_launch_error = what; }
const char* take_launch_error() { const char* e = g_launch_error; g_launch_error = nullptr; return e; }

void launch_gemm_bf16_batch(hipStream_t st, const GemmBf16Args* p, int count) {
  if (const char* e = check_gemm_bf16_batch(p, count)) { note_launch_error(e); return; }   // never run a shape the tiles cannot cover
  double flops = 0.0;
  for (int k = 0; k < count; ++k) flops += 2.0 * p[k].M * p[k].N * p[k].K * (p[k].B2 ? 2.0 : 1.0);   // hi + lo contracts over 2K
  const bool hilo = p[0].B2 != nullptr;
  ProfScope ps(st, p[0].a_trans ? F_GEMM_TN : (p[0].b_trans ? (hilo ? F_GEMM_NT_HILO : F_GEMM_NT) : (hilo ? F_GEMM_NN_HILO : F_GEMM_NN)), flops);
  // a_trans = 0: A is [M][K], contraction contiguous.  b_trans = 1: B is [N][K], contraction contiguous.
  if (!p[0].a_trans && p[0].b_trans) launch_class<true, true>(ps, st, p, count);
  else if (!p[0].a_trans && !p[0].b_trans) launch_class<true, false>(ps, st, p, count);
  else if (p[0].a_trans && !p[0].b_trans) launch_class<false, false>(ps, st, p, count);
  else launch_class<false, true>(ps, st, p, count);
}

void launch_gemm_bf16(hipStream_t st, const GemmBf16Args& a) { launch_gemm_bf16_batch(st, &a, 1); }

}  // namespace sama
