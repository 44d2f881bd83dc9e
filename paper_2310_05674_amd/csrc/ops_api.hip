// Op-level C entry points (include/sama_ops.h): thin argument checks around the kernel launchers.
#include <math.h>
#include <mutex>
#include <string>
#include "../../include/sama_ops.h"
#include "kernels.h"

using namespace sama;

// Scratch of sama_op_adapt_norm_static: the per-block partial sums of ||v||^2 that sama_op_adapt_norm takes from its
// caller.  One copy per GPU the library runs on, alive until the process ends; host code never uses the array's name
// as an address, only the per-device pointers resolved below.
static __device__ __align__(256) double scratch[EW_MAX_BLOCKS];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[MAX_DEVICES] = {};   // device address of `scratch` on each GPU, resolved at the first call there
thread_local std::string g_ops_error;

// The current device's copy of `scratch`; null (and g_ops_error set) if it cannot be resolved.
double* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) { g_ops_error = "no current HIP device (or device index above 63)"; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    double* p = nullptr;
    const hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) { g_ops_error = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e); return nullptr; }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

// Diagnostic switches (include/sama_ops.h): block shape of the bf16 GEMM, 0 = heuristic.
void sama_dev_gemm_shape(int32_t shape) { gemm_bf16_force_shape(shape); }
// 0 keeps every launch of the encoder's backward pass on the context's stream / makes the optimizer slices wait for its end.
void sama_dev_side_stream(int32_t on) { encoder_side_stream(on != 0); }
void sama_dev_side_sink(int32_t on) { encoder_side_sink(on != 0); }

sama_status sama_op_gemm_bf16(const void* A, int64_t lda, int32_t a_trans, const void* B, const void* B2, int64_t ldb,
                              int32_t b_trans, int32_t M, int32_t N, int32_t K, const float* bias, float* C32, void* C16,
                              int64_t ldc, void* hip_stream) {
  if (!A || !B || (!C32 && !C16)) return SAMA_EINVAL;
  GemmBf16Args g{};
  g.A = (const bf16_t*)A; g.lda = lda; g.a_trans = a_trans ? 1 : 0;
  g.B = (const bf16_t*)B; g.B2 = (const bf16_t*)B2; g.ldb = ldb; g.b_trans = b_trans ? 1 : 0;
  g.M = M; g.N = N; g.K = K; g.ldc = ldc; g.bias = bias; g.C32 = C32; g.C16 = (bf16_t*)C16;
  if (check_gemm_bf16(g) != nullptr) return SAMA_EINVAL;
  (void)hipGetLastError();
  launch_gemm_bf16((hipStream_t)hip_stream, g);
  return hipGetLastError() == hipSuccess ? SAMA_OK : SAMA_EHIP;
}

sama_status sama_op_gemm_bf16_batch(int32_t count, const void* const* A, const void* const* B, const void* const* B2,
                                    float* const* C32, const int32_t* M, const int32_t* N, const int32_t* K, int32_t a_trans,
                                    int32_t b_trans, void* hip_stream) {
  if (count < 1 || count > GEMM_MAX_BATCH || !A || !B || !C32 || !M || !N || !K) return SAMA_EINVAL;
  GemmBf16Args g[GEMM_MAX_BATCH];
  for (int k = 0; k < count; ++k) {
    if (!A[k] || !B[k] || !C32[k] || (B2 && !B2[k])) return SAMA_EINVAL;
    g[k] = GemmBf16Args{};
    g[k].A = (const bf16_t*)A[k]; g[k].a_trans = a_trans ? 1 : 0; g[k].lda = a_trans ? M[k] : K[k];
    g[k].B = (const bf16_t*)B[k]; g[k].B2 = B2 ? (const bf16_t*)B2[k] : nullptr; g[k].b_trans = b_trans ? 1 : 0;
    g[k].ldb = b_trans ? K[k] : N[k];
    g[k].M = M[k]; g[k].N = N[k]; g[k].K = K[k]; g[k].ldc = N[k]; g[k].C32 = C32[k];
  }
  if (check_gemm_bf16_batch(g, count) != nullptr) return SAMA_EINVAL;
  (void)hipGetLastError();
  launch_gemm_bf16_batch((hipStream_t)hip_stream, g, count);
  return hipGetLastError() == hipSuccess ? SAMA_OK : SAMA_EHIP;
}

sama_status sama_op_adam(float* g, float* m, float* v, float* theta, void* theta16, int64_t n, int64_t n16, int64_t t,
                         float lr, float beta1, float beta2, float eps, float weight_decay, void* hip_stream) {
  if (!g || !m || !v || !theta || n < 0 || n16 < 0 || n16 > n || t < 1) return SAMA_EINVAL;
  if (((uintptr_t)g | (uintptr_t)m | (uintptr_t)v | (uintptr_t)theta) & 15 || ((uintptr_t)theta16 & 7)) return SAMA_EINVAL;
  AdamArgs a{};
  a.beta1 = beta1; a.one_m_beta1 = (float)(1.0 - (double)beta1); a.beta2 = beta2; a.one_m_beta2 = (float)(1.0 - (double)beta2);
  a.lr_c1 = (float)((double)lr / (1.0 - pow((double)beta1, (double)t)));
  a.c2 = (float)(1.0 / sqrt(1.0 - pow((double)beta2, (double)t)));
  a.eps = eps; a.weight_decay = weight_decay;
  (void)hipGetLastError();
  launch_adam((hipStream_t)hip_stream, g, m, v, theta, (bf16_t*)theta16, n, theta16 ? n16 : 0, a);
  return hipGetLastError() == hipSuccess ? SAMA_OK : SAMA_EHIP;
}

sama_status sama_op_adapt_norm(const float* g, const float* m, const float* v, const float* gmeta, float* vdir, double* partial,
                               int64_t n, int64_t t, float lr, float beta1, float beta2, float eps, float alpha, float* scalars,
                               int64_t* status, void* hip_stream) {
  if (!g || !m || !v || !gmeta || !vdir || !partial || !scalars || !status || n < 1 || t < 1) return SAMA_EINVAL;
  if (((uintptr_t)g | (uintptr_t)m | (uintptr_t)v | (uintptr_t)gmeta | (uintptr_t)vdir) & 15) return SAMA_EINVAL;
  const double c1 = 1.0 / (1.0 - pow((double)beta1, (double)t)), c2 = 1.0 / sqrt(1.0 - pow((double)beta2, (double)t));
  AdaptArgs ad{};
  ad.mode = 0; ad.one_m_beta1 = (float)(1.0 - (double)beta1); ad.one_m_beta2 = (float)(1.0 - (double)beta2);
  ad.lr_c1_c2 = (float)((double)lr * c1 * c2); ad.c2 = (float)c2; ad.eps = eps;
  (void)hipGetLastError();
  launch_adapt_norm((hipStream_t)hip_stream, g, m, v, gmeta, vdir, partial, n, ad, alpha, scalars, status);
  return hipGetLastError() == hipSuccess ? SAMA_OK : SAMA_EHIP;
}

sama_status sama_op_adapt_norm_static(const float* g, const float* m, const float* v, const float* gmeta, float* vdir, int64_t n,
                                      int64_t t, float lr, float beta1, float beta2, float eps, float alpha, float* scalars,
                                      int64_t* status, void* hip_stream) {
  g_ops_error.clear();
  if (n > SAMA_OP_STATIC_MAX_N) {
    g_ops_error = "sama_op_adapt_norm_static: n exceeds SAMA_OP_STATIC_MAX_N (2^29 elements); use sama_op_adapt_norm with a caller-owned scratch";
    return SAMA_EINVAL;
  }
  double* partial = static_scratch();
  if (partial == nullptr) return SAMA_EHIP;
  const sama_status s = sama_op_adapt_norm(g, m, v, gmeta, vdir, partial, n, t, lr, beta1, beta2, eps, alpha, scalars, status, hip_stream);
  if (s == SAMA_EINVAL) g_ops_error = "sama_op_adapt_norm_static: null or misaligned pointer, n < 1 or t < 1";
  return s;
}

const char* sama_op_last_error(void) { return g_ops_error.c_str(); }

sama_status sama_op_perturb_lo(const float* theta, const float* vdir, const float* eps_ptr, void* lo_p, void* lo_m, int64_t n16,
                               void* hip_stream) {
  if (!theta || !vdir || !eps_ptr || !lo_p || !lo_m || n16 < 0) return SAMA_EINVAL;
  if ((((uintptr_t)theta | (uintptr_t)vdir) & 15) || (((uintptr_t)lo_p | (uintptr_t)lo_m) & 7)) return SAMA_EINVAL;
  (void)hipGetLastError();
  launch_perturb_lo((hipStream_t)hip_stream, theta, vdir, eps_ptr, (bf16_t*)lo_p, (bf16_t*)lo_m, n16);
  return hipGetLastError() == hipSuccess ? SAMA_OK : SAMA_EHIP;
}

sama_status sama_op_nudge(float* theta, const float* vdir, const float* eps_ptr, void* theta16, int64_t n, int64_t n16,
                          void* hip_stream) {
  if (!theta || !vdir || !eps_ptr || n < 0 || n16 < 0 || n16 > n) return SAMA_EINVAL;
  if ((((uintptr_t)theta | (uintptr_t)vdir) & 15) || ((uintptr_t)theta16 & 7)) return SAMA_EINVAL;
  (void)hipGetLastError();
  launch_nudge((hipStream_t)hip_stream, theta, vdir, eps_ptr, nullptr, (bf16_t*)theta16, nullptr, n, theta16 ? n16 : 0);
  return hipGetLastError() == hipSuccess ? SAMA_OK : SAMA_EHIP;
}

}  // extern "C"
