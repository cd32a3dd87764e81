// Kernel-level C entry points (include/rrfp_kernels.h): thin argument checks around the
// launchers the stage tasks use.
#include "../../include/rrfp_kernels.h"
#include "../../include/rrfp_stage.h"
#include "kernels.h"

using namespace rrfp;

extern "C" int rrfp_gemm(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                         int ldc, int ldr, int trans_a, int trans_b, int in_dtype, int out_dtype, int family,
                         void* stream) {
  return rrfp_gemm_ws(A, B, C, R, M, N, K, lda, ldb, ldc, ldr, trans_a, trans_b, in_dtype, out_dtype, family, nullptr, 0, stream);
}

extern "C" int rrfp_gemm_ws(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                            int ldc, int ldr, int trans_a, int trans_b, int in_dtype, int out_dtype, int family,
                            void* workspace, size_t workspace_bytes, void* stream) {
  if (!A || !B || !C || M < 1 || N < 1 || K < 1) return STAGE_EINVAL;
  if (workspace && ((uintptr_t)workspace & 255)) return STAGE_EINVAL;
  if (in_dtype != F32 && in_dtype != BF16) return STAGE_EINVAL;
  if (out_dtype != F32 && !(out_dtype == BF16 && in_dtype == BF16)) return STAGE_EINVAL;
  if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N || (R && ldr < N)) return STAGE_EINVAL;
  GemmArgs g{};
  g.A = A; g.B = B; g.C = C; g.R = (const float*)R; g.M = M; g.N = N; g.K = K;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.ldr = ldr;
  g.transA = trans_a != 0; g.transB = trans_b != 0; g.in_dtype = in_dtype; g.out_dtype = out_dtype;
  g.ws = workspace; g.ws_bytes = workspace ? workspace_bytes : 0;
  hipError_t e;
  if (family == RRFP_GEMM_AUTO) e = launch_gemm(g, (hipStream_t)stream);
  else if (family == RRFP_GEMM_SIMT) e = launch_gemm_simt(g, (hipStream_t)stream);
  else if (family == RRFP_GEMM_MFMA) {
    if (!gemm_mfma_supports(g)) return STAGE_EINVAL;
    e = launch_gemm_mfma(g, (hipStream_t)stream);
  } else return STAGE_EINVAL;
  return e == hipSuccess ? STAGE_OK : STAGE_EHIP;
}

extern "C" int rrfp_gemm_plan(int M, int N, int K, int lda, int ldb, int ldc, int trans_a, int trans_b, int out_dtype,
                              int have_scratch, int n_cu, int32_t out[5]) {
  if (!out || M < 1 || N < 1 || K < 1 || n_cu < 1) return STAGE_EINVAL;
  if (out_dtype != F32 && out_dtype != BF16) return STAGE_EINVAL;
  GemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.ldr = ldc;
  g.transA = trans_a != 0; g.transB = trans_b != 0; g.in_dtype = BF16; g.out_dtype = out_dtype;
  const GemmPlan p = gemm_mfma_plan(g, n_cu, have_scratch != 0);
  out[0] = p.kernel; out[1] = p.wavefronts; out[2] = p.main_workgroups; out[3] = p.short_workgroups; out[4] = p.split_k;
  return STAGE_OK;
}

extern "C" int rrfp_rmsnorm_fwd(const float* x, const void* g, void* h, float* r_out, int T, int H, float eps, int dtype,
                                void* stream) {
  if (!x || !g || !h || !r_out || T < 1 || H < 1 || !(eps >= 0.0f)) return STAGE_EINVAL;
  if (dtype != F32 && dtype != BF16) return STAGE_EINVAL;
  return launch_rmsnorm_fwd(x, g, h, r_out, T, H, eps, dtype, (hipStream_t)stream) == hipSuccess ? STAGE_OK : STAGE_EHIP;
}

extern "C" int rrfp_attn_dkv_subsets(int n_q_heads, int n_kv_heads, int n_kv_tiles, int n_cu) {
  if (n_q_heads < 1 || n_kv_heads < 1 || n_kv_tiles < 1 || n_cu < 1 || n_q_heads % n_kv_heads) return STAGE_EINVAL;
  return attn_dkv_subsets(n_q_heads, n_kv_heads, n_kv_tiles, n_cu);
}

extern "C" size_t rrfp_rmsnorm_bwd_workspace(int T, int H, int dtype) {
  if (T < 1 || H < 1 || (dtype != F32 && dtype != BF16)) return 0;
  return (size_t)norm_bwd_partials(T, H, dtype) * (size_t)H * sizeof(float);
}

extern "C" int rrfp_rmsnorm_bwd(const float* dh, const float* x, const float* r, const void* g, const float* add_in,
                                float* out32, void* out_t, float* dg, void* workspace, size_t workspace_bytes, int T, int H,
                                int dtype, void* stream) {
  if (!dh || !x || !r || !g || !add_in || !dg || !workspace || T < 1 || H < 1) return STAGE_EINVAL;
  if (dtype != F32 && dtype != BF16) return STAGE_EINVAL;
  if (workspace_bytes < rrfp_rmsnorm_bwd_workspace(T, H, dtype) || ((uintptr_t)workspace & 15)) return STAGE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (launch_rmsnorm_bwd(dh, x, r, g, add_in, out32, out_t, (float*)workspace, T, H, dtype, s) != hipSuccess) return STAGE_EHIP;
  if (launch_colsum((const float*)workspace, norm_bwd_partials(T, H, dtype), H, dg, s) != hipSuccess) return STAGE_EHIP;
  return STAGE_OK;
}

extern "C" int rrfp_grad_reduce(const float* slots, size_t slot_stride, int M, float* out, size_t n, void* stream) {
  if (!slots || !out || M < 1 || n < 1 || (n & 3) || (slot_stride & 3) || (M > 1 && slot_stride < n)) return STAGE_EINVAL;
  if (((uintptr_t)slots & 15) || ((uintptr_t)out & 15)) return STAGE_EINVAL;
  return launch_grad_reduce(slots, slot_stride, M, out, n, (hipStream_t)stream) == hipSuccess ? STAGE_OK : STAGE_EHIP;
}
