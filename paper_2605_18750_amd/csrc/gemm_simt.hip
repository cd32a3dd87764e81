// Plain LDS-tiled fp32-FMA GEMM for any shape, stride and operand orientation.  It is the
// GEMM of the fp32 path and of bf16 shapes the MFMA kernels do not take.  The k loop runs
// in ascending order in one thread per output element: one fixed summation order.
#include "kernels.h"
#include "numeric.h"

namespace rrfp {
namespace {

template <typename TI, typename TO, bool TA, bool TB, bool HAS_R>
__global__ __launch_bounds__(256) void gemm_simt_kernel(const TI* __restrict__ A, const TI* __restrict__ B,
                                                        TO* __restrict__ C, const float* __restrict__ R, int M, int N,
                                                        int K, int lda, int ldb, int ldc, int ldr,
                                                        const TI* __restrict__ bias) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = threadIdx.x + i * 256;
      int m, k;
      if (!TA) { k = idx & 15; m = idx >> 4; } else { m = idx & 63; k = idx >> 6; }
      const int gm = m0 + m, gk = k0 + k;
      float v = 0.f;
      if (gm < M && gk < K) v = to_float(TA ? A[(size_t)gk * lda + gm] : A[(size_t)gm * lda + gk]);
      As[k][m] = v;
      int n, kb;
      if (!TB) { n = idx & 63; kb = idx >> 6; } else { kb = idx & 15; n = idx >> 4; }
      const int gn = n0 + n, gkb = k0 + kb;
      float w = 0.f;
      if (gn < N && gkb < K) w = to_float(TB ? B[(size_t)gn * ldb + gkb] : B[(size_t)gkb * ldb + gn]);
      Bs[kb][n] = w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      float v = acc[i][j];
      if (bias) v += to_float(bias[gn]);
      if (HAS_R) v += R[(size_t)gm * ldr + gn];
      C[(size_t)gm * ldc + gn] = from_float<TO>(v);
    }
  }
}

template <typename TI, typename TO>
hipError_t launch_typed(const GemmArgs& g, hipStream_t s) {
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
#define GO(TA, TB, HR)                                                                                     \
  hipLaunchKernelGGL((gemm_simt_kernel<TI, TO, TA, TB, HR>), grid, block, 0, s, (const TI*)g.A, (const TI*)g.B, \
                     (TO*)g.C, g.R, g.M, g.N, g.K, g.lda, g.ldb, g.ldc, g.ldr, (const TI*)g.bias)
  const bool hr = g.R != nullptr;
  if (!g.transA && !g.transB) { if (hr) GO(false, false, true); else GO(false, false, false); }
  else if (!g.transA && g.transB) { if (hr) GO(false, true, true); else GO(false, true, false); }
  else if (g.transA && !g.transB) { if (hr) GO(true, false, true); else GO(true, false, false); }
  else { if (hr) GO(true, true, true); else GO(true, true, false); }
#undef GO
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_simt(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if (g.in_dtype == F32 && g.out_dtype == F32) return launch_typed<float, float>(g, s);
  if (g.in_dtype == BF16 && g.out_dtype == BF16) return launch_typed<bf16_t, bf16_t>(g, s);
  if (g.in_dtype == BF16 && g.out_dtype == F32) return launch_typed<bf16_t, float>(g, s);
  return hipErrorInvalidValue;
}

}  // namespace rrfp
