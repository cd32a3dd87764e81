// Plain fp32 attention forward and backward over packed segments (any head_dim that is a
// multiple of 16, up to 128; GQA; causal or bidirectional).  It is the attention of the fp32
// path.  Work items are the row tiles the host carved inside each segment.  No atomics: the
// dK/dV kernel owns a key tile and walks the query heads of its group and the query rows in
// ascending order; the dQ kernel owns a query tile and walks the keys in ascending order.
#include "kernels.h"
#include "numeric.h"

namespace rrfp {
namespace {

constexpr int SUBQ = 32;    // query rows per pass
constexpr int SUBK = 16;    // keys per pass
constexpr int DMAX = 128;

template <typename T>
__device__ inline void load_rows(float* dst, const T* src, int ld, int row0, int row_end, int rows, int col0, int d) {
  // dst [rows][DMAX]; rows beyond row_end are zero-filled
  for (int idx = threadIdx.x; idx < rows * d; idx += 256) {
    const int r = idx / d, c = idx - r * d;
    const int gr = row0 + r;
    dst[r * DMAX + c] = gr < row_end ? to_float(src[(size_t)gr * ld + col0 + c]) : 0.f;
  }
}

// ------------------------------------------------------------------------- forward
template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simt_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                            float* __restrict__ lse, const AttnTile* __restrict__ tiles,
                                                            int Tn, int nq, int nkv, int d, int causal) {
  __shared__ float Qs[SUBQ * DMAX];
  __shared__ float Ks[SUBK * DMAX];
  __shared__ float Vs[SUBK * DMAX];
  __shared__ float Ps[SUBQ][SUBK + 1];
  const AttnTile tl = tiles[blockIdx.x];
  const int a = blockIdx.y, b = a / (nq / nkv);
  const int ld = (nq + 2 * nkv) * d;
  const int qcol = a * d, kcol = (nq + b) * d, vcol = (nq + nkv + b) * d;
  const float scale = 1.0f / sqrtf((float)d);
  const int tr = threadIdx.x >> 3;       // row inside the pass, 0..31
  const int tq = threadIdx.x & 7;        // 8 threads share a row
  const int ncol = d / 8;                // output columns per thread: tq + 8 * cc

  for (int q0 = tl.r0; q0 < tl.r1; q0 += SUBQ) {
    const int q_end = min(q0 + SUBQ, tl.r1);
    __syncthreads();
    load_rows<T>(Qs, qkv, ld, q0, q_end, SUBQ, qcol, d);
    float m_run = -INFINITY, l_run = 0.f;
    float acc[DMAX / 8];
#pragma unroll
    for (int cc = 0; cc < DMAX / 8; ++cc) acc[cc] = 0.f;
    const int i = q0 + tr;
    const int k_end = causal ? q_end : tl.s1;
    for (int k0 = tl.s0; k0 < k_end; k0 += SUBK) {
      __syncthreads();
      load_rows<T>(Ks, qkv, ld, k0, k_end, SUBK, kcol, d);
      load_rows<T>(Vs, qkv, ld, k0, k_end, SUBK, vcol, d);
      __syncthreads();
      float sc[2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int jl = tq * 2 + jj, j = k0 + jl;
        float dot = 0.f;
        for (int c = 0; c < d; ++c) dot = fmaf(Qs[tr * DMAX + c], Ks[jl * DMAX + c], dot);
        const bool ok = (i < q_end) && (j < k_end) && (!causal || j <= i);
        sc[jj] = ok ? dot * scale : -INFINITY;
      }
      float mx = fmaxf(sc[0], sc[1]);
#pragma unroll
      for (int off = 1; off < 8; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      const float m_new = fmaxf(m_run, mx);
      float p[2], ps = 0.f;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        p[jj] = (sc[jj] == -INFINITY) ? 0.f : __expf(sc[jj] - m_new);
        ps += p[jj];
        Ps[tr][tq * 2 + jj] = p[jj];
      }
#pragma unroll
      for (int off = 1; off < 8; off <<= 1) ps += __shfl_xor(ps, off, 64);
      const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
      l_run = l_run * alpha + ps;
      m_run = m_new;
      __syncthreads();
      for (int cc = 0; cc < ncol; ++cc) {
        const int c = tq + 8 * cc;
        float v = acc[cc] * alpha;
#pragma unroll
        for (int jl = 0; jl < SUBK; ++jl) v = fmaf(Ps[tr][jl], Vs[jl * DMAX + c], v);
        acc[cc] = v;
      }
    }
    if (i < q_end) {
      const float inv = 1.0f / l_run;
      for (int cc = 0; cc < ncol; ++cc) o[(size_t)i * nq * d + qcol + tq + 8 * cc] = from_float<T>(acc[cc] * inv);
      if (tq == 0) lse[(size_t)a * Tn + i] = m_run + __logf(l_run);
    }
  }
}

// ------------------------------------------------------------------------- delta = rowsum(dO * O)
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ o, const T* __restrict__ d_o,
                                                         float* __restrict__ delta, int Tn, int nq, int d) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= Tn * nq) return;
  const int i = idx / nq, a = idx - i * nq;
  const size_t off = (size_t)i * nq * d + (size_t)a * d;
  float s = 0.f;
  for (int c = 0; c < d; ++c) s = fmaf(to_float(o[off + c]), to_float(d_o[off + c]), s);
  delta[(size_t)a * Tn + i] = s;
}

// Scores, probabilities and score gradients of a (SUBQ x SUBK) patch into LDS.
__device__ inline void patch_p_ds(const float* Qs, const float* Ks, const float* Vs, const float* dOs,
                                  float (*Ps)[SUBK + 1], float (*dSs)[SUBK + 1], const float* lse_s,
                                  const float* delta_s, int q0, int q_end, int k0, int k_end, int d, float scale,
                                  int causal) {
  const int tr = threadIdx.x >> 3, tq = threadIdx.x & 7;
  const int i = q0 + tr;
#pragma unroll
  for (int jj = 0; jj < 2; ++jj) {
    const int jl = tq * 2 + jj, j = k0 + jl;
    float dot = 0.f, dp = 0.f;
    for (int c = 0; c < d; ++c) {
      dot = fmaf(Qs[tr * DMAX + c], Ks[jl * DMAX + c], dot);
      dp = fmaf(dOs[tr * DMAX + c], Vs[jl * DMAX + c], dp);
    }
    const bool ok = (i < q_end) && (j < k_end) && (!causal || j <= i);
    const float p = ok ? __expf(dot * scale - lse_s[tr]) : 0.f;
    Ps[tr][jl] = p;
    dSs[tr][jl] = p * (dp - delta_s[tr]);
  }
}

// ------------------------------------------------------------------------- dQ
template <typename T>
__global__ __launch_bounds__(256) void attn_dq_simt_kernel(const T* __restrict__ qkv, const T* __restrict__ d_o,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           T* __restrict__ dqkv, const AttnTile* __restrict__ tiles,
                                                           int Tn, int nq, int nkv, int d, int causal) {
  __shared__ float Qs[SUBQ * DMAX];
  __shared__ float dOs[SUBQ * DMAX];
  __shared__ float Ks[SUBK * DMAX];
  __shared__ float Vs[SUBK * DMAX];
  __shared__ float Ps[SUBQ][SUBK + 1];
  __shared__ float dSs[SUBQ][SUBK + 1];
  __shared__ float lse_s[SUBQ], delta_s[SUBQ];
  const AttnTile tl = tiles[blockIdx.x];
  const int a = blockIdx.y, b = a / (nq / nkv);
  const int ld = (nq + 2 * nkv) * d;
  const int qcol = a * d, kcol = (nq + b) * d, vcol = (nq + nkv + b) * d;
  const float scale = 1.0f / sqrtf((float)d);
  const int tr = threadIdx.x >> 3, tq = threadIdx.x & 7;
  const int ncol = d / 8;
  for (int q0 = tl.r0; q0 < tl.r1; q0 += SUBQ) {
    const int q_end = min(q0 + SUBQ, tl.r1);
    __syncthreads();
    load_rows<T>(Qs, qkv, ld, q0, q_end, SUBQ, qcol, d);
    load_rows<T>(dOs, d_o, nq * d, q0, q_end, SUBQ, qcol, d);
    if (threadIdx.x < SUBQ) {
      const int i = q0 + threadIdx.x;
      lse_s[threadIdx.x] = i < q_end ? lse[(size_t)a * Tn + i] : 0.f;
      delta_s[threadIdx.x] = i < q_end ? delta[(size_t)a * Tn + i] : 0.f;
    }
    float acc[DMAX / 8];
#pragma unroll
    for (int cc = 0; cc < DMAX / 8; ++cc) acc[cc] = 0.f;
    const int k_end = causal ? q_end : tl.s1;
    for (int k0 = tl.s0; k0 < k_end; k0 += SUBK) {
      __syncthreads();
      load_rows<T>(Ks, qkv, ld, k0, k_end, SUBK, kcol, d);
      load_rows<T>(Vs, qkv, ld, k0, k_end, SUBK, vcol, d);
      __syncthreads();
      patch_p_ds(Qs, Ks, Vs, dOs, Ps, dSs, lse_s, delta_s, q0, q_end, k0, k_end, d, scale, causal);
      __syncthreads();
      for (int cc = 0; cc < ncol; ++cc) {
        const int c = tq + 8 * cc;
        float v = acc[cc];
#pragma unroll
        for (int jl = 0; jl < SUBK; ++jl) v = fmaf(dSs[tr][jl], Ks[jl * DMAX + c], v);
        acc[cc] = v;
      }
    }
    const int i = q0 + tr;
    if (i < q_end)
      for (int cc = 0; cc < ncol; ++cc) dqkv[(size_t)i * ld + qcol + tq + 8 * cc] = from_float<T>(acc[cc] * scale);
  }
}

// ------------------------------------------------------------------------- dK, dV
template <typename T>
__global__ __launch_bounds__(256) void attn_dkv_simt_kernel(const T* __restrict__ qkv, const T* __restrict__ d_o,
                                                            const float* __restrict__ lse, const float* __restrict__ delta,
                                                            T* __restrict__ dqkv, const AttnTile* __restrict__ tiles,
                                                            int Tn, int nq, int nkv, int d, int causal) {
  __shared__ float Qs[SUBQ * DMAX];
  __shared__ float dOs[SUBQ * DMAX];
  __shared__ float Ks[SUBK * DMAX];
  __shared__ float Vs[SUBK * DMAX];
  __shared__ float Ps[SUBQ][SUBK + 1];
  __shared__ float dSs[SUBQ][SUBK + 1];
  __shared__ float lse_s[SUBQ], delta_s[SUBQ];
  const AttnTile tl = tiles[blockIdx.x];
  const int b = blockIdx.y, G = nq / nkv;
  const int ld = (nq + 2 * nkv) * d;
  const int kcol = (nq + b) * d, vcol = (nq + nkv + b) * d;
  const float scale = 1.0f / sqrtf((float)d);
  const int tj = threadIdx.x >> 4;       // key inside the pass, 0..15
  const int tc = threadIdx.x & 15;       // columns tc + 16 * cc
  const int ncol = d / 16;
  for (int k0 = tl.r0; k0 < tl.r1; k0 += SUBK) {
    const int k_end = min(k0 + SUBK, tl.r1);
    __syncthreads();
    load_rows<T>(Ks, qkv, ld, k0, k_end, SUBK, kcol, d);
    load_rows<T>(Vs, qkv, ld, k0, k_end, SUBK, vcol, d);
    float dk[DMAX / 16], dv[DMAX / 16];
#pragma unroll
    for (int cc = 0; cc < DMAX / 16; ++cc) { dk[cc] = 0.f; dv[cc] = 0.f; }
    const int q_begin = causal ? k0 : tl.s0;
    for (int a = b * G; a < (b + 1) * G; ++a) {
      const int qcol = a * d;
      for (int q0 = q_begin; q0 < tl.s1; q0 += SUBQ) {
        const int q_end = min(q0 + SUBQ, tl.s1);
        __syncthreads();
        load_rows<T>(Qs, qkv, ld, q0, q_end, SUBQ, qcol, d);
        load_rows<T>(dOs, d_o, nq * d, q0, q_end, SUBQ, qcol, d);
        if (threadIdx.x < SUBQ) {
          const int i = q0 + threadIdx.x;
          lse_s[threadIdx.x] = i < q_end ? lse[(size_t)a * Tn + i] : 0.f;
          delta_s[threadIdx.x] = i < q_end ? delta[(size_t)a * Tn + i] : 0.f;
        }
        __syncthreads();
        patch_p_ds(Qs, Ks, Vs, dOs, Ps, dSs, lse_s, delta_s, q0, q_end, k0, k_end, d, scale, causal);
        __syncthreads();
        for (int cc = 0; cc < ncol; ++cc) {
          const int c = tc + 16 * cc;
          float vk = dk[cc], vv = dv[cc];
#pragma unroll
          for (int il = 0; il < SUBQ; ++il) {
            vk = fmaf(dSs[il][tj], Qs[il * DMAX + c], vk);
            vv = fmaf(Ps[il][tj], dOs[il * DMAX + c], vv);
          }
          dk[cc] = vk; dv[cc] = vv;
        }
      }
    }
    const int j = k0 + tj;
    if (j < k_end)
      for (int cc = 0; cc < ncol; ++cc) {
        dqkv[(size_t)j * ld + kcol + tc + 16 * cc] = from_float<T>(dk[cc] * scale);
        dqkv[(size_t)j * ld + vcol + tc + 16 * cc] = from_float<T>(dv[cc]);
      }
  }
}

template <typename T>
hipError_t fwd_typed(const AttnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(attn_fwd_simt_kernel<T>, dim3(a.n_q_tiles, a.nq), dim3(256), 0, s, (const T*)a.qkv, (T*)a.o, a.lse,
                     a.q_tiles, a.T, a.nq, a.nkv, a.d, a.causal);
  return hipGetLastError();
}

template <typename T>
hipError_t bwd_typed(const AttnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(attn_delta_kernel<T>, dim3((a.T * a.nq + 255) / 256), dim3(256), 0, s, (const T*)a.o,
                     (const T*)a.d_o, a.delta, a.T, a.nq, a.d);
  hipLaunchKernelGGL(attn_dkv_simt_kernel<T>, dim3(a.n_kv_tiles, a.nkv), dim3(256), 0, s, (const T*)a.qkv,
                     (const T*)a.d_o, a.lse, a.delta, (T*)a.dqkv, a.kv_tiles, a.T, a.nq, a.nkv, a.d, a.causal);
  hipLaunchKernelGGL(attn_dq_simt_kernel<T>, dim3(a.n_q_tiles, a.nq), dim3(256), 0, s, (const T*)a.qkv,
                     (const T*)a.d_o, a.lse, a.delta, (T*)a.dqkv, a.q_tiles, a.T, a.nq, a.nkv, a.d, a.causal);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_fwd_simt(const AttnArgs& a, hipStream_t s) {
  if (a.d % 16 || a.d > DMAX || a.n_q_tiles < 1) return hipErrorInvalidValue;
  return a.dtype == F32 ? fwd_typed<float>(a, s) : fwd_typed<bf16_t>(a, s);
}

hipError_t launch_attn_bwd_simt(const AttnArgs& a, hipStream_t s) {
  if (a.d % 16 || a.d > DMAX || a.n_q_tiles < 1 || a.n_kv_tiles < 1) return hipErrorInvalidValue;
  return a.dtype == F32 ? bwd_typed<float>(a, s) : bwd_typed<bf16_t>(a, s);
}

}  // namespace rrfp
