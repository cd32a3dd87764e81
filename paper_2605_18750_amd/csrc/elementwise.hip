// HBM-bound kernels of the stage tasks: RMSNorm forward/backward, SwiGLU and GELU
// forward/backward, the fixed-order column sum for norm-gain gradients and the
// index-ordered gradient reduction.  All arithmetic is fp32; storage is fp32 or bf16.
// None of these kernels uses atomics: every sum has one fixed order.
#include <algorithm>

#include "kernels.h"
#include "numeric.h"

namespace rrfp {
namespace {

constexpr int WAVE = 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}

// Vec<T>::N consecutive fp32 values (the residual stream is fp32 whatever the storage type).
template <int V>
__device__ inline void load_f32(const float* p, float* out) {
#pragma unroll
  for (int i = 0; i < V; i += 4) {
    const float4 v = *reinterpret_cast<const float4*>(p + i);
    out[i] = v.x; out[i + 1] = v.y; out[i + 2] = v.z; out[i + 3] = v.w;
  }
}
template <int V>
__device__ inline void store_f32(float* p, const float* in) {
#pragma unroll
  for (int i = 0; i < V; i += 4) *reinterpret_cast<float4*>(p + i) = make_float4(in[i], in[i + 1], in[i + 2], in[i + 3]);
}

// ---------------------------------------------------------------- storage type -> fp32 copy
// copy, when given, also receives the values unchanged (one read of src serves both outputs).
template <typename T>
__global__ __launch_bounds__(256) void widen_kernel(const T* __restrict__ src, float* __restrict__ dst, size_t n,
                                                    T* __restrict__ copy) {
  constexpr int V = Vec<T>::N;
  const size_t nv = n / V;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    float v[V];
    load_vec<T>(src + i * V, v);
    store_f32<V>(dst + i * V, v);
    if (copy) store_vec<T>(copy + i * V, v);     // widening and rounding back is the identity
  }
  for (size_t i = nv * V + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    dst[i] = to_float(src[i]);
    if (copy) copy[i] = src[i];
  }
}

// ---------------------------------------------------------------- gradient scale
// max |v| over the tensor in two steps (per-workgroup maxima, then one workgroup): a maximum has no summation
// order, so the result does not depend on how the work was cut.
template <typename T>
__global__ __launch_bounds__(256) void absmax_partial_kernel(const T* __restrict__ src, size_t n, float* __restrict__ partial) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[4];
  float mx = 0.f;
  const size_t nv = n / V;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    float v[V];
    load_vec<T>(src + i * V, v);
#pragma unroll
    for (int e = 0; e < V; ++e) mx = fmaxf(mx, fabsf(v[e]));      // fmaxf drops NaNs: a NaN in dy shows in the results, not here
  }
  for (size_t i = nv * V + (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) mx = fmaxf(mx, fabsf(to_float(src[i])));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, WAVE));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__global__ __launch_bounds__(256) void grad_scale_kernel(const float* __restrict__ partial, int n_partial, float* __restrict__ scale) {
  __shared__ float red[4];
  float mx = 0.f;
  for (int i = threadIdx.x; i < n_partial; i += 256) mx = fmaxf(mx, partial[i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, WAVE));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float s = 1.0f;
    if (mx > 0.f && mx < INFINITY) {
      int ex;
      frexpf(mx, &ex);                               // mx = f * 2^ex, f in [0.5, 1)
      ex = max(-100, min(100, ex - 1));              // 2^ex <= mx < 2^(ex+1)
      s = ldexpf(1.0f, -ex);                         // s * mx in [1, 2)
    }
    scale[0] = s;
    scale[1] = 1.0f / s;                             // exact: s is a power of two
  }
}

// ---------------------------------------------------------------- RMSNorm forward
// One wavefront per row; 4 rows per workgroup.  Two sweeps over the row (the second is
// served by cache): sum of squares, then scale.  x is the fp32 residual stream.
// h16, when given (bf16 storage only), receives the same values rounded to IEEE half: the copy the QKV
// projection reads (the bf16 one then serves the weight-gradient GEMM, whose other operand is a bf16 gradient).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const float* __restrict__ x, const T* __restrict__ g,
                                                          T* __restrict__ h, float* __restrict__ r_out,
                                                          int Tn, int H, float eps, f16_t* __restrict__ h16) {
  constexpr int V = Vec<T>::N;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Tn) return;
  const float* xr = x + (size_t)row * H;
  T* hr = h + (size_t)row * H;
  float ss = 0.f;
  const bool vec = (H % V) == 0;
  if (vec) {
    for (int c = lane * V; c < H; c += WAVE * V) {
      float v[V];
      load_f32<V>(xr + c, v);
#pragma unroll
      for (int i = 0; i < V; ++i) ss += v[i] * v[i];
    }
  } else {
    for (int c = lane; c < H; c += WAVE) { float v = xr[c]; ss += v * v; }
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)H + eps);
  if (lane == 0) r_out[row] = r;
  if (vec) {
    for (int c = lane * V; c < H; c += WAVE * V) {
      float v[V], gv[V];
      load_f32<V>(xr + c, v);
      load_vec<T>(g + c, gv);
#pragma unroll
      for (int i = 0; i < V; ++i) v[i] = v[i] * r * gv[i];
      store_vec<T>(hr + c, v);
      if constexpr (V == 8) {
        if (h16) store_vec<f16_t>(h16 + (size_t)row * H + c, v);
      }
    }
  } else {
    for (int c = lane; c < H; c += WAVE) {
      const float v = xr[c] * r * to_float(g[c]);
      hr[c] = from_float<T>(v);
      if (h16) h16[(size_t)row * H + c] = from_float<f16_t>(v);
    }
  }
}

// The same for rows of up to NV * 64 vectors (H % Vec<T>::N == 0): the row is read once, all its loads issued
// before the first use, and stays in registers between the two sweeps.  Same arithmetic in the same order as the
// kernel above (bit-identical results).
template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_fwd_rows_kernel(const float* __restrict__ x, const T* __restrict__ g,
                                                               T* __restrict__ h, float* __restrict__ r_out,
                                                               int Tn, int H, float eps, f16_t* __restrict__ h16) {
  constexpr int V = Vec<T>::N;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Tn) return;
  const float* xr = x + (size_t)row * H;
  float a[NV][V];
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int c = (v * WAVE + lane) * V;
    if (c < H) load_f32<V>(xr + c, a[v]);
  }
  float ss = 0.f;
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    if ((v * WAVE + lane) * V < H) {
#pragma unroll
      for (int i = 0; i < V; ++i) ss += a[v][i] * a[v][i];
    }
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)H + eps);
  if (lane == 0) r_out[row] = r;
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int c = (v * WAVE + lane) * V;
    if (c < H) {
      float gv[V];
      load_vec<T>(g + c, gv);
#pragma unroll
      for (int i = 0; i < V; ++i) a[v][i] = a[v][i] * r * gv[i];
      store_vec<T>(h + (size_t)row * H + c, a[v]);
      if constexpr (V == 8) {
        if (h16) store_vec<f16_t>(h16 + (size_t)row * H + c, a[v]);
      }
    }
  }
}

// ---------------------------------------------------------------- RMSNorm backward, rows
// dx = add_in + r * (w - xhat * mean(w * xhat)),  w = dh * g,  xhat = x * r.
// dh (a GEMM output consumed only here), x and add_in (residual stream) are fp32.  dx goes to out32 (fp32, next link of the residual-gradient
// chain) and/or out_t (storage type: GEMM operand, or the task's dx output); either may be null.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_bwd_rows_kernel(const float* __restrict__ dh, const float* __restrict__ x,
                                                               const float* __restrict__ r, const T* __restrict__ g,
                                                               const float* __restrict__ add_in, float* __restrict__ out32,
                                                               T* __restrict__ out_t, int Tn, int H) {
  constexpr int V = Vec<T>::N;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Tn) return;
  const size_t off = (size_t)row * H;
  const float rr = r[row];
  float dot = 0.f;
  const bool vec = (H % V) == 0;
  if (vec) {
    for (int c = lane * V; c < H; c += WAVE * V) {
      float a[V], b[V], gv[V];
      load_f32<V>(dh + off + c, a);
      load_f32<V>(x + off + c, b);
      load_vec<T>(g + c, gv);
#pragma unroll
      for (int i = 0; i < V; ++i) dot += a[i] * gv[i] * (b[i] * rr);
    }
  } else {
    for (int c = lane; c < H; c += WAVE) dot += dh[off + c] * to_float(g[c]) * (x[off + c] * rr);
  }
  dot = wave_sum(dot) / (float)H;
  if (vec) {
    for (int c = lane * V; c < H; c += WAVE * V) {
      float a[V], b[V], gv[V], ad[V];
      load_f32<V>(dh + off + c, a);
      load_f32<V>(x + off + c, b);
      load_vec<T>(g + c, gv);
      load_f32<V>(add_in + off + c, ad);
#pragma unroll
      for (int i = 0; i < V; ++i) a[i] = ad[i] + rr * (a[i] * gv[i] - (b[i] * rr) * dot);
      if (out32) store_f32<V>(out32 + off + c, a);
      if (out_t) store_vec<T>(out_t + off + c, a);
    }
  } else {
    for (int c = lane; c < H; c += WAVE) {
      const float w = dh[off + c] * to_float(g[c]);
      const float v = add_in[off + c] + rr * (w - (x[off + c] * rr) * dot);
      if (out32) out32[off + c] = v;
      if (out_t) out_t[off + c] = from_float<T>(v);
    }
  }
}

// ---------------------------------------------------------------- RMSNorm backward, gain partials
// partial[chunk][c] = sum over the chunk's rows (ascending) of dh[t][c] * x[t][c] * r[t].
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_bwd_gain_kernel(const float* __restrict__ dh, const float* __restrict__ x,
                                                               const float* __restrict__ r, float* __restrict__ partial,
                                                               int Tn, int H) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int chunk = blockIdx.y;
  if (c >= H) return;
  const int t0 = chunk * NORM_BWD_ROWS;
  const int t1 = min(t0 + NORM_BWD_ROWS, Tn);
  float acc = 0.f;
  for (int t = t0; t < t1; ++t) acc += dh[(size_t)t * H + c] * (x[(size_t)t * H + c] * r[t]);
  partial[(size_t)chunk * H + c] = acc;
}

// ---------------------------------------------------------------- RMSNorm backward, fused
// Rows and gain partials in one pass over dh and x.  A workgroup owns FUSED_ROWS consecutive rows, two
// per wavefront; every lane keeps the running sums of dh * xhat of its own columns (NV vectors of
// Vec<T>::N columns) in registers, the four wavefronts are added in wavefront order through LDS, and
// the workgroup writes one partial row.  H <= NV * 64 * Vec<T>::N and H % Vec<T>::N == 0.
constexpr int FUSED_ROWS = 8;

template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_bwd_fused_kernel(const float* __restrict__ dh, const float* __restrict__ x,
                                                                const float* __restrict__ r, const T* __restrict__ g,
                                                                const float* __restrict__ add_in, float* __restrict__ out32,
                                                                T* __restrict__ out_t, float* __restrict__ partial,
                                                                int Tn, int H) {
  constexpr int V = Vec<T>::N;
  extern __shared__ float red[];                 // [4][H]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float gsum[NV][V];
#pragma unroll
  for (int v = 0; v < NV; ++v)
#pragma unroll
    for (int i = 0; i < V; ++i) gsum[v][i] = 0.f;
  for (int rr_ = 0; rr_ < FUSED_ROWS / 4; ++rr_) {
    const int row = blockIdx.x * FUSED_ROWS + wave * (FUSED_ROWS / 4) + rr_;
    if (row >= Tn) break;
    const size_t off = (size_t)row * H;
    const float rr = r[row];
    float dot = 0.f;
    if constexpr (NV <= 8) {
      // rows of up to 4096 values: dh and x stay in registers between the two sweeps (each is read from memory
      // once; 254 registers, two wavefronts per SIMD).  Measured at hidden 4096: 84 -> 78 us stand-alone, B task -0.8 %.
      float a[NV][V], b[NV][V];
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int c = (v * WAVE + lane) * V;
        if (c < H) {
          load_f32<V>(dh + off + c, a[v]);
          load_f32<V>(x + off + c, b[v]);
        }
      }
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int c = (v * WAVE + lane) * V;
        if (c < H) {
          float gv[V];
          load_vec<T>(g + c, gv);
#pragma unroll
          for (int i = 0; i < V; ++i) {
            b[v][i] *= rr;                       // xhat
            dot += a[v][i] * gv[i] * b[v][i];
            gsum[v][i] += a[v][i] * b[v][i];
          }
        }
      }
      dot = wave_sum(dot) / (float)H;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int c = (v * WAVE + lane) * V;
        if (c < H) {
          float gv[V], ad[V];
          load_vec<T>(g + c, gv);
          load_f32<V>(add_in + off + c, ad);
#pragma unroll
          for (int i = 0; i < V; ++i) ad[i] += rr * (a[v][i] * gv[i] - b[v][i] * dot);
          if (out32) store_f32<V>(out32 + off + c, ad);
          if (out_t) store_vec<T>(out_t + off + c, ad);
        }
      }
    } else {
      // longer rows (hidden 8192): keeping them would leave one wavefront per SIMD, measured slower (174 -> 197 us);
      // the second sweep re-reads the row, served by cache
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int c = (v * WAVE + lane) * V;
        if (c < H) {
          float a[V], b[V], gv[V];
          load_f32<V>(dh + off + c, a);
          load_f32<V>(x + off + c, b);
          load_vec<T>(g + c, gv);
#pragma unroll
          for (int i = 0; i < V; ++i) {
            const float xh = b[i] * rr;
            dot += a[i] * gv[i] * xh;
            gsum[v][i] += a[i] * xh;
          }
        }
      }
      dot = wave_sum(dot) / (float)H;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int c = (v * WAVE + lane) * V;
        if (c < H) {
          float a[V], b[V], gv[V], ad[V];
          load_f32<V>(dh + off + c, a);
          load_f32<V>(x + off + c, b);
          load_vec<T>(g + c, gv);
          load_f32<V>(add_in + off + c, ad);
#pragma unroll
          for (int i = 0; i < V; ++i) ad[i] += rr * (a[i] * gv[i] - (b[i] * rr) * dot);
          if (out32) store_f32<V>(out32 + off + c, ad);
          if (out_t) store_vec<T>(out_t + off + c, ad);
        }
      }
    }
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) {
    const int c = (v * WAVE + lane) * V;
    if (c < H) store_f32<V>(red + (size_t)wave * H + c, gsum[v]);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < H; c += 256)
    partial[(size_t)blockIdx.x * H + c] = ((red[c] + red[H + c]) + red[2 * H + c]) + red[3 * H + c];
}

// Column sums of `partial` [n_partial][H] in one fixed order: 16 contiguous slices of the rows are
// summed front to back by 16 thread groups (4 columns per thread), then added in slice order.
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ partial, int n_partial, int H,
                                                     float* __restrict__ out) {
  __shared__ float red[16][64];
  const int cv = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int c = blockIdx.x * 64 + cv * 4;
  const int per = (n_partial + 15) / 16;
  const int p0 = grp * per, p1 = min(p0 + per, n_partial);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (c + 3 < H && (H & 3) == 0) {
    // eight loads in flight at a time, added in row order (the loop is bound by the latency of its loads)
    int p = p0;
    for (; p + 8 <= p1; p += 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(partial + (size_t)(p + u) * H + c);
#pragma unroll
      for (int u = 0; u < 8; ++u) { acc[0] += v[u].x; acc[1] += v[u].y; acc[2] += v[u].z; acc[3] += v[u].w; }
    }
    for (; p < p1; ++p) {
      const float4 v = *reinterpret_cast<const float4*>(partial + (size_t)p * H + c);
      acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
    }
  } else {
    for (int p = p0; p < p1; ++p)
      for (int i = 0; i < 4; ++i)
        if (c + i < H) acc[i] += partial[(size_t)p * H + c + i];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) red[grp][cv * 4 + i] = acc[i];
  __syncthreads();
  if (threadIdx.x < 64) {
    const int cc = blockIdx.x * 64 + threadIdx.x;
    if (cc < H) {
      float t = red[0][threadIdx.x];
#pragma unroll
      for (int q = 1; q < 16; ++q) t += red[q][threadIdx.x];
      out[cc] = t;
    }
  }
}

// ---------------------------------------------------------------- SwiGLU / GELU
__device__ inline float sigmoidf_(float z) { return 1.0f / (1.0f + __expf(-z)); }

template <typename T>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const T* __restrict__ gu, T* __restrict__ m, int Tn, int F) {
  constexpr int V = Vec<T>::N;
  const int fv = F / V;
  const size_t n = (size_t)Tn * fv;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const size_t t = i / fv;
    const int f = (int)(i % fv) * V;
    float a[V], b[V];
    load_vec<T>(gu + t * 2 * F + f, a);
    load_vec<T>(gu + t * 2 * F + F + f, b);
#pragma unroll
    for (int k = 0; k < V; ++k) a[k] = a[k] * sigmoidf_(a[k]) * b[k];
    store_vec<T>(m + t * F + f, a);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const float* __restrict__ dm, const T* __restrict__ gu,
                                                         T* __restrict__ dgu, int Tn, int F) {
  constexpr int V = Vec<T>::N;
  const int fv = F / V;
  const size_t n = (size_t)Tn * fv;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const size_t t = i / fv;
    const int f = (int)(i % fv) * V;
    float a[V], b[V], d[V], da[V], db[V];
    load_vec<T>(gu + t * 2 * F + f, a);
    load_vec<T>(gu + t * 2 * F + F + f, b);
    load_f32<V>(dm + t * F + f, d);
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const float sg = sigmoidf_(a[k]);
      da[k] = d[k] * b[k] * sg * (1.0f + a[k] * (1.0f - sg));
      db[k] = d[k] * a[k] * sg;
    }
    store_vec<T>(dgu + t * 2 * F + f, da);
    store_vec<T>(dgu + t * 2 * F + F + f, db);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const T* __restrict__ u, T* __restrict__ m, size_t nv) {
  constexpr int V = Vec<T>::N;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    float a[V];
    load_vec<T>(u + i * V, a);
#pragma unroll
    for (int k = 0; k < V; ++k) a[k] = 0.5f * a[k] * (1.0f + erff(a[k] * 0.70710678118654752f));
    store_vec<T>(m + i * V, a);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(const float* __restrict__ dm, const T* __restrict__ u,
                                                       T* __restrict__ du, size_t nv) {
  constexpr int V = Vec<T>::N;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (size_t)gridDim.x * 256) {
    float a[V], d[V];
    load_vec<T>(u + i * V, a);
    load_f32<V>(dm + i * V, d);
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const float Phi = 0.5f * (1.0f + erff(a[k] * 0.70710678118654752f));
      const float phi = 0.39894228040143268f * __expf(-0.5f * a[k] * a[k]);
      d[k] = d[k] * (Phi + a[k] * phi);
    }
    store_vec<T>(du + i * V, d);
  }
}

// ---------------------------------------------------------------- LayerNorm (model-fidelity variant)
// Plain kernels, one wavefront per row: h = (x - mu) * r * g + b with r = (var + eps)^-1/2 (biased
// variance, two passes over the row: mean first, then squared deviations).
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const float* __restrict__ x, const T* __restrict__ g,
                                                            const T* __restrict__ b, T* __restrict__ h,
                                                            float* __restrict__ r_out, float* __restrict__ mu_out,
                                                            int Tn, int H, float eps, f16_t* __restrict__ h16) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Tn) return;
  const float* xr = x + (size_t)row * H;
  float sum = 0.f;
  for (int c = lane; c < H; c += WAVE) sum += xr[c];
  const float mu = wave_sum(sum) / (float)H;
  float ss = 0.f;
  for (int c = lane; c < H; c += WAVE) { const float dlt = xr[c] - mu; ss += dlt * dlt; }
  const float r = 1.0f / sqrtf(wave_sum(ss) / (float)H + eps);
  if (lane == 0) { r_out[row] = r; mu_out[row] = mu; }
  T* hr = h + (size_t)row * H;
  for (int c = lane; c < H; c += WAVE) {
    const float v = (xr[c] - mu) * r * to_float(g[c]) + to_float(b[c]);
    hr[c] = from_float<T>(v);
    if (h16) h16[(size_t)row * H + c] = from_float<f16_t>(v);
  }
}

// dx = add_in + r * (w - mean(w) - xhat * mean(w * xhat)),  w = dh * g,  xhat = (x - mu) * r.
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_rows_kernel(const float* __restrict__ dh, const float* __restrict__ x,
                                                                 const float* __restrict__ r, const float* __restrict__ mu,
                                                                 const T* __restrict__ g, const float* __restrict__ add_in,
                                                                 float* __restrict__ out32, T* __restrict__ out_t, int Tn, int H) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Tn) return;
  const size_t off = (size_t)row * H;
  const float rr = r[row], m = mu[row];
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane; c < H; c += WAVE) {
    const float w = dh[off + c] * to_float(g[c]);
    s1 += w;
    s2 += w * ((x[off + c] - m) * rr);
  }
  s1 = wave_sum(s1) / (float)H;
  s2 = wave_sum(s2) / (float)H;
  for (int c = lane; c < H; c += WAVE) {
    const float w = dh[off + c] * to_float(g[c]);
    const float v = add_in[off + c] + rr * (w - s1 - ((x[off + c] - m) * rr) * s2);
    if (out32) out32[off + c] = v;
    if (out_t) out_t[off + c] = from_float<T>(v);
  }
}

// Per-chunk partial sums for the LayerNorm gain and bias gradients: partial_g[chunk][c] = sum over the
// chunk's rows (ascending) of dh * xhat, partial_b[chunk][c] = sum of dh.  One thread per column.
__global__ __launch_bounds__(256) void layernorm_bwd_partials_kernel(const float* __restrict__ dh, const float* __restrict__ x,
                                                                     const float* __restrict__ r, const float* __restrict__ mu,
                                                                     float* __restrict__ partial_g, float* __restrict__ partial_b,
                                                                     int Tn, int H) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= H) return;
  const int r0 = blockIdx.y * NORM_BWD_ROWS, r1 = min(r0 + NORM_BWD_ROWS, Tn);
  float sg = 0.f, sb = 0.f;
  for (int row = r0; row < r1; ++row) {
    const float d = dh[(size_t)row * H + c];
    sg += d * ((x[(size_t)row * H + c] - mu[row]) * r[row]);
    sb += d;
  }
  partial_g[(size_t)blockIdx.y * H + c] = sg;
  partial_b[(size_t)blockIdx.y * H + c] = sb;
}

// Per-chunk column sums of a [Tn, N] tensor of the storage type (row pitch ld): partial[chunk][c] = sum
// over the chunk's rows in ascending order.  With launch_colsum this gives the bias gradients.
template <typename T>
__global__ __launch_bounds__(256) void colsum_rows_kernel(const T* __restrict__ src, int ld, float* __restrict__ partial,
                                                          int Tn, int N) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= N) return;
  const int r0 = blockIdx.y * NORM_BWD_ROWS, r1 = min(r0 + NORM_BWD_ROWS, Tn);
  float acc = 0.f;
  for (int row = r0; row < r1; ++row) acc += to_float(src[(size_t)row * ld + c]);
  partial[(size_t)blockIdx.y * N + c] = acc;
}

// ---------------------------------------------------------------- head norm (QK-norm variant)
// RMSNorm over head_dim of every (token, head) d-vector of the first n_heads heads of a [T, ld] tensor, in
// place: x <- xhat * g, with xhat = x * r saved (storage type) and r saved (fp32) for the backward.
// Heads [0, nq) use gq, heads [nq, n_heads) use gk.  One wavefront per (token, head).
// TP = type of the gains (the parameter storage type); T = type of the tensor and of the saved xhat.
template <typename T, typename TP>
__global__ __launch_bounds__(256) void headnorm_fwd_kernel(T* __restrict__ x, int ld, int nq, int n_heads, int d,
                                                           const TP* __restrict__ gq, const TP* __restrict__ gk,
                                                           T* __restrict__ xhat, float* __restrict__ r_out, int Tn, float eps) {
  const size_t pair = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (pair >= (size_t)Tn * n_heads) return;
  const int t = (int)(pair / n_heads), hd = (int)(pair - (size_t)t * n_heads);
  T* p = x + (size_t)t * ld + hd * d;
  const TP* g = hd < nq ? gq : gk;
  float ss = 0.f;
  for (int c = lane; c < d; c += WAVE) { const float v = to_float(p[c]); ss += v * v; }
  const float r = 1.0f / sqrtf(wave_sum(ss) / (float)d + eps);
  if (lane == 0) r_out[pair] = r;
  for (int c = lane; c < d; c += WAVE) {
    const float xh = to_float(p[c]) * r;
    xhat[pair * d + c] = from_float<T>(xh);
    p[c] = from_float<T>(xh * to_float(g[c]));
  }
}

// Backward, in place on the gradient tensor: dx = r * (w - xhat * mean(w * xhat)), w = dy * g.  A workgroup
// handles 64 consecutive (token, head) pairs of ONE kind (grid y = 0: query heads, 1: key heads) and writes
// one partial row of the gain gradient, sum over its pairs (ascending, wavefronts combined in order) of dy * xhat.
// TX = type of the saved xhat (the forward's tensor type); T = type of the gradient tensor and of the gains.
template <typename T, typename TX>
__global__ __launch_bounds__(256) void headnorm_bwd_kernel(T* __restrict__ dy, int ld, int nq, int n_heads, int d,
                                                           const T* __restrict__ gq, const T* __restrict__ gk,
                                                           const TX* __restrict__ xhat, const float* __restrict__ r_in,
                                                           float* __restrict__ partial_q, float* __restrict__ partial_k, int Tn,
                                                           float* __restrict__ dk32) {
  __shared__ float red[4][128];
  const int kind = blockIdx.y, nh = kind == 0 ? nq : n_heads - nq, h0 = kind == 0 ? 0 : nq;
  const T* g = kind == 0 ? gq : gk;
  float* partial = kind == 0 ? partial_q : partial_k;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const size_t n_pairs = (size_t)Tn * nh;
  if ((size_t)blockIdx.x * 64 >= n_pairs) return;
  float gs[2] = {0.f, 0.f};
  for (int i = 0; i < 16; ++i) {
    const size_t q = (size_t)blockIdx.x * 64 + wave * 16 + i;       // pair index inside this kind
    if (q >= n_pairs) break;
    const int t = (int)(q / nh), hd = h0 + (int)(q - (size_t)t * nh);
    const size_t pair = (size_t)t * n_heads + hd;
    T* p = dy + (size_t)t * ld + hd * d;
    const float rr = r_in[pair];
    float w[2], xh[2], dv[2], dot = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = lane + u * WAVE;
      w[u] = 0.f; xh[u] = 0.f; dv[u] = 0.f;
      if (c < d) {
        dv[u] = to_float(p[c]);
        xh[u] = to_float(xhat[pair * d + c]);
        w[u] = dv[u] * to_float(g[c]);
        dot += w[u] * xh[u];
        gs[u] += dv[u] * xh[u];
      }
    }
    dot = wave_sum(dot) / (float)d;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = lane + u * WAVE;
      if (c < d) {
        const float dxv = rr * (w[u] - xh[u] * dot);
        p[c] = from_float<T>(dxv);
        // un-rounded copy of the key-head gradients [Tn, nk * d]: their column sum (the key bias gradient) is a
        // small remainder of cancelling terms and would lose its leading digits to the storage rounding
        if (dk32 && kind == 1) dk32[((size_t)t * nh + (hd - h0)) * d + c] = dxv;
      }
    }
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) red[wave][lane + u * WAVE] = gs[u];
  __syncthreads();
  if ((int)threadIdx.x < d) partial[(size_t)blockIdx.x * d + threadIdx.x] =
      ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
}

// ---------------------------------------------------------------- rotary embedding
// One workgroup per (query tile, head); a wavefront per row, a lane per pair.  The angle is formed in
// double precision and reduced to [0, 2 pi) before the single-precision sine and cosine, so that the
// fp32 path keeps its 1e-4 budget at positions in the thousands.
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ x, const AttnTile* __restrict__ tiles, int d, int ld,
                                                   double log2_base, float sign) {
  const AttnTile tl = tiles[blockIdx.x];
  const int head = blockIdx.y, half = d >> 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i0 = lane; i0 < half; i0 += 64) {
    const double theta = exp2(-2.0 * (double)i0 / (double)d * log2_base);
    for (int row = tl.r0 + wave; row < tl.r1; row += 4) {
      double ang = (double)(row - tl.s0) * theta;
      ang -= 6.283185307179586476925 * floor(ang * 0.1591549430918953357689);
      float sn, cs;
      __sincosf((float)ang, &sn, &cs);
      sn *= sign;
      T* p = x + (size_t)row * ld + head * d + i0;
      const float a = to_float(p[0]), b = to_float(p[half]);
      p[0] = from_float<T>(a * cs - b * sn);
      p[half] = from_float<T>(b * cs + a * sn);
    }
  }
}

// ---------------------------------------------------------------- gradient reduction
// Slots are streamed once: all loads of a group of up to 8 slots are issued before the first add (the
// adds then run in microbatch index order, which is what fixes the result bit for bit), and the loads
// bypass temporal caching.
typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void grad_reduce_kernel(const f32x4* __restrict__ slots, size_t stride4, int M,
                                                          f32x4* __restrict__ out, size_t n4) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    f32x4 acc = __builtin_nontemporal_load(slots + i);
    for (int j0 = 1; j0 < M; j0 += 8) {
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (j0 + u < M) v[u] = __builtin_nontemporal_load(slots + (size_t)(j0 + u) * stride4 + i);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (j0 + u < M) acc += v[u];
    }
    __builtin_nontemporal_store(acc, out + i);
  }
}

inline int grid_for(size_t n, int cap = 256 * 32) {
  size_t b = (n + 255) / 256;
  return (int)(b < 1 ? 1 : (b > (size_t)cap ? cap : b));
}

}  // namespace

#define DISPATCH_T(dtype, ...)                       \
  if ((dtype) == F32) { using T = float; __VA_ARGS__; } \
  else { using T = bf16_t; __VA_ARGS__; }

// bf16 -> IEEE half, element by element (exact except below half's normal range; saturating).
__global__ __launch_bounds__(256) void bf16_to_f16_kernel(const bf16_t* __restrict__ src, f16_t* __restrict__ dst, size_t n8) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
    float v[8];
    load_vec<bf16_t>(src + i * 8, v);
    store_vec<f16_t>(dst + i * 8, v);
  }
}

hipError_t launch_widen(const void* src, float* dst, size_t n, int dtype, hipStream_t s, void* copy) {
  DISPATCH_T(dtype, hipLaunchKernelGGL(widen_kernel<T>, dim3(grid_for(n / Vec<T>::N + 1)), dim3(256), 0, s, (const T*)src, dst, n, (T*)copy));
  return hipGetLastError();
}

hipError_t launch_rope(void* x, const AttnTile* q_tiles, int n_q_tiles, int n_heads, int d, int ld, float base,
                       float sign, int dtype, hipStream_t s) {
  if (n_q_tiles < 1 || n_heads < 1 || (d & 1) || !(base > 1.0f)) return hipErrorInvalidValue;
  if (dtype == F16) {
    hipLaunchKernelGGL(rope_kernel<f16_t>, dim3(n_q_tiles, n_heads), dim3(256), 0, s, (f16_t*)x, q_tiles, d, ld, log2((double)base), sign);
    return hipGetLastError();
  }
  DISPATCH_T(dtype, hipLaunchKernelGGL(rope_kernel<T>, dim3(n_q_tiles, n_heads), dim3(256), 0, s, (T*)x, q_tiles, d, ld,
                                       log2((double)base), sign));
  return hipGetLastError();
}

hipError_t launch_rmsnorm_fwd(const float* x, const void* g, void* h, float* r_out, int Tn, int H, float eps,
                              int dtype, hipStream_t s, void* h16) {
  if (h16 && dtype != BF16) return hipErrorInvalidValue;
  const int V = dtype == F32 ? 4 : 8;
  if ((H % V) == 0) {
    const int nv = (H + WAVE * V - 1) / (WAVE * V);
#define RRFP_ROWS(NVV)                                                                                              \
  if (nv <= NVV) {                                                                                                  \
    DISPATCH_T(dtype, hipLaunchKernelGGL((rmsnorm_fwd_rows_kernel<T, NVV>), dim3((Tn + 3) / 4), dim3(256), 0, s, x, \
                                         (const T*)g, (T*)h, r_out, Tn, H, eps, (f16_t*)h16));                      \
    return hipGetLastError();                                                                                       \
  }
    RRFP_ROWS(1) RRFP_ROWS(2) RRFP_ROWS(4) RRFP_ROWS(8) RRFP_ROWS(16)
#undef RRFP_ROWS
  }
  DISPATCH_T(dtype, hipLaunchKernelGGL(rmsnorm_fwd_kernel<T>, dim3((Tn + 3) / 4), dim3(256), 0, s, x, (const T*)g, (T*)h,
                                       r_out, Tn, H, eps, (f16_t*)h16));
  return hipGetLastError();
}

template <typename T, int NV>
hipError_t launch_bwd_fused(const float* dh, const float* x, const float* r, const void* g, const float* add_in,
                            float* out32, void* out_t, float* dg_partial, int Tn, int H, hipStream_t s) {
  auto kern = rmsnorm_bwd_fused_kernel<T, NV>;
  const size_t smem = (size_t)4 * H * sizeof(float);
  static std::once_flag once;
  static hipError_t once_status = hipSuccess;
  if (hipError_t e = set_max_dynamic_lds_once(once, once_status, (const void*)kern, 4 * NV * WAVE * Vec<T>::N * 4); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((Tn + FUSED_ROWS - 1) / FUSED_ROWS), dim3(256), smem, s, dh, x, r, (const T*)g, add_in, out32,
                     (T*)out_t, dg_partial, Tn, H);
  return hipGetLastError();
}

int norm_bwd_partials(int Tn, int H, int dtype) {
  const int V = dtype == F32 ? 4 : 8;
  const bool fused = (H % V) == 0 && H <= 16 * WAVE * V && (dtype != F32 || H <= 8 * WAVE * V);
  return fused ? (Tn + FUSED_ROWS - 1) / FUSED_ROWS : (Tn + NORM_BWD_ROWS - 1) / NORM_BWD_ROWS;
}

hipError_t launch_rmsnorm_bwd(const float* dh, const float* x, const float* r, const void* g, const float* add_in,
                              float* out32, void* out_t, float* dg_partial, int Tn, int H, int dtype, hipStream_t s) {
  const int V = dtype == F32 ? 4 : 8;
  if (norm_bwd_partials(Tn, H, dtype) == (Tn + FUSED_ROWS - 1) / FUSED_ROWS && (H % V) == 0) {
    const int nv = (H + WAVE * V - 1) / (WAVE * V);
#define RRFP_FUSED(NVV)                                                                                         \
  if (nv <= NVV) {                                                                                              \
    DISPATCH_T(dtype, return (launch_bwd_fused<T, NVV>(dh, x, r, g, add_in, out32, out_t, dg_partial, Tn, H, s))); \
  }
    RRFP_FUSED(1) RRFP_FUSED(2) RRFP_FUSED(3) RRFP_FUSED(4) RRFP_FUSED(6) RRFP_FUSED(8)
    if (dtype != F32) { RRFP_FUSED(16) }
#undef RRFP_FUSED
  }
  const int chunks = (Tn + NORM_BWD_ROWS - 1) / NORM_BWD_ROWS;
  DISPATCH_T(dtype, {
    hipLaunchKernelGGL(rmsnorm_bwd_gain_kernel<T>, dim3((H + 255) / 256, chunks), dim3(256), 0, s, dh, x, r,
                       dg_partial, Tn, H);
    hipLaunchKernelGGL(rmsnorm_bwd_rows_kernel<T>, dim3((Tn + 3) / 4), dim3(256), 0, s, dh, x, r, (const T*)g,
                       add_in, out32, (T*)out_t, Tn, H);
  });
  return hipGetLastError();
}

int headnorm_partials(int Tn, int n_heads_of_kind) { return (int)(((size_t)Tn * n_heads_of_kind + 63) / 64); }

hipError_t launch_headnorm_fwd(void* x, int ld, int nq, int n_heads, int d, const void* gq, const void* gk, void* xhat,
                               float* r_out, int Tn, float eps, int dtype, hipStream_t s) {
  if (d > 128) return hipErrorInvalidValue;
  const size_t pairs = (size_t)Tn * n_heads;
  if (dtype == F16) {   // half tensor, bf16 gains
    hipLaunchKernelGGL((headnorm_fwd_kernel<f16_t, bf16_t>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, s, (f16_t*)x, ld, nq,
                       n_heads, d, (const bf16_t*)gq, (const bf16_t*)gk, (f16_t*)xhat, r_out, Tn, eps);
    return hipGetLastError();
  }
  DISPATCH_T(dtype, hipLaunchKernelGGL((headnorm_fwd_kernel<T, T>), dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, s, (T*)x, ld, nq,
                                       n_heads, d, (const T*)gq, (const T*)gk, (T*)xhat, r_out, Tn, eps));
  return hipGetLastError();
}

hipError_t launch_headnorm_bwd(void* dy, int ld, int nq, int n_heads, int d, const void* gq, const void* gk, const void* xhat,
                               const float* r_in, float* partial_q, float* partial_k, int Tn, int dtype, hipStream_t s,
                               float* dk32, int xhat_dtype) {
  if (d > 128) return hipErrorInvalidValue;
  const int nb = std::max(headnorm_partials(Tn, nq), headnorm_partials(Tn, n_heads - nq));
  if (xhat_dtype == F16) {
    if (dtype != BF16) return hipErrorInvalidValue;
    hipLaunchKernelGGL((headnorm_bwd_kernel<bf16_t, f16_t>), dim3(nb, 2), dim3(256), 0, s, (bf16_t*)dy, ld, nq, n_heads, d,
                       (const bf16_t*)gq, (const bf16_t*)gk, (const f16_t*)xhat, r_in, partial_q, partial_k, Tn, dk32);
    return hipGetLastError();
  }
  DISPATCH_T(dtype, hipLaunchKernelGGL((headnorm_bwd_kernel<T, T>), dim3(nb, 2), dim3(256), 0, s, (T*)dy, ld, nq, n_heads, d,
                                       (const T*)gq, (const T*)gk, (const T*)xhat, r_in, partial_q, partial_k, Tn, dk32));
  return hipGetLastError();
}

int colsum_chunks(int Tn) { return (Tn + NORM_BWD_ROWS - 1) / NORM_BWD_ROWS; }

hipError_t launch_layernorm_fwd(const float* x, const void* g, const void* b, void* h, float* r_out, float* mu_out,
                                int Tn, int H, float eps, int dtype, hipStream_t s, void* h16) {
  if (h16 && dtype != BF16) return hipErrorInvalidValue;
  DISPATCH_T(dtype, hipLaunchKernelGGL(layernorm_fwd_kernel<T>, dim3((Tn + 3) / 4), dim3(256), 0, s, x, (const T*)g,
                                       (const T*)b, (T*)h, r_out, mu_out, Tn, H, eps, (f16_t*)h16));
  return hipGetLastError();
}

hipError_t launch_layernorm_bwd(const float* dh, const float* x, const float* r, const float* mu, const void* g,
                                const float* add_in, float* out32, void* out_t, float* partial_g, float* partial_b,
                                int Tn, int H, int dtype, hipStream_t s) {
  hipLaunchKernelGGL(layernorm_bwd_partials_kernel, dim3((H + 255) / 256, colsum_chunks(Tn)), dim3(256), 0, s, dh, x, r, mu,
                     partial_g, partial_b, Tn, H);
  DISPATCH_T(dtype, hipLaunchKernelGGL(layernorm_bwd_rows_kernel<T>, dim3((Tn + 3) / 4), dim3(256), 0, s, dh, x, r, mu,
                                       (const T*)g, add_in, out32, (T*)out_t, Tn, H));
  return hipGetLastError();
}

hipError_t launch_colsum_rows(const void* src, int ld, float* partial, int Tn, int N, int dtype, hipStream_t s) {
  DISPATCH_T(dtype, hipLaunchKernelGGL(colsum_rows_kernel<T>, dim3((N + 255) / 256, colsum_chunks(Tn)), dim3(256), 0, s,
                                       (const T*)src, ld, partial, Tn, N));
  return hipGetLastError();
}

hipError_t launch_colsum(const float* partial, int n_partial, int H, float* out, hipStream_t s) {
  hipLaunchKernelGGL(colsum_kernel, dim3((H + 63) / 64), dim3(256), 0, s, partial, n_partial, H, out);
  return hipGetLastError();
}

hipError_t launch_swiglu_fwd(const void* gu, void* m, int Tn, int F, int dtype, hipStream_t s) {
  DISPATCH_T(dtype, {
    if (F % Vec<T>::N) return hipErrorInvalidValue;
    hipLaunchKernelGGL(swiglu_fwd_kernel<T>, dim3(grid_for((size_t)Tn * F / Vec<T>::N)), dim3(256), 0, s, (const T*)gu,
                       (T*)m, Tn, F);
  });
  return hipGetLastError();
}

hipError_t launch_swiglu_bwd(const float* dm, const void* gu, void* dgu, int Tn, int F, int dtype, hipStream_t s) {
  DISPATCH_T(dtype, {
    if (F % Vec<T>::N) return hipErrorInvalidValue;
    hipLaunchKernelGGL(swiglu_bwd_kernel<T>, dim3(grid_for((size_t)Tn * F / Vec<T>::N)), dim3(256), 0, s, dm,
                       (const T*)gu, (T*)dgu, Tn, F);
  });
  return hipGetLastError();
}

hipError_t launch_gelu_fwd(const void* u, void* m, int Tn, int F, int dtype, hipStream_t s) {
  DISPATCH_T(dtype, {
    if (F % Vec<T>::N) return hipErrorInvalidValue;
    const size_t nv = (size_t)Tn * F / Vec<T>::N;
    hipLaunchKernelGGL(gelu_fwd_kernel<T>, dim3(grid_for(nv)), dim3(256), 0, s, (const T*)u, (T*)m, nv);
  });
  return hipGetLastError();
}

hipError_t launch_gelu_bwd(const float* dm, const void* u, void* du, int Tn, int F, int dtype, hipStream_t s) {
  DISPATCH_T(dtype, {
    if (F % Vec<T>::N) return hipErrorInvalidValue;
    const size_t nv = (size_t)Tn * F / Vec<T>::N;
    hipLaunchKernelGGL(gelu_bwd_kernel<T>, dim3(grid_for(nv)), dim3(256), 0, s, dm, (const T*)u, (T*)du, nv);
  });
  return hipGetLastError();
}

int grad_scale_partials(size_t n) { return grid_for(n / 8 + 1, 1024); }

hipError_t launch_grad_scale(const void* dy, size_t n, int dtype, float* partial, float* scale, hipStream_t s) {
  const int nb = grad_scale_partials(n);
  DISPATCH_T(dtype, hipLaunchKernelGGL(absmax_partial_kernel<T>, dim3(nb), dim3(256), 0, s, (const T*)dy, n, partial));
  hipLaunchKernelGGL(grad_scale_kernel, dim3(1), dim3(256), 0, s, (const float*)partial, nb, scale);
  return hipGetLastError();
}

hipError_t launch_bf16_to_f16(const void* src, void* dst, size_t n, hipStream_t s) {
  if (n % 8 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bf16_to_f16_kernel, dim3(grid_for(n / 8)), dim3(256), 0, s, (const bf16_t*)src, (f16_t*)dst, n / 8);
  return hipGetLastError();
}

hipError_t launch_grad_reduce(const float* slots, size_t slot_stride, int M, float* out, size_t n, hipStream_t s) {
  if (n % 4 || slot_stride % 4) return hipErrorInvalidValue;
  // one 16-byte element per thread where the grid allows it: measured 5.3 TB/s against 4.6 TB/s for a grid-stride
  // loop over 8192 workgroups (8 slots of 1 GiB; a pure read of the same bytes runs at 5.7 TB/s on this chip)
  hipLaunchKernelGGL(grad_reduce_kernel, dim3(grid_for(n / 4, 1 << 24)), dim3(256), 0, s, (const f32x4*)slots, slot_stride / 4,
                     M, (f32x4*)out, n / 4);
  return hipGetLastError();
}

}  // namespace rrfp
