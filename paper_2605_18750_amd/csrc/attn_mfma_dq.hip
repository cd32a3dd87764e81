// dQ kernel of the MFMA attention backward (see attn_mfma.hip for the scheme).  It lives in its own
// translation unit because it is compiled with a different instruction-scheduling strategy than the other
// attention kernels (the build passes -mllvm -amdgpu-sched-strategy=iterative-ilp for this file: measured
// 8-10 % faster for this kernel, slower for the dK/dV kernel, neutral for the forward).
#include "attn_mfma_common.h"

namespace rrfp {
namespace {

template <int D>
struct DqCfg {
  static constexpr int DP = (D + 31) / 32 * 32;
  static constexpr int KP = 304;                     // K tile: row fragments AND transposed fragments.  304 = 48 (mod 256):
                                                     // 16 rows x 16 B and 4 rows x 32 B both land on distinct banks
  static constexpr int VP = D * 2 + 16;              // V tile: row fragments only
  static constexpr int K_BYTES = BKV * KP;
  static constexpr int STAGE = (K_BYTES + BKV * VP + 255) / 256 * 256;
  static constexpr int SMEM = 2 * STAGE;
};

template <int D, int NIB>
__global__ __launch_bounds__(FWD_Q_ROWS / (32 * NIB) * 64) void attn_dq_mfma_kernel(const el_t* __restrict__ qkv, const el_t* __restrict__ d_o,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           bf16_t* __restrict__ dqkv, const AttnTile* __restrict__ tiles,
                                                           int Tn, int nq, int nkv, int causal, float scale,
                                                           const float* __restrict__ grad_scale) {
  constexpr int NT = FWD_Q_ROWS / (32 * NIB) * 64;   // threads: one wavefront per 32 * NIB query rows
  constexpr int WQ = 32 * NIB;
  using C = DqCfg<D>;
  constexpr int NDS = D / 16, NDB = C::DP / 32;
  constexpr float LOG2E = 1.4426950408889634f;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const AttnTile tl = tiles[blockIdx.y];
  const int a = blockIdx.x, b = a / (nq / nkv);
  const int ld = (nq + 2 * nkv) * D;
  const int qcol = a * D, kcol = (nq + b) * D, vcol = (nq + nkv + b) * D;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: wave-level branches stay uniform
  const int h = lane >> 5, li = lane & 31;
  const int wq0 = tl.r0 + wave * WQ;
  const bool wave_has_rows = wq0 < tl.r1;
  const float scale_log2e = scale * LOG2E;

  frag_t qf[NIB][NDS], dof[NIB][NDS];
  float lse2[NIB], dl[NIB];
#pragma unroll
  for (int ib = 0; ib < NIB; ++ib) {
    const int i = wq0 + ib * 32 + li;
    const bool ok = i < tl.r1;
    lse2[ib] = ok ? lse[(size_t)a * Tn + i] * LOG2E : 0.f;
    dl[ib] = ok ? delta[(size_t)a * Tn + i] : 0.f;
#pragma unroll
    for (int ds = 0; ds < NDS; ++ds) {
      uint4 v = make_uint4(0, 0, 0, 0), w = v;
      if (ok) {
        v = *reinterpret_cast<const uint4*>(qkv + (size_t)i * ld + qcol + ds * 16 + h * 8);
        w = *reinterpret_cast<const uint4*>(d_o + (size_t)i * nq * D + qcol + ds * 16 + h * 8);
      }
      qf[ib][ds] = __builtin_bit_cast(frag_t, v);
      dof[ib][ds] = __builtin_bit_cast(frag_t, w);
    }
  }
  floatx16 acc[NDB][NIB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[db][ib][e] = 0.f;

  const int kv_end = causal ? tl.r1 : tl.s1;
  const int nsteps = (kv_end - tl.s0 + BKV - 1) / BKV;
  uint4 rk[TileRegs<D, BKV, NT>::N], rv[TileRegs<D, BKV, NT>::N];
  tile_load<D, BKV, NT>(rk, qkv + kcol, ld, tl.s0, kv_end);
  tile_load<D, BKV, NT>(rv, qkv + vcol, ld, tl.s0, kv_end);
  tile_store<D, BKV, C::KP, C::DP, NT>(rk, smem);
  tile_store<D, BKV, C::VP, D, NT>(rv, smem + C::K_BYTES);
  __syncthreads();

  // Leading steps in which this wavefront has unmasked keys; the rest only move data.  The dQ
  // accumulators are touched in the first loop alone and unconditionally (they stay in place).
  const int n_active = !wave_has_rows ? 0 : (causal ? min(nsteps, (wq0 + WQ - 1 - tl.s0) / BKV + 1) : nsteps);
  auto io_begin = [&](int st) {
    if (st + 1 < nsteps) {
      tile_load<D, BKV, NT>(rk, qkv + kcol, ld, tl.s0 + (st + 1) * BKV, kv_end);
      tile_load<D, BKV, NT>(rv, qkv + vcol, ld, tl.s0 + (st + 1) * BKV, kv_end);
    }
  };
  auto io_end = [&](int st) {
    if (st + 1 < nsteps) {
      char* nk = smem + ((st + 1) & 1) * C::STAGE;
      tile_store<D, BKV, C::KP, C::DP, NT>(rk, nk);
      tile_store<D, BKV, C::VP, D, NT>(rv, nk + C::K_BYTES);
    }
    __syncthreads();
  };
  int st = 0;
  for (; st < n_active; ++st) {
    const int k0 = tl.s0 + st * BKV;
    const char* sk = smem + (st & 1) * C::STAGE;
    const char* sv = sk + C::K_BYTES;
    io_begin(st);
    const bool need_mask = (causal && k0 + BKV - 1 > wq0) || (k0 + BKV > kv_end);
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib) {
      const int i = wq0 + ib * 32 + li;
      floatx16 s[2], dp[2];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        frag_t kfr[NDS], vfr[NDS];      // all fragments of the 32-key block before its MFMAs
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
          kfr[ds] = frag_rows(sk, C::KP, jb * 32, ds, lane);
          vfr[ds] = frag_rows(sv, C::VP, jb * 32, ds, lane);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) { s[jb][e] = 0.f; dp[jb][e] = 0.f; }
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) {
          s[jb] = mfma16(kfr[ds], qf[ib][ds], s[jb]);
          dp[jb] = mfma16(vfr[ds], dof[ib][ds], dp[jb]);
        }
      }
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        float dsv[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[jb][e], scale_log2e, -lse2[ib]));
          dsv[e] = p * (dp[jb][e] - dl[ib]);
        }
        if (need_mask) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int j = k0 + jb * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
            float v = (j >= kv_end || (causal && j > i)) ? 0.f : dsv[e];
            asm volatile("" : "+v"(v));   // pins the select inside this (wave-uniform) branch
            dsv[e] = v;
          }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const frag_t dsf = pack8(dsv + u * 8);
          frag_t ktr[NDB];
#pragma unroll
          for (int db = 0; db < NDB; ++db) ktr[db] = frag_cols_tr(sk, C::KP, jb * 32 + u * 16, db * 32, lane);
#pragma unroll
          for (int db = 0; db < NDB; ++db)
            acc[db][ib] = mfma16(ktr[db], dsf, acc[db][ib]);
        }
      }
    }
    io_end(st);
  }
  for (; st < nsteps; ++st) {
    io_begin(st);
    io_end(st);
  }
#pragma unroll
  for (int ib = 0; ib < NIB; ++ib) {
    const int i = wq0 + ib * 32 + li;
    if (i >= tl.r1) continue;
    const float out_scale = scale * (grad_scale ? grad_scale[1] : 1.0f);    // d_o held s * dO: undo it (a power of two: exact)
    bf16_t* row = dqkv + (size_t)i * ld + qcol;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int dd = db * 32 + g * 8 + h * 4;
        if (dd >= D) continue;
        uint2 w;
        w.x = pack_bf16x2(acc[db][ib][g * 4 + 0] * out_scale, acc[db][ib][g * 4 + 1] * out_scale);
        w.y = pack_bf16x2(acc[db][ib][g * 4 + 2] * out_scale, acc[db][ib][g * 4 + 3] * out_scale);
        *reinterpret_cast<uint2*>(row + dd) = w;
      }
  }
}

template <int D>
hipError_t dq_launch(const AttnArgs& a, hipStream_t s) {
  auto kq = attn_dq_mfma_kernel<D, DQ_NIB>;
  static std::once_flag once;
  static hipError_t once_status = hipSuccess;
  if (hipError_t e = set_max_dynamic_lds_once(once, once_status, (const void*)kq, DqCfg<D>::SMEM); e != hipSuccess) return e;
  const float scale = 1.0f / sqrtf((float)D);
  hipLaunchKernelGGL(kq, dim3(a.nq, a.n_q_tiles), dim3(FWD_Q_ROWS / (32 * DQ_NIB) * 64), DqCfg<D>::SMEM, s, (const el_t*)a.qkv,
                     (const el_t*)a.d_o, a.lse, a.delta, (bf16_t*)a.dqkv, a.q_tiles, a.T, a.nq, a.nkv, a.causal, scale, a.grad_scale);
  return hipGetLastError();
}

}  // namespace

// Needs a.delta (the delta kernel) on the same stream before it; writes the dq columns of a.dqkv.
hipError_t launch_attn_dq_mfma(const AttnArgs& a, hipStream_t s) {
  if (a.d == 64) return dq_launch<64>(a, s);
  if (a.d == 80) return dq_launch<80>(a, s);
  if (a.d == 128) return dq_launch<128>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace rrfp
