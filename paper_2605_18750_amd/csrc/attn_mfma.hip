// MFMA attention for gfx950 (the bf16 storage path of the stage): tiled online-softmax forward over packed
// segments with GQA, causal or bidirectional masks and head_dim 64 / 80 / 128.  q, k, v (and dO in the
// backward) arrive as IEEE halves, the output and dq, dk, dv leave as bf16: see attn_mfma_common.h.
//
// Forward.  A workgroup (8 wavefronts, two per SIMD) owns one query tile (up to 256 rows inside one
// segment) of one query head; each wavefront owns 32 query rows and stays under 256 registers, so
// that the softmax arithmetic of one wavefront runs under the MFMAs of the other one on its SIMD.
// Keys and values stream through LDS in
// steps of 64 rows with two stages (global loads of step k+1 are in flight while step k runs).
// Scores are computed TRANSPOSED, S^T[key, query] = K Q^T with v_mfma_f32_32x32x16_f16, so
// that a lane holds one query column: the softmax row statistics are lane-local except one
// exchange between the two halves of the wavefront, and the probabilities, converted to halves, are
// already in the B-operand layout of the second product O^T[d, query] += V^T P^T.  V stays in
// LDS in its memory orientation and its fragments come from the LDS transpose read.
// Exponentials are base 2 (scores pre-multiplied by log2 e / sqrt(d)); the saved log-sum-exp
// is in natural-log units.
#include "attn_mfma_common.h"

namespace rrfp {

hipError_t launch_attn_dq_mfma(const AttnArgs& a, hipStream_t s);   // attn_mfma_dq.hip

namespace {

template <int D, int NT>
struct FwdCfg {
  static constexpr int DP = (D + 31) / 32 * 32;      // value columns padded to whole 32-wide MFMA blocks
  static constexpr int KP = D * 2 + 16;              // K row pitch in bytes: 16-byte skew per row
  static constexpr int VP = DP * 2 + 32;             // V row pitch in bytes: 32 or 96 (mod 128)
  static constexpr int K_BYTES = BKV * KP;
  static constexpr int V_BYTES = BKV * VP;
  static constexpr int STAGE = (K_BYTES + V_BYTES + 255) / 256 * 256;
  static constexpr int SMEM = 2 * STAGE;
  static constexpr int CH = D / 8;                   // 16-byte chunks per row
  static constexpr int NCHUNK = BKV * CH;            // chunks per K (or V) tile
  static constexpr int PER_THREAD = (NCHUNK + NT - 1) / NT;
};

template <int D, int NT>
using KvRegs = uint4[FwdCfg<D, NT>::PER_THREAD];

template <int D, int NT>
__device__ __forceinline__ void kv_load(KvRegs<D, NT>& rk, KvRegs<D, NT>& rv,
                                        const el_t* __restrict__ qkv, int ld, int kcol, int vcol, int k0, int k_end) {
  using C = FwdCfg<D, NT>;
#pragma unroll
  for (int i = 0; i < C::PER_THREAD; ++i) {
    // No branches: a thread past the last chunk repeats that chunk (kv_store drops it) and rows at or past
    // k_end repeat row k_end - 1 (finite values; those keys are masked, so their probabilities are zero).
    const int q = min(i * NT + (int)threadIdx.x, C::NCHUNK - 1);
    const int row = q / C::CH, c = q - row * C::CH;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const el_t* p = qkv + (size_t)min(k0 + row, k_end - 1) * ld + c * 8;
    rk[i] = __builtin_bit_cast(uint4, *reinterpret_cast<const u32x4*>(p + kcol));
    rv[i] = __builtin_bit_cast(uint4, *reinterpret_cast<const u32x4*>(p + vcol));
  }
}

template <int D, int NT>
__device__ __forceinline__ void kv_store(const KvRegs<D, NT>& rk, const KvRegs<D, NT>& rv,
                                         char* stage) {
  using C = FwdCfg<D, NT>;
#pragma unroll
  for (int i = 0; i < C::PER_THREAD; ++i) {
    const int q = i * NT + threadIdx.x;
    const int row = q / C::CH, c = q - row * C::CH;
    if (C::NCHUNK % NT == 0 || q < C::NCHUNK) {
      *reinterpret_cast<uint4*>(stage + row * C::KP + c * 16) = rk[i];
      *reinterpret_cast<uint4*>(stage + C::K_BYTES + row * C::VP + c * 16) = rv[i];
    }
  }
  if (C::DP != D) {   // zero the padded value columns so that the unused output rows stay finite
    constexpr int PADCH = (C::DP - D) / 8;
    for (int q = threadIdx.x; q < BKV * PADCH; q += NT) {
      const int row = q / PADCH, c = q - row * PADCH;
      *reinterpret_cast<uint4*>(stage + C::K_BYTES + row * C::VP + (C::CH + c) * 16) = make_uint4(0, 0, 0, 0);
    }
  }
}

template <int D, int NIB>
__global__ __launch_bounds__(FWD_Q_ROWS / (32 * NIB) * 64) void attn_fwd_mfma_kernel(const el_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                            float* __restrict__ o32, el_t* __restrict__ o16, float* __restrict__ lse,
                                                            const AttnTile* __restrict__ tiles,
                                                            int Tn, int nq, int nkv, int causal, float scale_log2e) {
  constexpr int NT = FWD_Q_ROWS / (32 * NIB) * 64;   // threads: one wavefront per 32 * NIB query rows
  constexpr int WQ = 32 * NIB;
  using C = FwdCfg<D, NT>;
  constexpr int NDS = D / 16;        // contraction steps of Q K^T
  constexpr int NDB = C::DP / 32;    // 32-row blocks of O^T
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

  // Q fragments (B operand): column = query wq0 + ib*32 + li, k = ds*16 + h*8 .. +8.
  frag_t qf[NIB][NDS];
#pragma unroll
  for (int ib = 0; ib < NIB; ++ib) {
    const int i = wq0 + ib * 32 + li;
#pragma unroll
    for (int ds = 0; ds < NDS; ++ds) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (i < tl.r1) v = *reinterpret_cast<const uint4*>(qkv + (size_t)i * ld + qcol + ds * 16 + h * 8);
      qf[ib][ds] = __builtin_bit_cast(frag_t, v);
    }
  }

  floatx16 oacc[NDB][NIB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[db][ib][e] = 0.f;
  float m_run[NIB], l_run[NIB];
#pragma unroll
  for (int ib = 0; ib < NIB; ++ib) { m_run[ib] = -INFINITY; l_run[ib] = 0.f; }

  const int kv_end = causal ? tl.r1 : tl.s1;
  const int nsteps = (kv_end - tl.s0 + BKV - 1) / BKV;
  uint4 rk[C::PER_THREAD], rv[C::PER_THREAD];
  kv_load<D, NT>(rk, rv, qkv, ld, kcol, vcol, tl.s0, kv_end);
  kv_store<D, NT>(rk, rv, smem);
  __syncthreads();

  // The running maximum is a REFERENCE point only: the result is exact for any reference as long as
  // exp2(score - reference) stays in range.  A "fast" step keeps the reference fixed and never touches
  // the output accumulators except through MFMAs, so they stay in place in the accumulator registers;
  // it gives up (before changing any state) when a lane's sum of exp2(score - reference) over the step exceeds
  // LIMIT, which bounds every single one of them.  A "slow" step moves the reference to the new maximum and
  // rescales.  The first step of a wavefront is slow; with typical data nearly all the others are fast.
  constexpr float LIMIT = 4096.0f;
  // number of leading steps in which this wavefront has unmasked keys (the rest only move data)
  const int n_active = !wave_has_rows ? 0 : (causal ? min(nsteps, (wq0 + WQ - 1 - tl.s0) / BKV + 1) : nsteps);

  auto io_end = [&](int st) {
    if (st + 1 < nsteps) kv_store<D, NT>(rk, rv, smem + ((st + 1) & 1) * C::STAGE);
    __syncthreads();
  };
  // One key step.  RESCALE is a compile-time flag; returns false (fast step only) if the step must be
  // redone as a slow step: nothing but registers local to the step has been changed then.
  auto step = [&](int st, auto rescale_tag) -> bool {
    constexpr bool RESCALE = decltype(rescale_tag)::value;
    const int k0 = tl.s0 + st * BKV;
    const char* sk = smem + (st & 1) * C::STAGE;
    const char* sv = sk + C::K_BYTES;
    if (st + 1 < nsteps) kv_load<D, NT>(rk, rv, qkv, ld, kcol, vcol, k0 + BKV, kv_end);
    // S^T[jb][ib]: rows = keys k0 + jb*32 + .., columns = queries.  All K fragments of a 32-key block
    // are read before its MFMAs.
    floatx16 s[2][NIB];
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
      frag_t kfr[NDS];
#pragma unroll
      for (int ds = 0; ds < NDS; ++ds) {
        const uint4 kv4 = *reinterpret_cast<const uint4*>(sk + (jb * 32 + li) * C::KP + (ds * 2 + h) * 16);
        kfr[ds] = __builtin_bit_cast(frag_t, kv4);
      }
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[jb][ib][e] = 0.f;
#pragma unroll
        for (int ds = 0; ds < NDS; ++ds) s[jb][ib] = mfma16(kfr[ds], qf[ib][ds], s[jb][ib]);
      }
    }
    const bool need_mask = (causal && k0 + BKV - 1 > wq0) || (k0 + BKV > kv_end);
    if (need_mask) {
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) {
        const int i = wq0 + ib * 32 + li;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int j = k0 + jb * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
            float v = (j >= kv_end || (causal && j > i)) ? -INFINITY : s[jb][ib][e];
            asm volatile("" : "+v"(v));   // pins the select inside this (wave-uniform) branch
            s[jb][ib][e] = v;
          }
      }
    }
    if constexpr (RESCALE) {
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) {
        float mx = -INFINITY;   // maximum of the raw scores (the scale is positive)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
          for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[jb][ib][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run[ib], mx * scale_log2e);
        const float alpha = __builtin_amdgcn_exp2f(m_run[ib] - m_new);
        m_run[ib] = m_new;
        l_run[ib] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[db][ib][e] *= alpha;
      }
    }
    frag_t pf[NIB][2][2];   // [ib][jb][u]: probabilities of 16 keys as a B operand
    float ps[NIB];
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib) {
      ps[ib] = 0.f;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        float p[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          p[e] = __builtin_amdgcn_exp2f(fmaf(s[jb][ib][e], scale_log2e, -m_run[ib]));
          ps[ib] += p[e];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) pf[ib][jb][u] = pack8(p + u * 8);
      }
    }
    if constexpr (!RESCALE) {
      // The lane's sum bounds each of its terms, and it is needed anyway: no maximum over the scores and no exchange
      // between the halves of the wavefront on this path.
      bool over = false;
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) over = over || !(ps[ib] <= LIMIT);
      if (__any(over)) return false;
    }
#pragma unroll
    for (int ib = 0; ib < NIB; ++ib) l_run[ib] += ps[ib];
    // O^T[db][ib] += V^T P^T.  B-operand slot s of half h is key 16u + (s/4)*8 + h*4 + s%4 of the
    // 32-key block, so the matching V fragment is two transpose reads starting at keys h*4 and 8 + h*4.
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        frag_t vfr[NDB];
#pragma unroll
        for (int db = 0; db < NDB; ++db) vfr[db] = frag_cols_tr(sv, C::VP, jb * 32 + u * 16, db * 32, lane);
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int ib = 0; ib < NIB; ++ib)
            oacc[db][ib] = mfma16(vfr[db], pf[ib][jb][u], oacc[db][ib]);
      }
    io_end(st);
    return true;
  };

  int st = 0;
  while (st < n_active) {
    step(st, std::true_type{});
    ++st;
    while (st < n_active && step(st, std::false_type{})) ++st;
  }
  for (; st < nsteps; ++st) {      // steps that are fully masked for this wavefront: data movement only
    if (st + 1 < nsteps) kv_load<D, NT>(rk, rv, qkv, ld, kcol, vcol, tl.s0 + (st + 1) * BKV, kv_end);
    io_end(st);
  }

  // Finalise: the two halves of the wavefront hold disjoint key subsets of every query column.  The K/V stages are free
  // (every wavefront is past the last barrier): the output goes through this wavefront's part of them, see emit_block_rows.
  float* stage_out = reinterpret_cast<float*>(smem + wave * OUT_STAGE_BYTES);
#pragma unroll
  for (int ib = 0; ib < NIB; ++ib) {
    const int i = wq0 + ib * 32 + li;
    const float l_tot = l_run[ib] + __shfl_xor(l_run[ib], 32, 64);
    const float inv = 1.0f / l_tot;       // rows past the tile: never stored
    if (i < tl.r1 && h == 0) lse[(size_t)a * Tn + i] = (m_run[ib] + log2f(l_tot)) * 0.69314718055994531f;
    const int i_base = wq0 + ib * 32;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
      emit_block_rows(stage_out, oacc[db][ib], inv, lane, [&](int row, int c, float4 v) {
        const int ir = i_base + row, dd = db * 32 + c;
        if (ir >= tl.r1 || dd >= D) return;
        const size_t off = (size_t)ir * nq * D + qcol + dd;
        uint2 w;
        w.x = pack_bf16x2(v.x, v.y);
        w.y = pack_bf16x2(v.z, v.w);
        *reinterpret_cast<uint2*>(o + off) = w;
        if (o32) *reinterpret_cast<float4*>(o32 + off) = v;
        if (o16) {     // the copy the output projection reads (halves); the bf16 one above serves the weight gradient
          w.x = pack_f16x2(v.x, v.y);
          w.y = pack_f16x2(v.z, v.w);
          *reinterpret_cast<uint2*>(o16 + off) = w;
        }
      });
  }
}


// ------------------------------------------------------------------------------------------
// Backward.  Three kernels, no atomics; P and dS are formed once:
//   delta:  delta[a][i] = sum_d dO[i,a,d] * O[i,a,d]
//   dK/dV:  a workgroup owns 128 keys of one KV head (32 per wavefront, K and V fragments held
//           in registers) and walks the query heads of its group and the query rows in ascending
//           order; S = Q K^T and dP = dO V^T are computed UNtransposed so that a lane holds one
//           key column and P, dS are B operands of dV^T += dO^T P and dK^T += Q^T dS.  The dS
//           operand (IEEE halves, exactly what the dK product consumed) also goes to a scratch.
//   dQ:     (attn_mfma_dq.hip) streams that scratch: dQ^T += K^T dS^T, no recomputation.
// The scratch is block-linear: the 32 keys x 64 queries a wavefront handles in one step are one 4 KB block, written as
// four 1 KB stores, one per 16-row quarter (32-row half ib, 16-row half u) of the step: lane l stores 16 bytes, the dS
// of key l % 32 for the query rows 16u + 4 (l / 32) + {0..3} and 16u + 8 + 4 (l / 32) + {0..3} of half ib.  Blocks are
// indexed [query head][32-key block row][64-query step], rows and steps counted from the segment start (rows offset by
// the tile's kb0).  Every block a dQ wavefront reads has been written in full: masked entries hold the zeros the dK
// product saw.
// ------------------------------------------------------------------------------------------

template <int D>
__global__ __launch_bounds__(256) void attn_delta_mfma_kernel(const bf16_t* __restrict__ o, const float* __restrict__ o32,
                                                              const el_t* __restrict__ d_o, float* __restrict__ delta,
                                                              int Tn, int nq) {
  // 16 lanes per (token, head) pair, 8 elements per lane.
  const int pair = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int c = threadIdx.x & 15;
  float s = 0.f;
  if (pair < Tn * nq && c < D / 8) {
    float x[8], y[8];
    if (o32) {
      const float4 a0 = *reinterpret_cast<const float4*>(o32 + (size_t)pair * D + c * 8);
      const float4 a1 = *reinterpret_cast<const float4*>(o32 + (size_t)pair * D + c * 8 + 4);
      x[0] = a0.x; x[1] = a0.y; x[2] = a0.z; x[3] = a0.w; x[4] = a1.x; x[5] = a1.y; x[6] = a1.z; x[7] = a1.w;
    } else {
      load_vec<bf16_t>(o + (size_t)pair * D + c * 8, x);
    }
    load_vec<el_t>(d_o + (size_t)pair * D + c * 8, y);
#pragma unroll
    for (int e = 0; e < 8; ++e) s += x[e] * y[e];
  }
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) s += __shfl_xor(s, off, 64);
  if (c == 0 && pair < Tn * nq) {
    const int i = pair / nq, a = pair - i * nq;
    delta[(size_t)a * Tn + i] = s;
  }
}

constexpr int BQ_KV = 64;      // query rows per step of the dK/dV kernel
constexpr int WK = 32;         // keys per wavefront of the dK/dV kernel
constexpr int DKV_VALU_PER_MFMA = 8;    // vector instructions of the P / dS arithmetic issued after each MFMA of a group

// N_MFMA times (one MFMA, a share of the N_READS LDS reads, of the N_VMEM global loads and of the N_WRITES LDS
// writes, N_VALU vector instructions) in the instruction scheduler's order.  A wavefront issues in order, so
// whatever it issues in a run holds its MFMAs back: reads in one run fill its 16 outstanding-LDS-operation slots
// and then wait for the LDS, global loads in one run wait for the texture path (16 cycles per 1 KB instruction, and
// the four wavefronts of the workgroup arrive together).  One or two under each MFMA cost nothing.  The reads
// (fragments of the NEXT group) go under the first N_MFMA - 2 MFMAs.
template <int N_MFMA, int N_VALU, int N_READS, int N_VMEM = 0, int N_WRITES = 0, int I = 0>
__device__ __forceinline__ void interleave_mfma_valu() {
  if constexpr (I < N_MFMA) {
    // with LDS writes in the group (which the compiler must keep behind the reads: it cannot tell the two LDS
    // stages apart), the reads take the first half of the MFMAs and the writes the second
    constexpr int SPREAD = N_WRITES > 0 ? N_MFMA / 2 : (N_MFMA > 2 ? N_MFMA - 2 : 1);
    constexpr int R = I < SPREAD ? ((I + 1) * N_READS) / SPREAD - (I * N_READS) / SPREAD : 0;
    constexpr int G = ((I + 1) * N_VMEM) / N_MFMA - (I * N_VMEM) / N_MFMA;
    constexpr int WS = N_MFMA - SPREAD;
    constexpr int W = (N_WRITES > 0 && I >= SPREAD) ? ((I - SPREAD + 1) * N_WRITES) / WS - ((I - SPREAD) * N_WRITES) / WS : 0;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (R > 0) __builtin_amdgcn_sched_group_barrier(0x100, R, 0);
    if constexpr (G > 0) __builtin_amdgcn_sched_group_barrier(0x020, G, 0);
    if constexpr (W > 0) __builtin_amdgcn_sched_group_barrier(0x200, W, 0);
    if constexpr (N_VALU > 0) __builtin_amdgcn_sched_group_barrier(0x002, N_VALU, 0);
    interleave_mfma_valu<N_MFMA, N_VALU, N_READS, N_VMEM, N_WRITES, I + 1>();
  }
}

template <int D>
struct DkvCfg {
  static constexpr int DP = (D + 31) / 32 * 32;
  static constexpr int QP = 304;                     // Q and dO tiles: row and transposed fragments (as the K tile of the dQ kernel in attn_mfma_dq.hip)
  static constexpr int T_BYTES = BQ_KV * QP;
  static constexpr int STAGE = (2 * T_BYTES + 2 * BQ_KV * 4 + 255) / 256 * 256;   // Q, dO, lse2[64], delta[64]
  static constexpr int SMEM = 2 * STAGE;
};

template <int D>
__global__ __launch_bounds__(256) void attn_dkv_mfma_kernel(const el_t* __restrict__ qkv, const el_t* __restrict__ d_o,
                                                            const float* __restrict__ lse, const float* __restrict__ delta,
                                                            bf16_t* __restrict__ dqkv, const AttnTile* __restrict__ tiles,
                                                            int Tn, int nq, int nkv, int causal, float scale,
                                                            const float* __restrict__ grad_scale, el_t* __restrict__ ds,
                                                            int ds_rows, int ds_nqs, int n_sub, float* __restrict__ part) {
  using C = DkvCfg<D>;
  constexpr int NDS = D / 16, NDB = C::DP / 32;
  constexpr float LOG2E = 1.4426950408889634f;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const AttnTile tl = tiles[blockIdx.y];
  // n_sub > 1: the query heads of a KV head are dealt to n_sub workgroups (few KV heads and long causal tiles leave
  // the chip half empty otherwise); each writes its sums as an fp32 partial plane and dkv_combine_kernel adds the planes
  // in subset order.  G = query heads this workgroup walks, a0 = the first of them.
  const int b = blockIdx.x / n_sub, sub = blockIdx.x - b * n_sub;
  const int G = nq / nkv / n_sub, a0 = b * (nq / nkv) + sub * G;
  const int ld = (nq + 2 * nkv) * D;
  const int kcol = (nq + b) * D, vcol = (nq + nkv + b) * D;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: wave-level branches stay uniform
  const int h = lane >> 5, li = lane & 31;
  const int wj0 = tl.r0 + wave * WK;
  const int j = wj0 + li;                       // this lane's key column
  const bool wave_has_keys = wj0 < tl.r1;
  const float scale_log2e = scale * LOG2E;
  // dS scratch: this wavefront's block row; the block of a step and the query head are added per step
  const int ds_krow = tl.kb0 + ((wj0 - tl.s0) >> 5);
  el_t* ds_head = ds;

  frag_t kf[NDS], vf[NDS];
#pragma unroll
  for (int ds = 0; ds < NDS; ++ds) {
    uint4 v = make_uint4(0, 0, 0, 0), w = v;
    if (j < tl.r1) {
      v = *reinterpret_cast<const uint4*>(qkv + (size_t)j * ld + kcol + ds * 16 + h * 8);
      w = *reinterpret_cast<const uint4*>(qkv + (size_t)j * ld + vcol + ds * 16 + h * 8);
    }
    kf[ds] = __builtin_bit_cast(frag_t, v);
    vf[ds] = __builtin_bit_cast(frag_t, w);
    // MFMA operands only from here on: keep them in the accumulation half of the register file, which has
    // room, so that the fragment sets and the tile in flight fit in the other half without spilling
    asm volatile("" : "+a"(kf[ds]), "+a"(vf[ds]));
  }
  floatx16 dk[NDB], dv[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[db][e] = 0.f; dv[db][e] = 0.f; }

  const int q_begin = causal ? tl.r0 : tl.s0;
  const int nq_steps = (tl.s1 - q_begin + BQ_KV - 1) / BQ_KV;
  const int nsteps = G * nq_steps;
  uint4 rq[TileRegs<D, BQ_KV>::N], rd[TileRegs<D, BQ_KV>::N];
  float r_stat = 0.f;

  // Rows past the end of the segment repeat its last row (finite values): P and dS are exactly zero there.
  auto fetch_q = [&](int step) {
    const int a = a0 + step / nq_steps;
    const int q0 = q_begin + (step % nq_steps) * BQ_KV;
    tile_load_clamped<D, BQ_KV>(rq, qkv + a * D, ld, q0, tl.s1);
  };
  auto fetch_d = [&](int step) {
    const int a = a0 + step / nq_steps;
    const int q0 = q_begin + (step % nq_steps) * BQ_KV;
    tile_load_clamped<D, BQ_KV>(rd, d_o + a * D, nq * D, q0, tl.s1);
    // row statistics: threads 0..63 bring lse, 64..127 delta, the upper half of the workgroup the same again
    const int i = min(q0 + (int)(threadIdx.x & (BQ_KV - 1)), tl.s1 - 1);
    const bool is_dl = (threadIdx.x & BQ_KV) != 0;
    r_stat = (is_dl ? delta : lse)[(size_t)a * Tn + i];       // used (scaled) only in commit: no wait for it here
  };
  auto fetch = [&](int step) { fetch_q(step); fetch_d(step); };
  auto commit = [&](char* stage) {
    tile_store<D, BQ_KV, C::QP, C::DP, 256, true>(rq, stage);
    tile_store<D, BQ_KV, C::QP, C::DP, 256, true>(rd, stage + C::T_BYTES);
    reinterpret_cast<float*>(stage + 2 * C::T_BYTES)[threadIdx.x & (2 * BQ_KV - 1)] =
        r_stat * ((threadIdx.x & BQ_KV) ? 1.f : LOG2E);      // both halves of the workgroup write the same values
  };
  fetch(0);
  commit(smem);
  __syncthreads();

  // One 64-row query step is eight groups of MFMAs over its two 32-row blocks:
  //   S,dP(0) halves | S,dP(1) halves + arithmetic(0) | dV,dK(0) halves + arithmetic(1) | dV,dK(1) halves
  // (S,dP halved over the head dimension, dV,dK over the 16-row halves of the block).  There is one
  // wavefront per SIMD, so nothing but this wavefront's own instruction stream can fill the MFMA pipe:
  // every group issues the LDS fragment reads of the NEXT group under its own MFMAs (two fragment sets
  // alive, used in turn), and the P / dS arithmetic of a 16-row half (quarter-rate exponentials
  // included) issues between the MFMAs of a group that does not depend on it.  The next tile's global loads
  // are issued one under each MFMA of the first two groups and go to LDS under the MFMAs of the seventh; the
  // step's one barrier sits between the last two groups, under MFMAs in flight; the last group reads the
  // first fragments of the step after, from the other LDS stage.
  // MASK is a compile-time flag so that each variant of the step is one basic block.
  constexpr int NH0 = (NDS + 1) / 2, NH1 = NDS - NH0;      // head-dimension slices of 16 in the two halves
  constexpr int FS = NH0 > NDB ? NH0 : NDB;
  struct FragSet { frag_t a[FS], b[FS]; };                // (Q, dO) row fragments or (dO^T, Q^T) transposed ones
  FragSet fx;                                              // carried from step to step: rows of block 0, first half
  auto load_rows = [&](const char* sq, const char* sd, int ib, int half, FragSet& f) {
#pragma unroll
    for (int i = 0; i < (half ? NH1 : NH0); ++i) {
      f.a[i] = frag_rows(sq, C::QP, ib * 32, half * NH0 + i, lane);
      f.b[i] = frag_rows(sd, C::QP, ib * 32, half * NH0 + i, lane);
    }
  };
  auto compute_step = [&](const char* sq, const char* sd, const float* s_lse, const float* s_dl, int q0, int next_step,
                          char* next_stage, auto mask_tag) {
    constexpr bool MASK = decltype(mask_tag)::value;
    el_t* ds_block = ds_head + ((size_t)ds_krow * ds_nqs + ((q0 - tl.s0) >> 6)) * 2048 + lane * 8;
    floatx16 sacc[2], dpacc[2];
    frag_t pf[2][2], dsf[2][2];
    FragSet fy;
    auto load_tr = [&](int ib, int u, FragSet& f) {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        f.a[db] = frag_cols_tr(sd, C::QP, ib * 32 + u * 16, db * 32, lane);
        f.b[db] = frag_cols_tr(sq, C::QP, ib * 32 + u * 16, db * 32, lane);
      }
    };
    auto sdp = [&](int ib, int half, const FragSet& f) {
      if (half == 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[ib][e] = 0.f; dpacc[ib][e] = 0.f; }
      }
#pragma unroll
      for (int i = 0; i < (half ? NH1 : NH0); ++i) {
        sacc[ib] = mfma16(f.a[i], kf[half * NH0 + i], sacc[ib]);
        dpacc[ib] = mfma16(f.b[i], vf[half * NH0 + i], dpacc[ib]);
      }
    };
    // Row statistics of a 16-row half: read one group ahead of the arithmetic that uses them (LDS reads return in
    // order, so a read issued behind a group's fragment reads would make the arithmetic wait for all of those).
    struct Stats { float4 l[2], d[2]; };
    Stats sx, sy;
    auto stat_load = [&](int ib, int u, Stats& st) {
#pragma unroll
      for (int gg = 0; gg < 2; ++gg) {
        const int il = ib * 32 + (u * 2 + gg) * 8 + h * 4;
        st.l[gg] = *reinterpret_cast<const float4*>(s_lse + il);
        st.d[gg] = *reinterpret_cast<const float4*>(s_dl + il);
      }
    };
    auto arith = [&](int ib, int u, const Stats& st) {
      // accumulator value e belongs to row ib*32 + (e/4)*8 + h*4 + e%4; half u holds e = 8u .. 8u+7
      float pv[8], dsv[8];
#pragma unroll
      for (int gg = 0; gg < 2; ++gg) {
        const int g = u * 2 + gg;
        const int il = ib * 32 + g * 8 + h * 4;
        const float4 l4 = st.l[gg], d4 = st.d[gg];
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int e = g * 4 + c;
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[ib][e], scale_log2e, -lv[c]));
          if (MASK) {
            const int i = q0 + il + c;
            p = (i >= tl.s1 || j >= tl.r1 || (causal && j > i)) ? 0.f : p;
          }
          pv[gg * 4 + c] = p;
          dsv[gg * 4 + c] = p * (dpacc[ib][e] - dl4[c]);    // masked entries: P = 0 and dP finite, so dS = 0
        }
      }
      pf[ib][u] = pack8(pv);
      dsf[ib][u] = pack8(dsv);
      // the dQ kernel's copy: 16 bytes per lane = this key's dS for query rows 16u + h*4 .. +3 and 16u + 8 + h*4 .. +3
      // of half ib; streamed past the caches (read once, by another kernel)
      typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
      __builtin_nontemporal_store(__builtin_bit_cast(u32x4, dsf[ib][u]), reinterpret_cast<u32x4*>(ds_block + (ib * 2 + u) * 512));
    };
    auto dvdk = [&](int ib, int u, const FragSet& f) {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        dv[db] = mfma16(f.a[db], pf[ib][u], dv[db]);
        dk[db] = mfma16(f.b[db], dsf[ib][u], dk[db]);
      }
    };
    // Order inside a group: one MFMA, a few LDS reads, a handful of vector instructions, and again.
    auto group_order = [&](auto n_reads, auto n_mfma, auto n_valu, auto n_vmem, auto n_writes) {
      interleave_mfma_valu<decltype(n_mfma)::value, decltype(n_valu)::value, decltype(n_reads)::value, decltype(n_vmem)::value,
                           decltype(n_writes)::value>();
      __builtin_amdgcn_sched_barrier(0);
    };
    constexpr int V = DKV_VALU_PER_MFMA;
#define RRFP_IC(x) std::integral_constant<int, (x)>{}
    constexpr int NLD = TileRegs<D, BQ_KV>::N;       // global loads per thread and tile (Q, dO alike)
    // S,dP of block 0; the next tile's global loads (after the last step: the same tile again, never used), one
    // under each MFMA
    fetch_q(min(next_step, nsteps - 1));
    load_rows(sq, sd, 0, 1, fy);
    sdp(0, 0, fx);
    group_order(RRFP_IC(2 * NH1), RRFP_IC(2 * NH0), RRFP_IC(0), RRFP_IC(NLD), RRFP_IC(0));
    fetch_d(min(next_step, nsteps - 1));
    load_rows(sq, sd, 1, 0, fx);
    stat_load(0, 0, sx);
    sdp(0, 1, fy);
    group_order(RRFP_IC(2 * NH0 + 4), RRFP_IC(2 * NH1), RRFP_IC(0), RRFP_IC(NLD + 1), RRFP_IC(0));
    // S,dP of block 1 with the arithmetic of block 0
    load_rows(sq, sd, 1, 1, fy);
    stat_load(0, 1, sy);
    sdp(1, 0, fx);
    arith(0, 0, sx);
    group_order(RRFP_IC(2 * NH1 + 4), RRFP_IC(2 * NH0), RRFP_IC(V), RRFP_IC(0), RRFP_IC(0));
    load_tr(0, 0, fx);
    stat_load(1, 0, sx);
    sdp(1, 1, fy);
    arith(0, 1, sy);
    group_order(RRFP_IC(4 * NDB + 4), RRFP_IC(2 * NH1), RRFP_IC(V), RRFP_IC(0), RRFP_IC(0));
    // dV,dK of block 0 with the arithmetic of block 1
    load_tr(0, 1, fy);
    stat_load(1, 1, sy);
    dvdk(0, 0, fx);
    arith(1, 0, sx);
    group_order(RRFP_IC(4 * NDB + 4), RRFP_IC(2 * NDB), RRFP_IC(V), RRFP_IC(0), RRFP_IC(0));
    load_tr(1, 0, fx);
    dvdk(0, 1, fy);
    arith(1, 1, sy);
    group_order(RRFP_IC(4 * NDB), RRFP_IC(2 * NDB), RRFP_IC(V), RRFP_IC(0), RRFP_IC(0));
    // dV,dK of block 1; the next tile goes to LDS under the MFMAs of its first half
    load_tr(1, 1, fy);
    commit(next_stage);
    dvdk(1, 0, fx);
    group_order(RRFP_IC(4 * NDB), RRFP_IC(2 * NDB), RRFP_IC(0), RRFP_IC(0), RRFP_IC(2 * NLD + 1));
    __syncthreads();
    load_rows(next_stage, next_stage + C::T_BYTES, 0, 0, fx);   // stale data after the last step: read, never used
    dvdk(1, 1, fy);
    group_order(RRFP_IC(2 * NH0), RRFP_IC(2 * NDB), RRFP_IC(0), RRFP_IC(0), RRFP_IC(0));
#undef RRFP_IC
  };

  // Steps are (query head of the group, 64-row query block) pairs in ascending order.  Under a causal
  // mask the first n_skip blocks of every head lie wholly before this wavefront's keys: those steps
  // only move data.  The MFMA accumulators are touched in the second loop alone and unconditionally,
  // so they stay in place in the accumulator registers for the whole kernel.
  const int n_skip = !wave_has_keys ? nq_steps : (causal ? min(nq_steps, (wj0 - q_begin) / BQ_KV) : 0);
  const bool ragged_keys = wj0 + WK > tl.r1;
  const int t_lead_end = ragged_keys ? nq_steps
                         : (causal ? min(nq_steps, max(n_skip, (wj0 + WK - 1 - q_begin + BQ_KV - 1) / BQ_KV)) : n_skip);
  const int t_tail_begin = (q_begin + nq_steps * BQ_KV > tl.s1) ? nq_steps - 1 : nq_steps;
  auto run_steps = [&](int t, int t_end, int& st, auto mask_tag) -> int {
    if (t < t_end) load_rows(smem + (st & 1) * C::STAGE, smem + (st & 1) * C::STAGE + C::T_BYTES, 0, 0, fx);
    for (; t < t_end; ++t, ++st) {
      const int q0 = q_begin + t * BQ_KV;
      const char* sq = smem + (st & 1) * C::STAGE;
      const char* sd = sq + C::T_BYTES;
      const float* s_lse = reinterpret_cast<const float*>(sq + 2 * C::T_BYTES);
      const float* s_dl = s_lse + BQ_KV;
      compute_step(sq, sd, s_lse, s_dl, q0, st + 1, smem + ((st + 1) & 1) * C::STAGE, mask_tag);
    }
    return t;
  };
  int st = 0;
  for (int ah = 0; ah < G; ++ah) {
    ds_head = ds + (size_t)(a0 + ah) * ds_rows * ds_nqs * 2048;
    int t = 0;
    for (; t < n_skip; ++t, ++st) {
      if (st + 1 < nsteps) { fetch(st + 1); commit(smem + ((st + 1) & 1) * C::STAGE); }
      __syncthreads();
    }
    // Masked steps come first (the diagonal of a causal segment, or every step when this wavefront's
    // key block is ragged), then the unmasked bulk, then the ragged last query block: three loops, each
    // with one compile-time variant of the step, so no loop mixes register assignments.
    t = run_steps(t, t_lead_end, st, std::true_type{});
    t = run_steps(t, max(t, t_tail_begin), st, std::false_type{});
    t = run_steps(t, nq_steps, st, std::true_type{});
  }
  {
    const float inv_s = grad_scale ? grad_scale[1] : 1.0f;     // d_o held s * dO: undo it (a power of two: exact)
    scale *= inv_s;
    __syncthreads();      // nobody reads the tile stages any more: they stage the output (emit_block_rows)
    float* st = reinterpret_cast<float*>(smem + wave * OUT_STAGE_BYTES);
    auto put = [&](const floatx16& acc, float mul, int col, int db) {
      emit_block_rows(st, acc, mul, lane, [&](int row, int c, float4 v) {
        const int jr = wj0 + row, dd = db * 32 + c;
        if (jr >= tl.r1 || dd >= D) return;
        uint2 w;
        w.x = pack_bf16x2(v.x, v.y);
        w.y = pack_bf16x2(v.z, v.w);
        *reinterpret_cast<uint2*>(dqkv + (size_t)jr * ld + col + dd) = w;
      });
    };
    // partial plane [tensor][subset][token][KV head * D + d], unscaled (dkv_combine_kernel scales the sum)
    auto put_part = [&](const floatx16& acc, int tensor, int db) {
      float* plane = part + ((size_t)(tensor * n_sub + sub) * Tn) * (nkv * D);
      emit_block_rows(st, acc, 1.0f, lane, [&](int row, int c, float4 v) {
        const int jr = wj0 + row, dd = db * 32 + c;
        if (jr >= tl.r1 || dd >= D) return;
        *reinterpret_cast<float4*>(plane + (size_t)jr * (nkv * D) + b * D + dd) = v;
      });
    };
    if (n_sub > 1) {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        put_part(dk[db], 0, db);
        put_part(dv[db], 1, db);
      }
    } else {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        put(dk[db], scale, kcol, db);
        put(dv[db], inv_s, vcol, db);
      }
    }
  }
}

// dk, dv = the sum of the n_sub partial planes in subset order, scaled, rounded to bf16 into the K and V columns of dqkv.
// One thread per 4 values of a [T, nkv * D] plane.
__global__ __launch_bounds__(256) void dkv_combine_kernel(const float* __restrict__ part, bf16_t* __restrict__ dqkv, int Tn, int nq,
                                                          int nkv, int D, int n_sub, float scale, const float* __restrict__ grad_scale) {
  const int W = nkv * D;
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (idx >= (size_t)Tn * W) return;
  const int j = (int)(idx / W), c = (int)(idx - (size_t)j * W);
  const float inv_s = grad_scale ? grad_scale[1] : 1.0f;
  const int ld = (nq + 2 * nkv) * D;
#pragma unroll
  for (int tensor = 0; tensor < 2; ++tensor) {
    float4 acc = *reinterpret_cast<const float4*>(part + ((size_t)(tensor * n_sub) * Tn) * W + idx);
    for (int sub = 1; sub < n_sub; ++sub) {
      const float4 v = *reinterpret_cast<const float4*>(part + ((size_t)(tensor * n_sub + sub) * Tn) * W + idx);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const float mul = tensor == 0 ? scale * inv_s : inv_s;
    uint2 w;
    w.x = pack_bf16x2(acc.x * mul, acc.y * mul);
    w.y = pack_bf16x2(acc.z * mul, acc.w * mul);
    *reinterpret_cast<uint2*>(dqkv + (size_t)j * ld + (nq + tensor * nkv) * D + c) = w;
  }
}

// Compute units of the current device (cached per device id; 256 if the query fails).
inline int attn_cu_count() {
  static int cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
    cached[dev] = v;
  }
  return cached[dev];
}

template <int D>
hipError_t bwd_launch(const AttnArgs& a, hipStream_t s) {
  auto kkv = attn_dkv_mfma_kernel<D>;
  static std::once_flag once;
  static hipError_t once_status = hipSuccess;
  if (hipError_t e = set_max_dynamic_lds_once(once, once_status, (const void*)kkv, DkvCfg<D>::SMEM); e != hipSuccess) return e;
  const float scale = 1.0f / sqrtf((float)D);
  hipLaunchKernelGGL(attn_delta_mfma_kernel<D>, dim3((a.T * a.nq + 15) / 16), dim3(256), 0, s, (const bf16_t*)a.o,
                     a.o32, (const el_t*)a.d_o, a.delta, a.T, a.nq);
  const int n_sub = a.dkv_part ? attn_dkv_subsets(a.nq, a.nkv, a.n_kv_tiles, attn_cu_count()) : 1;
  hipLaunchKernelGGL(kkv, dim3(a.nkv * n_sub, a.n_kv_tiles), dim3(256), DkvCfg<D>::SMEM, s, (const el_t*)a.qkv,
                     (const el_t*)a.d_o, a.lse, a.delta, (bf16_t*)a.dqkv, a.kv_tiles, a.T, a.nq, a.nkv, a.causal, scale, a.grad_scale,
                     (el_t*)a.ds, a.ds_rows, a.ds_nqs, n_sub, a.dkv_part);
  if (n_sub > 1) {
    const size_t n4 = (size_t)a.T * a.nkv * D / 4;
    hipLaunchKernelGGL(dkv_combine_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, a.dkv_part, (bf16_t*)a.dqkv, a.T, a.nq,
                       a.nkv, D, n_sub, scale, a.grad_scale);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_attn_dq_mfma(a, s);
}

template <int D>
hipError_t fwd_launch(const AttnArgs& a, hipStream_t s) {
  constexpr int NT = FWD_Q_ROWS / (32 * FWD_NIB) * 64;
  using C = FwdCfg<D, NT>;
  auto kern = attn_fwd_mfma_kernel<D, FWD_NIB>;
  static std::once_flag once;
  static hipError_t once_status = hipSuccess;
  if (hipError_t e = set_max_dynamic_lds_once(once, once_status, (const void*)kern, C::SMEM); e != hipSuccess) return e;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  hipLaunchKernelGGL(kern, dim3(a.nq, a.n_q_tiles), dim3(NT), C::SMEM, s, (const el_t*)a.qkv, (bf16_t*)a.o, a.o32, (el_t*)a.o16, a.lse,
                     a.q_tiles, a.T, a.nq, a.nkv, a.causal, scale_log2e);
  return hipGetLastError();
}

}  // namespace

bool attn_mfma_supports(const AttnArgs& a) {
  return a.dtype == BF16 && (a.d == 64 || a.d == 80 || a.d == 128) && a.n_q_tiles >= 1;
}

hipError_t launch_attn_fwd_mfma(const AttnArgs& a, hipStream_t s) {
  if (!attn_mfma_supports(a)) return hipErrorInvalidValue;
  if (a.d == 64) return fwd_launch<64>(a, s);
  if (a.d == 80) return fwd_launch<80>(a, s);
  return fwd_launch<128>(a, s);
}

hipError_t launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t s) {
  if (!attn_mfma_supports(a) || a.n_kv_tiles < 1 || !a.ds || a.ds_rows < 1 || a.ds_nqs < 5) return hipErrorInvalidValue;
  if (a.d == 64) return bwd_launch<64>(a, s);
  if (a.d == 80) return bwd_launch<80>(a, s);
  return bwd_launch<128>(a, s);
}

}  // namespace rrfp
