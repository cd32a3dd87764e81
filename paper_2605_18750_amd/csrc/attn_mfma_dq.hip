// dQ kernel of the MFMA attention backward (see attn_mfma.hip for the scheme): dQ^T += K^T dS^T, with dS read back
// from the scratch the dK/dV kernel filled, so that neither the scores nor dP are formed a second time.
//
// A workgroup (8 wavefronts) owns one query tile (up to 256 rows inside one segment) of one query head; a wavefront
// owns 32 query rows = one 32-row half of a 64-query step of the scratch.  Keys advance in steps of 128: the K tile of
// a step goes through LDS (shared by the wavefronts, two stages), the wavefront's own dS -- four blocks of 32 keys, 2 KB
// each, contiguous in the scratch -- through a private LDS area, and both operands of an MFMA come from the LDS
// transpose read: the scratch holds, per key, four consecutive queries in 8 bytes, which is the unit that read
// transposes.  Under a causal mask a wavefront contracts only over the 32-key blocks that hold a key at or before its
// last query; those are exactly the blocks the dK/dV kernel wrote for its query step, zeros included, so nothing is
// masked here.  The kernel is bound by the stream of dS out of memory (no reuse: it is read past the caches); loads
// run two steps ahead in two register sets.
#include "attn_mfma_common.h"

namespace rrfp {
namespace {

constexpr int DQ_BK = 128;       // keys per step

template <int D>
struct DqCfg {
  static constexpr int DP = (D + 31) / 32 * 32;
  static constexpr int KP = 304;                        // K tile row pitch in bytes; 304 = 48 (mod 256): the four rows of 32 B a
                                                        // transposed read touches land on distinct banks
  static constexpr int K_STAGE = (DQ_BK * KP + 255) / 256 * 256;
  static constexpr int DS_HALF = 512 + 64;              // 32 lanes x 16 B of a scratch store, then 64 B of padding so that the
                                                        // two halves of a store land on different banks
  static constexpr int DS_PAIR = 2 * DS_HALF;           // one 1 KB store of the dK/dV kernel
  static constexpr int DS_BLOCK = 2 * DS_PAIR;          // this wavefront's 32 queries of one 32-key block
  static constexpr int DS_WAVE = (DQ_BK / 32) * DS_BLOCK;
  static constexpr int SMEM = 2 * K_STAGE + 8 * DS_WAVE;
};

template <int D>
__global__ __launch_bounds__(512) void attn_dq_mfma_kernel(const el_t* __restrict__ qkv, const el_t* __restrict__ ds,
                                                           bf16_t* __restrict__ dqkv, const AttnTile* __restrict__ tiles,
                                                           int nq, int nkv, int causal, float scale,
                                                           const float* __restrict__ grad_scale, int ds_rows, int ds_nqs) {
  using C = DqCfg<D>;
  constexpr int NT = 512, NDB = C::DP / 32, NBLK = DQ_BK / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const AttnTile tl = tiles[blockIdx.y];
  const int a = blockIdx.x, b = a / (nq / nkv);
  const int ld = (nq + 2 * nkv) * D;
  const int qcol = a * D, kcol = (nq + b) * D;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: wave-level branches stay uniform
  const int h = lane >> 5, li = lane & 31;
  const int wq0 = tl.r0 + wave * 32;
  const bool wave_has_rows = wq0 < tl.r1;
  const int kv_end = causal ? tl.r1 : tl.s1;
  const int nsteps = (kv_end - tl.s0 + DQ_BK - 1) / DQ_BK;
  // 32-key blocks this wavefront contracts over: all that hold a key, under a causal mask those with a key at or
  // before its last query (wq0 - s0 is a multiple of 32)
  const int nblk_all = (kv_end - tl.s0 + 31) / 32;
  const int nblk = !wave_has_rows ? 0 : (causal ? min(nblk_all, ((wq0 - tl.s0) >> 5) + 1) : nblk_all);
  // this lane's 16 bytes of the first store of block row 0; the second store is 1 KB on, the next block row
  // ds_nqs blocks on
  const el_t* ds_wave = ds + (((size_t)a * ds_rows + tl.kb0) * ds_nqs + ((wq0 - tl.s0) >> 6)) * 2048 +
                        (((wq0 - tl.s0) >> 5) & 1) * 1024 + lane * 8;
  const size_t ds_row_stride = (size_t)ds_nqs * 2048;

  floatx16 acc[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[db][e] = 0.f;

  // two register sets: the loads of steps st + 1 and st + 2 are in flight while step st is computed
  struct Regs { uint4 rk[TileRegs<D, DQ_BK, NT>::N]; uint4 rd[NBLK][2]; };
  Regs ra, rb;
  char* dsw = smem + 2 * C::K_STAGE + wave * C::DS_WAVE;
  auto fetch = [&](int st, Regs& r) {
    tile_load<D, DQ_BK, NT>(r.rk, qkv + kcol, ld, tl.s0 + st * DQ_BK, kv_end);
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
      // no branch: a block past this wavefront's last one re-reads that one (never used)
      const int kb = min(st * NBLK + blk, max(nblk - 1, 0));
      typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
      const el_t* p = ds_wave + (size_t)kb * ds_row_stride;
      r.rd[blk][0] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
      r.rd[blk][1] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + 512)));
    }
  };
  auto commit = [&](int st, const Regs& r) {
    tile_store<D, DQ_BK, C::KP, C::DP, NT>(r.rk, smem + (st & 1) * C::K_STAGE);
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
      if (st * NBLK + blk < nblk) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
          *reinterpret_cast<uint4*>(dsw + blk * C::DS_BLOCK + u * C::DS_PAIR + h * C::DS_HALF + li * 16) = r.rd[blk][u];
      }
    }
  };
  // The private dS area is written and read by this wavefront alone, and the hardware executes one wavefront's LDS
  // instructions in order; these wavefront-scope fences keep the compiler from moving the next step's writes above
  // this step's reads.
  auto wave_sync = [] {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  // The dS^T fragment (B operand: column = query, k = keys) by the LDS transpose read, with the lane roles of
  // frag_cols_tr: a lane names the 8-byte unit (key row, four queries) it contributes.  Query group qg = queries
  // 4 qg .. 4 qg + 3 of the wavefront's 32 sits in store qg / 4, half qg % 2 of the lanes, bytes 8 ((qg / 2) % 2) .. of the
  // lane's 16.
  const int tr_krow = h * 4 + ((lane & 15) >> 2);
  const int tr_qg = ((lane >> 4) & 1) * 4 + (lane & 3);
  const int tr_off = (tr_qg >> 2) * C::DS_PAIR + (tr_qg & 1) * C::DS_HALF + ((tr_qg >> 1) & 1) * 8 + tr_krow * 16;
  auto compute = [&](int st) {
    const char* sk = smem + (st & 1) * C::K_STAGE;
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
      if (st * NBLK + blk < nblk) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {          // 16 keys each
          const char* p = dsw + blk * C::DS_BLOCK + tr_off + s2 * 256;
          union { short4v hh[2]; frag_t v; } f;
          f.hh[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)p);
          f.hh[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(p + 128));
          frag_t ktr[NDB];
#pragma unroll
          for (int db = 0; db < NDB; ++db) ktr[db] = frag_cols_tr(sk, C::KP, blk * 32 + s2 * 16, db * 32, lane);
#pragma unroll
          for (int db = 0; db < NDB; ++db) acc[db] = mfma16(ktr[db], f.v, acc[db]);
        }
      }
    }
    wave_sync();
  };
  fetch(0, ra);
  commit(0, ra);
  __syncthreads();
  if (1 < nsteps) fetch(1, ra);
  if (2 < nsteps) fetch(2, rb);
  for (int st = 0; st < nsteps; st += 2) {
    compute(st);
    if (st + 1 < nsteps) commit(st + 1, ra);
    __syncthreads();
    if (st + 3 < nsteps) fetch(st + 3, ra);
    if (st + 1 < nsteps) {
      compute(st + 1);
      if (st + 2 < nsteps) commit(st + 2, rb);
      __syncthreads();
      if (st + 4 < nsteps) fetch(st + 4, rb);
    }
  }
  // the K stages are free (every wavefront is past the last barrier): the output goes through this wavefront's part
  // of them, see emit_block_rows
  const float out_scale = scale * (grad_scale ? grad_scale[1] : 1.0f);    // d_o held s * dO: undo it (a power of two: exact)
  float* st = reinterpret_cast<float*>(smem + wave * OUT_STAGE_BYTES);
#pragma unroll
  for (int db = 0; db < NDB; ++db)
    emit_block_rows(st, acc[db], out_scale, lane, [&](int row, int c, float4 v) {
      const int ir = wq0 + row, dd = db * 32 + c;
      if (ir >= tl.r1 || dd >= D) return;
      uint2 w;
      w.x = pack_bf16x2(v.x, v.y);
      w.y = pack_bf16x2(v.z, v.w);
      *reinterpret_cast<uint2*>(dqkv + (size_t)ir * ld + qcol + dd) = w;
    });
}

template <int D>
hipError_t dq_launch(const AttnArgs& a, hipStream_t s) {
  auto kq = attn_dq_mfma_kernel<D>;
  static std::once_flag once;
  static hipError_t once_status = hipSuccess;
  if (hipError_t e = set_max_dynamic_lds_once(once, once_status, (const void*)kq, DqCfg<D>::SMEM); e != hipSuccess) return e;
  const float scale = 1.0f / sqrtf((float)D);
  hipLaunchKernelGGL(kq, dim3(a.nq, a.n_q_tiles), dim3(512), DqCfg<D>::SMEM, s, (const el_t*)a.qkv, (const el_t*)a.ds,
                     (bf16_t*)a.dqkv, a.q_tiles, a.nq, a.nkv, a.causal, scale, a.grad_scale, a.ds_rows, a.ds_nqs);
  return hipGetLastError();
}

}  // namespace

// Needs the dK/dV kernel (which fills a.ds) on the same stream before it; writes the dq columns of a.dqkv.
hipError_t launch_attn_dq_mfma(const AttnArgs& a, hipStream_t s) {
  if (!a.ds) return hipErrorInvalidValue;
  if (a.d == 64) return dq_launch<64>(a, s);
  if (a.d == 80) return dq_launch<80>(a, s);
  if (a.d == 128) return dq_launch<128>(a, s);
  return hipErrorInvalidValue;
}

}  // namespace rrfp
