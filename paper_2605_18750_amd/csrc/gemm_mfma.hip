// bf16 MFMA GEMM for gfx950: C[M,N] = A(m,k) B(k,n) (+R), fp32 accumulation, bf16 or fp32 out.
//
// Two kernels share the tile geometry (a workgroup owns a 256-wide tile of C):
//
//   gemm_mfma_dl_kernel  the main kernel.  8 wavefronts (2 x 4, 128 x 64 of C each), accumulators of
//     v_mfma_f32_16x16x32_bf16.  K advances in 32-deep steps through a ring of five LDS buffers that
//     are filled by direct global->LDS loads, issued for pairs of steps (so that both 64-byte halves of
//     a 128-byte line of a K-contiguous operand reach L2 as one request) and spread between the MFMAs;
//     epilogue staged through LDS so that all stores, residual loads and activation-operand loads are
//     row-contiguous; optional fused residual / bias / SwiGLU / GELU forward and backward epilogues; a
//     128-row tile variant and a split-K mode for grids that do not fill the CUs.
//   gemm_mfma_kernel     the fallback for K-contiguous operands whose K is not a multiple of 32: four
//     wavefronts, v_mfma_f32_32x32x16_bf16, 64-deep steps, two LDS stages filled through registers.
//
// Operand tiles sit in LDS in their memory orientation, so every global load is a coalesced
// 16-byte access:
//   K-contiguous operand ([rows][K] in memory): rows of 16-byte chunks, XOR-swizzled so that the lanes
//     one ds_read_b128 pass serves fall into distinct bank groups; a fragment (8 consecutive k of one
//     row) is one ds_read_b128.
//   K-strided operand ([K][rows] in memory): LDS [k][256 rows], chunks XOR-swizzled by k; a fragment is
//     two ds_read_b64_tr_b16, the LDS transpose read of gfx950 that hands each lane 4 consecutive k of
//     one row out of a 4(k) x 16(rows) block.
// The forward GEMMs use (A K-contiguous, B K-strided), the input-gradient GEMMs (both
// K-contiguous), the weight-gradient GEMMs (both K-strided, K = tokens).
//
// The MFMA is issued with the B fragment as its first operand, so a lane's four consecutive
// accumulator values are four consecutive columns of one row of C.  Rows beyond M, columns beyond N
// and k beyond K are zero-filled on load and masked on store.  The k loop order, the tile partition,
// the choice of 128-row tiles and the split-K factor depend only on the shape and on the device's CU
// count, never on what else is running, so a given call always sums in the same order.
#include <algorithm>
#include <type_traits>

#include "kernels.h"
#include "numeric.h"

namespace rrfp {
namespace {

constexpr int BM = 256, BN = 256, BK = 64, NTHREADS = 256;
constexpr int TILE_BYTES = 256 * 64 * 2;          // one operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;       // A + B
constexpr int SMEM_BYTES = 2 * STAGE_BYTES;       // two stages

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;

// Byte offset of the 16-byte chunk (row, c) of a K-contiguous tile [256][64].
__device__ __forceinline__ int kc_off(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }
// Byte offset of the 16-byte chunk (k, c) of a K-strided tile [64][256]; c in 0..31.
__device__ __forceinline__ int ks_off(int k, int c) {
  const int f = (k & 3) | (((k >> 3) & 1) << 2);
  return k * 512 + (((((c >> 2) ^ f) << 2) | (c & 3)) << 4);
}

// Global -> registers for one operand tile: 8 chunks of 16 bytes per thread.
template <bool KC>
__device__ __forceinline__ void load_tile(uint4 (&r)[8], const bf16_t* __restrict__ base, int ld, int outer0,
                                          int outer_n, int k0, int K) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int q = i * NTHREADS + t;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (KC) {
      const int row = q >> 3, c = q & 7;
      const int go = outer0 + row, gk = k0 + c * 8;
      if (go < outer_n && gk < K) v = *reinterpret_cast<const uint4*>(base + (size_t)go * ld + gk);
    } else {
      const int k = q >> 5, c = q & 31;
      const int gk = k0 + k, go = outer0 + c * 8;
      if (gk < K && go < outer_n) v = *reinterpret_cast<const uint4*>(base + (size_t)gk * ld + go);
    }
    r[i] = v;
  }
}

template <bool KC>
__device__ __forceinline__ void store_tile(const uint4 (&r)[8], char* tile) {
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int q = i * NTHREADS + t;
    const int off = KC ? kc_off(q >> 3, q & 7) : ks_off(q >> 5, q & 31);
    *reinterpret_cast<uint4*>(tile + off) = r[i];
  }
}

// Fragment of 32 rows starting at row0 (multiple of 32), k-step ks (16 k): lane l gets row
// row0 + (l & 31), k = ks*16 + (l >> 5)*8 + 0..7.
template <bool KC>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int row0, int ks, int lane) {
  if (KC) {
    const int row = row0 + (lane & 31);
    const uint4 v = *reinterpret_cast<const uint4*>(tile + kc_off(row, ks * 2 + (lane >> 5)));
    return __builtin_bit_cast(bf16x8, v);
  } else {
    const int kb = ks * 16 + (lane >> 5) * 8 + ((lane & 15) >> 2);
    const int c = (row0 >> 3) + ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    const int sub = (lane & 1) * 8;
    union { short4v h[2]; bf16x8 v; } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(tile + ks_off(kb, c) + sub));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(tile + ks_off(kb + 4, c) + sub));
    return u.v;
  }
}

// Output tile index from the hardware workgroup id.  Workgroups are dealt round-robin to the
// 8 XCDs, each with its own L2; give every XCD a contiguous run of tiles, and order tiles in
// groups of 8 tile-rows so that the tiles resident on an XCD together share A and B panels.
__device__ __forceinline__ void tile_coords(int tiles_m, int tiles_n, int& tm, int& tn) {
  const int nt = tiles_m * tiles_n;
  const int b = blockIdx.x;
  const int q = nt >> 3, r = nt & 7, xcd = b & 7, i = b >> 3;
  const int pid = xcd < r ? xcd * (q + 1) + i : r * (q + 1) + (xcd - r) * q + i;
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int g = pid / per_group;
  const int first_m = g * GM;
  const int gsize = min(tiles_m - first_m, GM);
  const int in_g = pid - g * per_group;
  tm = first_m + in_g % gsize;
  tn = in_g / gsize;
}

template <bool A_KC, bool B_KC, typename TO, bool HAS_R>
__global__ __launch_bounds__(NTHREADS) void gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                             TO* __restrict__ C, const float* __restrict__ R, int M,
                                                             int N, int K, int lda, int ldb, int ldc, int ldr,
                                                             int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int tm, tn;
  tile_coords(tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;

  floatx16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 ra[8], rb[8];
  const int nk = (K + BK - 1) / BK;
  load_tile<A_KC>(ra, A, lda, m0, M, 0, K);
  load_tile<B_KC>(rb, B, ldb, n0, N, 0, K);
  store_tile<A_KC>(ra, smem);
  store_tile<B_KC>(rb, smem + TILE_BYTES);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const char* sa = smem + (kt & 1) * STAGE_BYTES;
    const char* sb = sa + TILE_BYTES;
    const bool more = kt + 1 < nk;
    if (more) {
      load_tile<A_KC>(ra, A, lda, m0, M, (kt + 1) * BK, K);
      load_tile<B_KC>(rb, B, ldb, n0, N, (kt + 1) * BK, K);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = read_frag<A_KC>(sa, wm + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < 4; ++j) fb[j] = read_frag<B_KC>(sb, wn + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (more) {
      char* na = smem + ((kt + 1) & 1) * STAGE_BYTES;
      store_tile<A_KC>(ra, na);
      store_tile<B_KC>(rb, na + TILE_BYTES);
    }
    __syncthreads();
  }

  // Epilogue.  acc[i][j][g*4 + e] = C[m0 + wm + i*32 + (lane & 31)][n0 + wn + j*32 + g*8 + (lane >> 5)*4 + e].
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + wm + i * 32 + (lane & 31);
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn + j * 32 + g * 8 + (lane >> 5) * 4;
        if (n >= N) continue;     // N is a multiple of 8: the four columns are in or out together
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][g * 4 + e];
        if (HAS_R) {
          const float4 rr = *reinterpret_cast<const float4*>(R + (size_t)m * ldr + n);
          v[0] += rr.x; v[1] += rr.y; v[2] += rr.z; v[3] += rr.w;
        }
        if (sizeof(TO) == 4) {
          *reinterpret_cast<float4*>((float*)C + (size_t)m * ldc + n) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
          uint2 o;
          o.x = pack_bf16x2(v[0], v[1]);
          o.y = pack_bf16x2(v[2], v[3]);
          *reinterpret_cast<uint2*>((bf16_t*)C + (size_t)m * ldc + n) = o;
        }
      }
    }
  }
}


// ------------------------------------------------------------------------------------------
// Direct-to-LDS variant (the one the stage tasks run).
//   - global -> LDS copies are buffer_load ... lds instructions, 16 bytes per lane, which land
//     in LDS at base + lane * 16 without passing through registers.  The XOR swizzles of the
//     tile layouts are therefore applied on the GLOBAL side: lane p of a 1 KB block fetches the
//     chunk that belongs at LDS position p.
//   - buffer descriptors bound every operand, so rows past the end of an operand read as zero
//     (that is what zero-fills the ragged K tail of the weight-gradient GEMMs, K = tokens).
//   - K advances in steps of 32 through FIVE LDS buffers of 32 KB (all of the CU's LDS); the loads of
//     steps e and e+1 are issued together, three to four steps ahead of their use.  The buffers are
//     five separate __shared__ arrays and the loop is unrolled by ten, so the compiler can prove that
//     fragment reads of one buffer do not alias loads in flight to another.
// Requires K % 32 == 0 when an operand is K-contiguous (a K tail would wrap into the next row).
// ------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// Wavefronts per workgroup of the direct-load kernel.  With a K-contiguous operand: 2 x 4 (128 x 64 of C
// each, two per SIMD so that one wavefront's waits hide behind the other's MFMAs), v_mfma_f32_16x16x32_bf16.
// With both operands K-strided (the weight-gradient form) the kernel is bounded by the issue rate of the
// LDS transpose reads, two per fragment: 2 x 2 wavefronts (128 x 128 each) need a third fewer of them.
// 256 accumulator registers per wavefront only allocate cleanly as 16 tuples of 16 (with 64 tuples of 4
// the register allocator shuffles accumulators between MFMAs), so that form keeps v_mfma_f32_32x32x16_bf16;
// it is not power bound, so the cheaper 16x16x32 form would buy nothing there.
constexpr int dl_wm(bool, bool) { return 2; }
constexpr int dl_wn(bool a_kc, bool b_kc) { return (a_kc || b_kc) ? 4 : 2; }
constexpr bool dl_m32(bool a_kc, bool b_kc) { return !a_kc && !b_kc; }
constexpr int DBK = 32;                              // k per stage
constexpr int DTILE = 256 * DBK * 2;                 // bytes of one operand tile (16 KB)
constexpr int DSTAGE = 2 * DTILE;                    // A + B (32 KB)

// K-contiguous tile [256 rows][32 k]: 64-byte rows, 4 chunks; chunk c of row r sits at c ^ s(r), with
// s = 0, 2, 3, 1 for (r >> 2) & 3 = 0, 1, 2, 3.  LDS serves 256 bytes per clock (64 banks), 16 lanes of a
// ds_read_b128 at a time, and those 16 lanes are not consecutive: measured (a probe that times the
// read for lane -> address tables, and the bank-conflict counter), the four passes take lanes
// {0-3, 12-15, 20-23, 24-27}, {32-35, 44-47, 52-55, 56-59}, {4-7, 8-11, 16-19, 28-31} and
// {36-39, 40-43, 48-51, 60-63}.  A fragment read has lane l at row (l & 15), chunk l >> 4, so one pass
// holds the row quads and chunks (0, c), (3, c), (1, c + 1), (2, c + 1); rows that differ in bits 0..1
// fall into different 64-byte windows of the 256, and s(r) sends the four quads of a pass to four
// different 16-byte slots.
__device__ __forceinline__ int dkc_swz(int row) {
  const int q = (row >> 2) & 3;
  return ((q & 1) << 1) ^ ((q >> 1) * 3);
}
__device__ __forceinline__ int dkc_off(int row, int c) { return row * 64 + ((c ^ dkc_swz(row)) << 4); }

// K-strided tile [32 k][256 rows]: 512-byte rows of 32 chunks; chunk c of row k sits at c ^ dks_swz(k).
// A fragment read (below) touches, per 32 lanes, 8 k-rows (k & 3 and bit 3 of k vary) at the same pair of
// chunks; the swizzle sends them to 8 distinct 32-byte bank groups.
__device__ __forceinline__ int dks_swz(int k) { return ((k & 3) | (((k >> 3) & 1) << 2)) << 1; }

// NW = wavefronts per workgroup.
// SWZ32 (K-strided tiles only): the swizzle of the 32x32x16 fragment reads (64-byte units moved by k,
// as in ks_off) instead of the one of the 16x16x32 reads.
template <bool KC, int NW, int ROWS = 256, bool SWZ32 = false>
struct DirectLoader {
  static_assert(KC || ROWS == 256, "a K-strided tile is always 256 wide");
  static constexpr int NL = (ROWS / 16) / NW;      // 1 KB blocks of the tile per wavefront (16 rows of 64 B each when K-contiguous)
  static_assert(NL >= 1, "tile too small for this many wavefronts");
  __amdgpu_buffer_rsrc_t rsrc;
  int voff[NL];
  int k_stride;     // bytes per k-step
  // pair_f > 0 (K-strided operand only): the 256 tile columns are 4 groups of [32 "gate" columns
  // f .. f+31 | 32 "up" columns pair_f + f .. pair_f + f+31], f = outer0/2 + 32 * group, so that one
  // wavefront holds gate and up of the same 32 features.
  __device__ __forceinline__ void init(const bf16_t* base, int ld, int outer0, int outer_n, int K, int wave, int lane,
                                       int pair_f = 0) {
    const size_t bytes = KC ? ((size_t)(outer_n - 1) * ld + K) * 2 : ((size_t)(K - 1) * ld + outer_n) * 2;
    rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
    k_stride = KC ? DBK * 2 : DBK * ld * 2;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int blk = i * NW + wave;                 // 1 KB block of the 16 KB tile
      if (KC) {
        const int row = blk * 16 + (lane >> 2), c = (lane & 3) ^ dkc_swz(row);
        voff[i] = (outer0 + row < outer_n) ? ((outer0 + row) * ld + c * 8) * 2 : (int)0x80000000;
      } else {
        const int k = blk * 2 + (lane >> 5), cp = lane & 31;
        const int f = (k & 3) | (((k >> 3) & 1) << 2);
        const int c = SWZ32 ? ((((cp >> 2) ^ f) << 2) | (cp & 3)) : (cp ^ dks_swz(k));
        int col = outer0 + c * 8;
        if (pair_f > 0) {
          const int nl = c * 8;                                  // column inside the tile
          col = ((nl >> 5) & 1) * pair_f + (outer0 >> 1) + (nl >> 6) * 32 + (nl & 31);
        }
        voff[i] = (k * ld + col) * 2;
      }
    }
  }
  // Load instruction i (of NL) of this wavefront for the k-step whose byte offset is soff.
  // exists == false: every lane gets the per-lane offset that is past any buffer (the same marker rows
  // past the end of the operand carry), so the descriptor's range check turns the load into zeros.
  __device__ __forceinline__ void issue_one(char* tile, int i, int soff, int wave, bool exists) const {
    const int vo = exists ? voff[i] : (int)0x80000000;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(tile + (i * NW + wave) * 1024), 16, vo, soff, 0, 0);
  }
};

// One quarter (Q = 0..3) of the loads of a pair of consecutive k-steps (e, e+1), e even: step e goes to
// bufE, step e+1 to bufO.  A wavefront's LA + LB load instructions per step are dealt to the quarters in
// order (A first); the two instructions that fetch the same rows for the two steps are issued back to
// back.  For a K-contiguous operand they are the two 64-byte halves of the same 128-byte lines: issued
// together they reach L2 as one request per line, issued a step apart (as two separate fetches) as two.
// Steps at or beyond nk are issued with a per-lane offset past every buffer (2^31; operands are smaller),
// which the descriptor turns into a load of zeros without a memory access: the number of loads in flight
// never depends on the position in K.
template <int Q, int LA, int LB>
struct QuarterCount { static constexpr int PAIRS = (Q + 1) * (LA + LB) / 4 - Q * (LA + LB) / 4, LOADS = 2 * PAIRS; };
template <int Q, bool GUARD, typename LoaderA, typename LoaderB>
__device__ __forceinline__ void issue_quarter(const LoaderA& la, const LoaderB& lb, char* bufE, char* bufO, int e, int nk, int wave) {
  constexpr int LA = LoaderA::NL, LB = LoaderB::NL;
  constexpr int P0 = Q * (LA + LB) / 4, P1 = (Q + 1) * (LA + LB) / 4;
  if constexpr (P1 > P0) {
    const bool okE = !GUARD || e < nk, okO = !GUARD || e + 1 < nk;
    const int aE = okE ? e * la.k_stride : 0, aO = okO ? (e + 1) * la.k_stride : 0;
    const int bE = okE ? e * lb.k_stride : 0, bO = okO ? (e + 1) * lb.k_stride : 0;
#pragma unroll
    for (int p = P0; p < P1; ++p) {
      if (p < LA) {
        la.issue_one(bufE, p, aE, wave, okE);
        la.issue_one(bufO, p, aO, wave, okO);
      } else {
        lb.issue_one(bufE + DTILE, p - LA, bE, wave, okE);
        lb.issue_one(bufO + DTILE, p - LA, bO, wave, okO);
      }
    }
  }
}

// Fragments of v_mfma_f32_16x16x32_bf16 for a 16-row block and the 32 k of one stage: lane l gets row
// (l & 15) of the block, k = (l >> 4) * 8 + 0..7.
//   K-contiguous: one ds_read_b128 at dkc_off(row, l >> 4); blocks are 1024 bytes apart.
//   K-strided: two ds_read_b64_tr_b16 (k-rows kb and kb + 4, same swizzle); in each, the 16 lanes of a
//     group address a 4 (k) x 16 (rows) block (lane -> k-row (l & 15) >> 2, rows 4 * (l & 3) .. + 3) and
//     receive 4 consecutive k of row l & 15.  Block i of the wavefront sits at chunk (cw | 2i | cl),
//     cw = 16-aligned chunk of the wavefront's first row, cl = (l & 3) >> 1, and the swizzle XORs bits
//     1..3 of the chunk, so the byte offset of block i is lane_part ^ (i << 5): one XOR per block.
typedef __attribute__((address_space(3))) const char* lds_char_ptr;

// Per-lane part of the fragment address of this wavefront's blocks starting at row w0.
template <bool KC>
__device__ __forceinline__ int frag_lane_offset(int w0, int lane) {
  if (KC) return dkc_off(w0 + (lane & 15), lane >> 4);
  const int kb = (lane >> 4) * 8 + ((lane & 15) >> 2);
  return kb * 512 + (lane & 1) * 8 + ((((w0 >> 3) | ((lane & 3) >> 1)) ^ dks_swz(kb)) << 4);
}

template <bool KC, int N>
__device__ __forceinline__ void load_blocks(bf16x8 (&f)[N], const char* tile, int lane_off) {
  if (!KC) asm volatile("" : "+v"(lane_off));   // keeps the per-block addresses from being hoisted out of the k loop (register pressure)
  const lds_char_ptr t = (lds_char_ptr)tile;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (KC) {
      f[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) uint4*>(t + lane_off + i * 1024));
    } else {
      const int o = lane_off ^ (i << 5);
      union { short4v h[2]; bf16x8 v; } u;
      u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(t + o));
      u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(t + o + 2048));
      f[i] = u.v;
    }
  }
}

// Workgroup barrier between pipeline steps.  The caller has already waited (s_waitcnt vmcnt) for its
// own direct loads of the stage that is read next; a plain s_barrier then makes every wavefront's
// share of that stage visible.  No fence: a release fence would make the compiler drain ALL loads
// in flight, including those of the stages two and three steps ahead.  The empty asm statements
// keep the compiler from moving LDS accesses across the barrier.
__device__ __forceinline__ void stage_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("" ::: "memory");
}

// Fragments of one 32-deep step for v_mfma_f32_16x16x32_bf16: the wavefront's 16-row blocks of A in two
// halves (lo, hi: MA blocks each) and its NF 16-column blocks of B, the latter double-buffered by step parity.
template <int MA, int NF>
struct Frags { bf16x8 alo[MA], ahi[MA], b[2][NF]; };

// acc[i0 + i][j] += A block i x B block j.  The B fragment is the first operand: a lane's four accumulator
// values are four consecutive columns of one row of C.
// F16: the 16-bit operands are IEEE halves (v_mfma_f32_16x16x32_f16; same rate, same fragment layout).
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
template <int MA, int NF, int MI16, bool F16 = false>
__device__ __forceinline__ void mfma_blocks(floatx4 (&acc)[MI16][NF], const bf16x8 (&a)[MA], const bf16x8 (&b)[NF], int i0) {
#pragma unroll
  for (int i = 0; i < MA; ++i)
#pragma unroll
    for (int j = 0; j < NF; ++j) {
      if constexpr (F16)
        acc[i0 + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, b[j]), __builtin_bit_cast(halfx8, a[i]),
                                                                acc[i0 + i][j], 0, 0, 0);
      else
        acc[i0 + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i0 + i][j], 0, 0, 0);
    }
}

// 32x32x16 path (both operands K-strided): fragments of one 16-wide k-step, MI row blocks of A and NB column
// blocks of B (32 x 16 each, two transpose reads per fragment).
template <int MI, int NB>
struct Frags32 { bf16x8 a[MI], b[NB]; };
template <int MI, int NB>
__device__ __forceinline__ void load_frags32(Frags32<MI, NB>& f, const char* sa, int ks, int wm, int wn, int lane) {
  const char* sb = sa + DTILE;
#pragma unroll
  for (int i = 0; i < MI; ++i) f.a[i] = read_frag<false>(sa, wm + i * 32, ks, lane);
#pragma unroll
  for (int j = 0; j < NB; ++j) f.b[j] = read_frag<false>(sb, wn + j * 32, ks, lane);
}
template <int MI, int NB>
__device__ __forceinline__ void mfma32(floatx16 (&acc)[MI][NB], const Frags32<MI, NB>& f) {
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j], f.a[i], acc[i][j], 0, 0, 0);
}

// Ask the scheduler to interleave N_DS LDS reads, N_VM global->LDS loads and N_MFMA MFMAs in groups, reads
// leading.  The loads are spread over the groups on purpose: a wavefront that issues its loads of a step
// back to back sits at the (in-order) issue of the later ones while the texture path works through the
// earlier ones, and its MFMAs wait behind them; one load between every few MFMAs never queues.
template <int N_DS, int N_MFMA, int N_VM, int G, int Q>
__device__ __forceinline__ void interleave_group() {
  if constexpr (Q < G) {
    // LDS reads go into the first G-1 groups (the last MFMAs of the half-step cover the latency of the last reads)
    constexpr int DSG = G - 1;
    constexpr int DS = Q < DSG ? ((Q + 1) * N_DS + DSG - 1) / DSG - (Q * N_DS + DSG - 1) / DSG : 0;
    constexpr int VM = (Q + 1) * N_VM / G - Q * N_VM / G;
    constexpr int MF = (Q + 1) * N_MFMA / G - Q * N_MFMA / G;
    if constexpr (DS > 0) __builtin_amdgcn_sched_group_barrier(0x100, DS, 0);
    if constexpr (VM > 0) __builtin_amdgcn_sched_group_barrier(0x020, VM, 0);
    if constexpr (MF > 0) __builtin_amdgcn_sched_group_barrier(0x008, MF, 0);
    interleave_group<N_DS, N_MFMA, N_VM, G, Q + 1>();
  }
}
template <int N_DS, int N_MFMA, int N_VM>
__device__ __forceinline__ void interleave_ds_vm_mfma() {
  interleave_group<N_DS, N_MFMA, N_VM, (N_MFMA % 4 == 0) ? 4 : 2, 0>();
}

// WM x WN wavefronts tile the 256x256 block; each owns (256/WM) x (256/WN).
__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + __expf(-z)); }
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.0f + erff(u * 0.70710678118654752f)) + u * 0.39894228040143268f * __expf(-0.5f * u * u);
}
__device__ __forceinline__ void load_f32x8(const float* p, float* v) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void unpack4(uint2 w, float* v) {
  v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
  v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
}

// BMT = rows of the C tile: 256, or 128 for the short tiles that finish a GEMM whose tile count is
// not a multiple of the CU count (A K-contiguous only).  tn0 = first tile column of this launch.
// F16IN: A and B hold IEEE halves instead of bf16 (forms with a K-contiguous operand only); TO may be float,
// bf16_t or f16_t.
template <bool A_KC, bool B_KC, typename TO, bool HAS_R, int WM, int WN, int ACT, int BMT = 256, bool F16IN = false>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_dl_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                               TO* __restrict__ C, const float* __restrict__ R, int M,
                                                               int N, int K, int lda, int ldb, int ldc, int ldr,
                                                               int tiles_m, int tiles_n, bf16_t* __restrict__ E, int lde,
                                                               int tn0, int k_split, const bf16_t* __restrict__ bias,
                                                               const float* __restrict__ out_scale) {
  constexpr int NW = WM * WN;
  // Split-K launches (grid y = split): this workgroup contracts k in [y * k_split, min(K, (y+1) * k_split))
  // and writes its partial tile into the y-th [M, ldc] plane of C.
  if (k_split > 0) {
    const int k0 = blockIdx.y * k_split;
    A += A_KC ? (size_t)k0 : (size_t)k0 * lda;
    B += B_KC ? (size_t)k0 : (size_t)k0 * ldb;
    C += (size_t)blockIdx.y * M * ldc;
    K = min(k_split, K - k0);
  }
  constexpr int MI = (BMT / 32) / WM;               // 32-high row blocks per wavefront
  constexpr int NB = 8 / WN;                        // 32-wide column blocks per wavefront
  constexpr int WAVE_M = MI * 32, WAVE_N = NB * 32;
  __shared__ __attribute__((aligned(1024))) char stage0[DSTAGE];
  __shared__ __attribute__((aligned(1024))) char stage1[DSTAGE];
  __shared__ __attribute__((aligned(1024))) char stage2[DSTAGE];
  __shared__ __attribute__((aligned(1024))) char stage3[DSTAGE];
  __shared__ __attribute__((aligned(1024))) char stage4[DSTAGE];
  int tm, tn;
  tile_coords(tiles_m, tiles_n, tm, tn);
  const int m0 = tm * BMT, n0 = (tn + tn0) * BN;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave / WN) * WAVE_M, wn = (wave % WN) * WAVE_N;

  constexpr bool M32 = dl_m32(A_KC, B_KC);          // 32x32x16 accumulators (acc32) instead of 16x16x32 ones (acc)
  static_assert(!(M32 && F16IN), "half inputs are built for the 16x16x32 forms only");
  constexpr int MI16 = 2 * MI, NF = 2 * NB, MA = MI;   // 16-row / 16-column blocks per wavefront; A blocks per half
  floatx4 acc[M32 ? 1 : MI16][M32 ? 1 : NF];
  floatx16 acc32[M32 ? MI : 1][M32 ? NB : 1];
  if constexpr (M32) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc32[i][j][e] = 0.f;
  } else {
#pragma unroll
    for (int i = 0; i < MI16; ++i)
#pragma unroll
      for (int j = 0; j < NF; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  }

  DirectLoader<A_KC, NW, BMT, M32> la;
  DirectLoader<B_KC, NW, 256, M32> lb;
  la.init(A, lda, m0, M, K, wave, lane);
  lb.init(B, ldb, n0, N, K, wave, lane, ACT == ACT_SWIGLU_FWD ? N / 2 : 0);
  const int nk = (K + DBK - 1) / DBK;

  // Software pipeline over 32-deep steps through a ring of five LDS buffers (step t lives in buffer
  // t % 5).  Loads are issued for PAIRS of steps (e, e+1), e even, in four quarters spread over four
  // consecutive half-steps, starting right after the barrier in the middle of step e-4 (which frees the
  // buffer of step e-4 for step e+1; the buffer of step e-5 is free since the barrier before):
  //   quarter 0 in the second half of step e-4, 1 and 2 in the two halves of step e-3, 3 in the first
  //   half of step e-2.
  // Entering step t the fragments of the first half of the wavefront's A blocks and of all its B blocks
  // are in registers.  First half: read the second half of the A blocks under the MFMAs of the first
  // (after this, nobody reads buffer t % 5 any more).  Middle: wait for the own LDS reads and,
  // on odd steps, for this wavefront's loads of the pair (t+1, t+2): everything but quarters 0 and 1 of
  // the following pair, which were issued later; then barrier: buffer t % 5 is consumed by everybody and
  // the pair (t+1, t+2) is complete.  On even steps the next step's buffer is complete since the previous
  // barrier.  Second half: read step t+1's first A half and its B blocks (into the other B register
  // set) under the MFMAs of the second A half.
  using LoaderA = DirectLoader<A_KC, NW, BMT, M32>;
  using LoaderB = DirectLoader<B_KC, NW, 256, M32>;
  constexpr int LA = LoaderA::NL, LB = LoaderB::NL;
  constexpr int NQ0 = QuarterCount<0, LA, LB>::LOADS, NQ1 = QuarterCount<1, LA, LB>::LOADS;
  constexpr int NQ2 = QuarterCount<2, LA, LB>::LOADS, NQ3 = QuarterCount<3, LA, LB>::LOADS;
  constexpr int LGKM_ONLY = 0xC07F;                                // vmcnt(63), lgkmcnt(0)
  constexpr int VM_01 = 0x0070 | ((NQ0 + NQ1) & 15) | (((NQ0 + NQ1) >> 4) << 14);              // vmcnt(NQ0+NQ1), lgkmcnt(0)
  constexpr int VM_012 = 0x0070 | ((NQ0 + NQ1 + NQ2) & 15) | (((NQ0 + NQ1 + NQ2) >> 4) << 14);  // vmcnt(NQ0+NQ1+NQ2), lgkmcnt(0)
  constexpr int DS_A = A_KC ? MA : 2 * MA, DS_B = B_KC ? NF : 2 * NF;   // LDS read instructions of half the A blocks / all B blocks
  constexpr int N_MFMA = MA * NF;                                        // MFMAs of a half-step
  // One step.  PAR = parity of tt; b0..b4 = the buffers of steps tt..tt+4; GUARD = the step may be the
  // last one or beyond (the tail loop), else every step up to tt+5 exists.
#define RRFP_STEP(PAR, GUARD, b0, b1, b2, b3, b4, tt)                                                    \
  if (!GUARD || (tt) < nk) {                                                                             \
    if constexpr (PAR == 0) issue_quarter<3, GUARD>(la, lb, b2, b3, (tt) + 2, nk, wave);                 \
    else issue_quarter<1, GUARD>(la, lb, b3, b4, (tt) + 3, nk, wave);                                    \
    if constexpr (M32) {                                                                                 \
      load_frags32<MI, NB>(fy, b0, 1, wm, wn, lane);                                                     \
      mfma32<MI, NB>(acc32, fx);                                                                         \
      interleave_ds_vm_mfma<2 * (MI + NB), MI * NB, (PAR == 0 ? NQ3 : NQ1)>();                           \
    } else {                                                                                             \
      load_blocks<A_KC, MA>(fr.ahi, b0, off_ahi);                                                        \
      mfma_blocks<MA, NF, MI16, F16IN>(acc, fr.alo, fr.b[PAR], 0);                                       \
      interleave_ds_vm_mfma<DS_A, N_MFMA, (PAR == 0 ? NQ3 : NQ1)>();                                     \
    }                                                                                                    \
    if (!GUARD || (tt) + 1 < nk) {                                                                       \
      __builtin_amdgcn_s_waitcnt(PAR == 0 ? LGKM_ONLY : VM_01);                                          \
      stage_barrier();                                                                                   \
      if constexpr (PAR == 0) issue_quarter<0, GUARD>(la, lb, b4, b0, (tt) + 4, nk, wave);               \
      else issue_quarter<2, GUARD>(la, lb, b3, b4, (tt) + 3, nk, wave);                                  \
      if constexpr (M32) {                                                                               \
        load_frags32<MI, NB>(fx, b1, 0, wm, wn, lane);                                                   \
      } else {                                                                                           \
        load_blocks<A_KC, MA>(fr.alo, b1, off_alo);                                                      \
        load_blocks<B_KC, NF>(fr.b[1 - PAR], b1 + DTILE, off_b);                                         \
      }                                                                                                  \
    }                                                                                                    \
    if constexpr (M32) mfma32<MI, NB>(acc32, fy);                                                        \
    else mfma_blocks<MA, NF, MI16, F16IN>(acc, fr.ahi, fr.b[PAR], MA);                                   \
    if (!GUARD) {                                                                                        \
      if constexpr (M32) interleave_ds_vm_mfma<2 * (MI + NB), MI * NB, (PAR == 0 ? NQ0 : NQ2)>();        \
      else interleave_ds_vm_mfma<DS_A + DS_B, N_MFMA, (PAR == 0 ? NQ0 : NQ2)>();                         \
      __builtin_amdgcn_sched_barrier(0);   /* half-steps are scheduled one by one */                     \
    }                                                                                                    \
  }
#define RRFP_TEN_STEPS(GUARD, t)                                        \
  RRFP_STEP(0, GUARD, stage0, stage1, stage2, stage3, stage4, (t));     \
  RRFP_STEP(1, GUARD, stage1, stage2, stage3, stage4, stage0, (t) + 1); \
  RRFP_STEP(0, GUARD, stage2, stage3, stage4, stage0, stage1, (t) + 2); \
  RRFP_STEP(1, GUARD, stage3, stage4, stage0, stage1, stage2, (t) + 3); \
  RRFP_STEP(0, GUARD, stage4, stage0, stage1, stage2, stage3, (t) + 4); \
  RRFP_STEP(1, GUARD, stage0, stage1, stage2, stage3, stage4, (t) + 5); \
  RRFP_STEP(0, GUARD, stage1, stage2, stage3, stage4, stage0, (t) + 6); \
  RRFP_STEP(1, GUARD, stage2, stage3, stage4, stage0, stage1, (t) + 7); \
  RRFP_STEP(0, GUARD, stage3, stage4, stage0, stage1, stage2, (t) + 8); \
  RRFP_STEP(1, GUARD, stage4, stage0, stage1, stage2, stage3, (t) + 9)

  Frags<MA, NF> fr;
  Frags32<MI, NB> fx, fy;
  const int off_alo = frag_lane_offset<A_KC>(wm, lane), off_ahi = frag_lane_offset<A_KC>(wm + MA * 16, lane);
  const int off_b = frag_lane_offset<B_KC>(wn, lane);
  // Prologue: the pair (0, 1) in full and quarters 0..2 of the pair (2, 3); step 0's first half issues quarter 3.
  issue_quarter<0, true>(la, lb, stage0, stage1, 0, nk, wave);
  issue_quarter<1, true>(la, lb, stage0, stage1, 0, nk, wave);
  issue_quarter<2, true>(la, lb, stage0, stage1, 0, nk, wave);
  issue_quarter<3, true>(la, lb, stage0, stage1, 0, nk, wave);
  issue_quarter<0, true>(la, lb, stage2, stage3, 2, nk, wave);
  issue_quarter<1, true>(la, lb, stage2, stage3, 2, nk, wave);
  issue_quarter<2, true>(la, lb, stage2, stage3, 2, nk, wave);
  __builtin_amdgcn_s_waitcnt(VM_012);
  stage_barrier();
  if constexpr (M32) {
    load_frags32<MI, NB>(fx, stage0, 0, wm, wn, lane);
  } else {
    load_blocks<A_KC, MA>(fr.alo, stage0, off_alo);
    load_blocks<B_KC, NF>(fr.b[0], stage0 + DTILE, off_b);
  }

  int t = 0;
  for (; t + 13 < nk; t += 10) {    // every load these ten steps issue is for a step below nk
    RRFP_TEN_STEPS(false, t);
  }
  for (; t < nk; t += 10) {
    RRFP_TEN_STEPS(true, t);
  }
#undef RRFP_TEN_STEPS
#undef RRFP_STEP
  __builtin_amdgcn_s_waitcnt(0x0070);   // the zero loads of the steps past the end have landed too

  // Epilogue through LDS.  In the accumulator layout a lane owns 4 consecutive columns of one row, so a
  // direct store instruction would touch 32 different rows with 16 bytes each.  Instead every wavefront
  // writes one 32-row block of its accumulators to its own LDS scratch (the pipeline stages are free
  // now), and reads it back with 8 consecutive columns per lane and whole rows per group of lanes: all
  // global loads and stores of the epilogue (C, the residual, the activation operand) are then row-
  // contiguous 16- or 32-byte accesses per lane.
  __syncthreads();     // every wavefront has finished its fragment reads of the last step
  float* scratch;
  {
    constexpr int PER = DSTAGE * 4 / NW;            // bytes of scratch per wavefront: 16 KB (8 waves) or 32 KB (4)
    const int sel = wave * PER / DSTAGE, sub = (wave * PER) % DSTAGE;
    char* base = sel == 0 ? stage0 : sel == 1 ? stage1 : sel == 2 ? stage2 : stage3;
    scratch = reinterpret_cast<float*>(base + sub);
  }
  constexpr int NBC = NB * 32;                      // columns of the wavefront's tile
  constexpr int PITCH = NBC + 4;                    // floats; 16-byte skew per row
  const int li = lane & 15, hq = lane >> 4;
  // The epilogue's global operand loads (residual, activation operand) are issued for a whole 32-row
  // chunk before the chunk is staged, from addresses clamped into the matrix, so that their latency is
  // paid once per chunk and not once per sweep; only the stores are predicated.
  constexpr int LPR = NBC / 8;                      // lanes per row of the read-back
  constexpr int RPS = 64 / LPR;                     // rows per sweep
  constexpr int SW = 32 / RPS;                      // sweeps per chunk
  const int c0 = (lane % LPR) * 8, r0 = lane / LPR;
  const int n_col = n0 + wn + c0;                   // first of this lane's 8 columns (same for every sweep)
  const int n_ld = min(n_col, N - 8);
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (ACT != ACT_SWIGLU_FWD && bias) load_vec<bf16_t>(bias + n_ld, bv);
  // out_scale (plain 16-bit outputs only): a device scalar, a power of two, multiplied into the result before it
  // is rounded -- brings a gradient tensor into the range of IEEE halves whatever the scale of the loss
  const float oscale = (ACT == ACT_NONE && !HAS_R && sizeof(TO) == 2 && out_scale) ? *out_scale : 1.0f;
  struct Pre { float rv[8]; uint4 e0, e1; };
  auto prefetch = [&](Pre (&pre)[SW], int i) {
#pragma unroll
    for (int rr = 0; rr < SW; ++rr) {
      const int m_ld = min(m0 + wm + i * 32 + rr * RPS + r0, M - 1);
      if (HAS_R) load_f32x8(R + (size_t)m_ld * ldr + n_ld, pre[rr].rv);
      if (ACT == ACT_GELU_BWD || ACT == ACT_SWIGLU_BWD) pre[rr].e0 = *reinterpret_cast<const uint4*>(E + (size_t)m_ld * lde + n_ld);
      if (ACT == ACT_SWIGLU_BWD) pre[rr].e1 = *reinterpret_cast<const uint4*>(E + (size_t)m_ld * lde + N + n_ld);
    }
  };
  Pre pre[2][SW];
  if (ACT != ACT_SWIGLU_FWD) prefetch(pre[0], 0);
  // The lanes of a wavefront exchange values through the wavefront's own scratch: write in the accumulator
  // layout, read back row-contiguous, overwrite with the next chunk.  The hardware executes one wavefront's
  // LDS instructions in order; these wavefront-scope fences keep the compiler from reordering the three phases.
  auto wave_sync = [] {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    wave_sync();        // read-back of chunk i-1 precedes the writes of chunk i
    if constexpr (M32) {
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(scratch + (lane & 31) * PITCH + j * 32 + g * 8 + (lane >> 5) * 4) =
              make_float4(acc32[i][j][g * 4 + 0], acc32[i][j][g * 4 + 1], acc32[i][j][g * 4 + 2], acc32[i][j][g * 4 + 3]);
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < NF; ++j)
          *reinterpret_cast<float4*>(scratch + (h * 16 + li) * PITCH + j * 16 + hq * 4) =
              make_float4(acc[2 * i + h][j][0], acc[2 * i + h][j][1], acc[2 * i + h][j][2], acc[2 * i + h][j][3]);
    }
    wave_sync();        // the writes of chunk i precede its read-back
    if (ACT == ACT_SWIGLU_FWD) {
      // scratch columns 0..31 = gate, 32..63 = up of features f0 .. f0+31; 4 lanes per row, 16 rows per sweep
      const int F = N >> 1;
      const int f0 = (n0 >> 1) + (wn >> 6) * 32;
      const int fc = (lane & 3) * 8;
      float bg[8], bu[8];
      if (bias) {
        load_vec<bf16_t>(bias + f0 + fc, bg);
        load_vec<bf16_t>(bias + F + f0 + fc, bu);
      }
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        const int row = rr * 16 + (lane >> 2);
        const int m = m0 + wm + i * 32 + row;
        float gt[8], up[8], mm[8];
        load_f32x8(scratch + row * PITCH + fc, gt);
        load_f32x8(scratch + row * PITCH + 32 + fc, up);
        if (bias) {
#pragma unroll
          for (int e = 0; e < 8; ++e) { gt[e] += bg[e]; up[e] += bu[e]; }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) mm[e] = gt[e] * sigmoid_f(gt[e]) * up[e];
        if (m < M) {
          bf16_t* crow = (bf16_t*)C + (size_t)m * ldc + f0 + fc;
          store_vec<bf16_t>(crow, gt);
          store_vec<bf16_t>(crow + F, up);
          store_vec<bf16_t>(E + (size_t)m * lde + f0 + fc, mm);
        }
      }
    } else if (sizeof(TO) == 4 && ACT == ACT_NONE && !HAS_R && !bias) {
      // plain fp32 tile: 16 bytes per lane with the lanes of a row side by side, so that every store instruction
      // writes whole 128-byte lines (with 32 bytes per lane each of the two stores would write half of every line)
      constexpr int LPR4 = NBC / 4, RPS4 = 64 / LPR4, SW4 = 32 / RPS4;
      const int c4 = (lane % LPR4) * 4, r4 = lane / LPR4;
      const int n = n0 + wn + c4;
#pragma unroll
      for (int rr = 0; rr < SW4; ++rr) {
        const int row = rr * RPS4 + r4;
        const int m = m0 + wm + i * 32 + row;
        const float4 v = *reinterpret_cast<const float4*>(scratch + row * PITCH + c4);
        if (m < M && n < N) *reinterpret_cast<float4*>((float*)C + (size_t)m * ldc + n) = v;   // N is a multiple of 8
      }
    } else {
      if (i + 1 < MI) prefetch(pre[(i + 1) & 1], i + 1);
      const Pre (&cur)[SW] = pre[i & 1];
#pragma unroll
      for (int rr = 0; rr < SW; ++rr) {
        const int row = rr * RPS + r0;
        const int m = m0 + wm + i * 32 + row, n = n_col;
        float v[8];
        load_f32x8(scratch + row * PITCH + c0, v);
        const bool ok = m < M && n < N;             // N is a multiple of 8: the eight columns are in or out together
        if (bias) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += bv[e];
        }
        if (HAS_R) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += cur[rr].rv[e];
        }
        if (ACT == ACT_GELU_FWD) {
          float mm[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) mm[e] = gelu_f(v[e]);
          if (ok) {
            store_vec<bf16_t>((bf16_t*)C + (size_t)m * ldc + n, v);
            store_vec<bf16_t>(E + (size_t)m * lde + n, mm);
          }
        } else if (ACT == ACT_GELU_BWD) {
          float u[8];
          unpack4(make_uint2(cur[rr].e0.x, cur[rr].e0.y), u);
          unpack4(make_uint2(cur[rr].e0.z, cur[rr].e0.w), u + 4);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= gelu_grad_f(u[e]);
          if (ok) store_vec<bf16_t>((bf16_t*)C + (size_t)m * ldc + n, v);
        } else if (ACT == ACT_SWIGLU_BWD) {
          float gt[8], up[8], dg[8], du[8];
          unpack4(make_uint2(cur[rr].e0.x, cur[rr].e0.y), gt);
          unpack4(make_uint2(cur[rr].e0.z, cur[rr].e0.w), gt + 4);
          unpack4(make_uint2(cur[rr].e1.x, cur[rr].e1.y), up);
          unpack4(make_uint2(cur[rr].e1.z, cur[rr].e1.w), up + 4);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float sg = sigmoid_f(gt[e]);
            dg[e] = v[e] * up[e] * sg * (1.0f + gt[e] * (1.0f - sg));
            du[e] = v[e] * gt[e] * sg;
          }
          if (ok) {
            store_vec<bf16_t>((bf16_t*)C + (size_t)m * ldc + n, dg);
            store_vec<bf16_t>((bf16_t*)C + (size_t)m * ldc + N + n, du);
          }
        } else if (sizeof(TO) == 4) {
          if (ok) {
            float* crow = (float*)C + (size_t)m * ldc + n;
            *reinterpret_cast<float4*>(crow) = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4*>(crow + 4) = make_float4(v[4], v[5], v[6], v[7]);
          }
        } else {
          using T16 = std::conditional_t<sizeof(TO) == 2, TO, bf16_t>;    // bf16_t or f16_t
          if constexpr (ACT == ACT_NONE && !HAS_R) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] *= oscale;
          }
          if (ok) store_vec<T16>((T16*)C + (size_t)m * ldc + n, v);
        }
      }
    }
  }
}

// Explicit instantiations of every variant the launcher can pick.
#define RRFP_INST(AKC, BKC, TO, HR, ACT)                                                                     \
  template __global__ void gemm_mfma_dl_kernel<AKC, BKC, TO, HR, dl_wm(AKC, BKC), dl_wn(AKC, BKC), ACT>(      \
      const bf16_t*, const bf16_t*, TO*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);
#define RRFP_INST_SHORT(BKC, TO, HR, ACT)                                                                    \
  template __global__ void gemm_mfma_dl_kernel<true, BKC, TO, HR, dl_wm(true, BKC), dl_wn(true, BKC), ACT, 128>( \
      const bf16_t*, const bf16_t*, TO*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);
#define RRFP_INST_SHORT4(BKC) RRFP_INST_SHORT(BKC, float, true, ACT_NONE) RRFP_INST_SHORT(BKC, float, false, ACT_NONE) \
                              RRFP_INST_SHORT(BKC, bf16_t, true, ACT_NONE) RRFP_INST_SHORT(BKC, bf16_t, false, ACT_NONE)
RRFP_INST_SHORT4(false) RRFP_INST_SHORT4(true)
RRFP_INST_SHORT(false, bf16_t, false, ACT_SWIGLU_FWD) RRFP_INST_SHORT(false, bf16_t, false, ACT_GELU_FWD)
RRFP_INST_SHORT(true, bf16_t, false, ACT_SWIGLU_BWD) RRFP_INST_SHORT(true, bf16_t, false, ACT_GELU_BWD)
#undef RRFP_INST_SHORT4
#undef RRFP_INST_SHORT
#define RRFP_INST4(AKC, BKC) RRFP_INST(AKC, BKC, float, true, ACT_NONE) RRFP_INST(AKC, BKC, float, false, ACT_NONE) \
                             RRFP_INST(AKC, BKC, bf16_t, true, ACT_NONE) RRFP_INST(AKC, BKC, bf16_t, false, ACT_NONE)
RRFP_INST4(true, false) RRFP_INST4(true, true) RRFP_INST4(false, false) RRFP_INST4(false, true)
RRFP_INST(true, false, bf16_t, false, ACT_SWIGLU_FWD) RRFP_INST(true, false, bf16_t, false, ACT_GELU_FWD)
RRFP_INST(true, true, bf16_t, false, ACT_SWIGLU_BWD) RRFP_INST(true, true, bf16_t, false, ACT_GELU_BWD)
#undef RRFP_INST4
#undef RRFP_INST
// Half-precision forms of the attention path: the QKV projection (half in, half out), the output projection
// (half in, fp32 out with the residual) and the gradient of the attention output, dO = dx1 Wo^T (bf16 in, half
// out), each with its 128-row tile variant.
template __global__ void gemm_mfma_dl_kernel<true, false, f16_t, false, dl_wm(true, false), dl_wn(true, false), ACT_NONE, 256, true>(
    const bf16_t*, const bf16_t*, f16_t*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);
template __global__ void gemm_mfma_dl_kernel<true, false, f16_t, false, dl_wm(true, false), dl_wn(true, false), ACT_NONE, 128, true>(
    const bf16_t*, const bf16_t*, f16_t*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);
template __global__ void gemm_mfma_dl_kernel<true, false, float, true, dl_wm(true, false), dl_wn(true, false), ACT_NONE, 256, true>(
    const bf16_t*, const bf16_t*, float*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);
template __global__ void gemm_mfma_dl_kernel<true, false, float, true, dl_wm(true, false), dl_wn(true, false), ACT_NONE, 128, true>(
    const bf16_t*, const bf16_t*, float*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);
template __global__ void gemm_mfma_dl_kernel<true, true, f16_t, false, dl_wm(true, true), dl_wn(true, true), ACT_NONE, 256, false>(
    const bf16_t*, const bf16_t*, f16_t*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);
template __global__ void gemm_mfma_dl_kernel<true, true, f16_t, false, dl_wm(true, true), dl_wn(true, true), ACT_NONE, 128, false>(
    const bf16_t*, const bf16_t*, f16_t*, const float*, int, int, int, int, int, int, int, int, int, bf16_t*, int, int, int, const bf16_t*, const float*);

// True when the direct-to-LDS kernel can take the call (else the register-staged one does).
inline bool direct_ok(const GemmArgs& g) {
  const bool a_kc = !g.transA, b_kc = g.transB;
  if ((a_kc || b_kc) && (g.K % DBK)) return false;
  const size_t lim = (size_t)1 << 31;      // every operand byte offset stays below the per-lane offset that means "out of range"
  const size_t a_bytes = (size_t)(a_kc ? g.M + BM : g.K + BK) * g.lda * 2;
  const size_t b_bytes = (size_t)(b_kc ? g.N + BN : g.K + BK) * g.ldb * 2;
  return a_bytes < lim && b_bytes < lim;
}

// Compute units of the current device (cached per device id; 256 if the query fails).
inline int cu_count() {
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

// How a GEMM with A K-contiguous is cut into launches.  One workgroup occupies a CU, so t tiles of
// 256 x 256 run in ceil(t / n_cu) rounds.  (a) A grid that fills at most half the CUs is launched
// entirely with 128-row tiles (twice the workgroups).  (b) Otherwise, when the last round holds r
// tiles and carving ceil(r / tiles_m) trailing tile columns off removes that round, those columns
// are launched separately with 128-row tiles, provided they fit one round.  A pure function of the
// shape and the device.  Returns the number of tile columns of the 256-row launch.
inline int full_tile_columns(int tiles_m, int tiles_n, int n_cu) {
  const int t = tiles_m * tiles_n;
  if (2 * t <= n_cu) return 0;
  const int r = t % n_cu;
  if (t <= n_cu || r == 0) return tiles_n;
  const int ct = (r + tiles_m - 1) / tiles_m;
  if (ct >= tiles_n) return tiles_n;
  const int t_main = t - ct * tiles_m;
  const bool removes_round = (t_main + n_cu - 1) / n_cu < (t + n_cu - 1) / n_cu;
  const bool tail_fits = 2 * ct * tiles_m <= n_cu;
  return (removes_round && tail_fits) ? tiles_n - ct : tiles_n;
}

// Sum of S partial planes [M, ldw] (plane stride M * ldw floats) in plane order into the column block
// out[m, 0 .. width) of a matrix with row pitch ldo: the fixed-order finish of a split-K tail launch.
__global__ __launch_bounds__(256) void splitk_tail_reduce_kernel(const float* __restrict__ ws, int S, int M, int ldw,
                                                                 float* __restrict__ out, int ldo, int width) {
  const int w4 = width >> 2;
  const size_t n = (size_t)M * w4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const int m = (int)(i / w4), c = (int)(i - (size_t)m * w4) * 4;
    float4 acc = *reinterpret_cast<const float4*>(ws + (size_t)m * ldw + c);
    for (int p = 1; p < S; ++p) {
      const float4 v = *reinterpret_cast<const float4*>(ws + ((size_t)p * M + m) * ldw + c);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    *reinterpret_cast<float4*>(out + (size_t)m * ldo + c) = acc;
  }
}

// Weight-gradient form on a grid of more than one round: when the last round would be nearly empty and carving
// the trailing tile columns off removes it (the rule of full_tile_columns), those columns are a second launch
// whose tiles are split along K into TAIL_SPLIT ranges (so the tail fills the CUs for half a round instead of a
// fraction of them for a whole one); each range writes its own compact partial plane into the scratch and the
// planes are added in range order.  Returns the tile columns of the plain launch (tiles_n = no tail).
constexpr int TAIL_SPLIT = 2;
inline int wgrad_full_tile_columns(const GemmArgs& g, int tiles_m, int tiles_n, int n_cu, bool have_scratch) {
  if (!have_scratch || g.R || g.out_dtype != F32) return tiles_n;
  const int cn = full_tile_columns(tiles_m, tiles_n, n_cu);
  if (cn <= 0 || cn >= tiles_n) return tiles_n;
  const int steps = (g.K + DBK - 1) / DBK;
  const int width = g.N - cn * BN;
  if (steps < 16 * TAIL_SPLIT || (width & 3) || (g.ldc & 3)) return tiles_n;
  return cn;
}
inline size_t wgrad_tail_scratch_bytes(const GemmArgs& g, int cn) { return (size_t)TAIL_SPLIT * g.M * (g.N - cn * BN) * 4; }

// Split-K factor for a grid of t tiles and a contraction of K: as many ranges as fit the CUs, each at
// least 16 steps deep, at most 16 ranges; 1 = no split.  A pure function of the shape and the device.
inline int splitk_factor(int t, int K, int n_cu) {
  if (2 * t > n_cu) return 1;
  const int steps = (K + DBK - 1) / DBK;
  return std::max(1, std::min(std::min(n_cu / t, steps / 16), 16));
}

// Launch of the direct-to-LDS kernel for the forms with A K-contiguous, per the cut above.
template <bool B_KC, typename TO, bool HAS_R, int ACT, bool F16IN = false>
hipError_t launch_a_kc(const GemmArgs& g, hipStream_t s) {
  constexpr int WMv = dl_wm(true, B_KC), WNv = dl_wn(true, B_KC);
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const int cn = full_tile_columns(tiles_m, tiles_n, cu_count());
  if (cn > 0)
    hipLaunchKernelGGL((gemm_mfma_dl_kernel<true, B_KC, TO, HAS_R, WMv, WNv, ACT, 256, F16IN>), dim3(tiles_m * cn), dim3(WMv * WNv * 64),
                       0, s, (const bf16_t*)g.A, (const bf16_t*)g.B, (TO*)g.C, g.R, g.M, g.N, g.K, g.lda, g.ldb, g.ldc,
                       g.ldr, tiles_m, cn, (bf16_t*)g.E, g.lde, 0, 0, (const bf16_t*)g.bias, g.out_scale);
  if (cn < tiles_n) {
    const int tiles_m2 = (g.M + 127) / 128;
    hipLaunchKernelGGL((gemm_mfma_dl_kernel<true, B_KC, TO, HAS_R, WMv, WNv, ACT, 128, F16IN>), dim3(tiles_m2 * (tiles_n - cn)),
                       dim3(WMv * WNv * 64), 0, s, (const bf16_t*)g.A, (const bf16_t*)g.B, (TO*)g.C, g.R, g.M, g.N, g.K,
                       g.lda, g.ldb, g.ldc, g.ldr, tiles_m2, tiles_n - cn, (bf16_t*)g.E, g.lde, cn, 0, (const bf16_t*)g.bias, g.out_scale);
  }
  return hipGetLastError();
}

template <bool A_KC, bool B_KC, typename TO, bool HAS_R>
hipError_t launch_one(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  if (direct_ok(g)) {
    if constexpr (A_KC) return launch_a_kc<B_KC, TO, HAS_R, ACT_NONE>(g, s);
    // Weight-gradient form (both operands K-strided, fp32 out, K = tokens): when the output has too
    // few tiles to fill the CUs, the contraction is split into S ranges, every range writes its own
    // partial plane into the scratch, and the planes are summed in range order (one fixed order).
    if constexpr (!A_KC && !B_KC && !HAS_R && sizeof(TO) == 4) {
      const int S = splitk_factor(tiles_m * tiles_n, g.K, cu_count());
      if (S > 1 && g.ws && g.ldc == g.N && (size_t)S * g.M * g.N * 4 <= g.ws_bytes && ((size_t)g.M * g.N) % 4 == 0) {
        const int steps = (g.K + DBK - 1) / DBK, k_split = (steps + S - 1) / S * DBK;
        const int S_eff = (g.K + k_split - 1) / k_split;
        hipLaunchKernelGGL((gemm_mfma_dl_kernel<A_KC, B_KC, TO, HAS_R, dl_wm(A_KC, B_KC), dl_wn(A_KC, B_KC), ACT_NONE>),
                           dim3(tiles_m * tiles_n, S_eff), dim3(dl_wm(A_KC, B_KC) * dl_wn(A_KC, B_KC) * 64), 0,
                           s, (const bf16_t*)g.A, (const bf16_t*)g.B, (TO*)g.ws, g.R, g.M, g.N, g.K, g.lda,
                           g.ldb, g.ldc, g.ldr, tiles_m, tiles_n, (bf16_t*)nullptr, 0, 0, k_split, (const bf16_t*)nullptr, (const float*)nullptr);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_grad_reduce((const float*)g.ws, (size_t)g.M * g.N, S_eff, (float*)g.C, (size_t)g.M * g.N, s);
      }
      const int cn = wgrad_full_tile_columns(g, tiles_m, tiles_n, cu_count(), g.ws != nullptr);
      if (cn < tiles_n && wgrad_tail_scratch_bytes(g, cn) <= g.ws_bytes && ((uintptr_t)g.ws & 15) == 0) {
        constexpr int WMv = dl_wm(A_KC, B_KC), WNv = dl_wn(A_KC, B_KC);
        const int ct = tiles_n - cn, width = g.N - cn * BN;
        const int steps = (g.K + DBK - 1) / DBK, k_split = (steps + TAIL_SPLIT - 1) / TAIL_SPLIT * DBK;
        hipLaunchKernelGGL((gemm_mfma_dl_kernel<A_KC, B_KC, TO, HAS_R, WMv, WNv, ACT_NONE>), dim3(tiles_m * cn), dim3(WMv * WNv * 64), 0,
                           s, (const bf16_t*)g.A, (const bf16_t*)g.B, (TO*)g.C, g.R, g.M, g.N, g.K, g.lda, g.ldb, g.ldc, g.ldr,
                           tiles_m, cn, (bf16_t*)nullptr, 0, 0, 0, (const bf16_t*)nullptr, (const float*)nullptr);
        // the tail's planes are compact ([M, width]); the kernel addresses columns by their index in C, so the
        // plane pointer is moved left by the tail's first column (never dereferenced outside the planes)
        float* ws_shifted = (float*)g.ws - (size_t)cn * BN;
        hipLaunchKernelGGL((gemm_mfma_dl_kernel<A_KC, B_KC, TO, HAS_R, WMv, WNv, ACT_NONE>), dim3(tiles_m * ct, TAIL_SPLIT),
                           dim3(WMv * WNv * 64), 0, s, (const bf16_t*)g.A, (const bf16_t*)g.B, (TO*)ws_shifted, g.R, g.M, g.N, g.K,
                           g.lda, g.ldb, width, g.ldr, tiles_m, ct, (bf16_t*)nullptr, 0, cn, k_split, (const bf16_t*)nullptr, (const float*)nullptr);
        const size_t n4 = (size_t)g.M * (width / 4);
        hipLaunchKernelGGL(splitk_tail_reduce_kernel, dim3((unsigned)std::min<size_t>((n4 + 255) / 256, 8192)), dim3(256), 0, s,
                           (const float*)g.ws, TAIL_SPLIT, g.M, width, (float*)g.C + (size_t)cn * BN, g.ldc, width);
        return hipGetLastError();
      }
    }
    hipLaunchKernelGGL((gemm_mfma_dl_kernel<A_KC, B_KC, TO, HAS_R, dl_wm(A_KC, B_KC), dl_wn(A_KC, B_KC), ACT_NONE>),
                       dim3(tiles_m * tiles_n), dim3(dl_wm(A_KC, B_KC) * dl_wn(A_KC, B_KC) * 64), 0,
                       s, (const bf16_t*)g.A, (const bf16_t*)g.B, (TO*)g.C, g.R, g.M, g.N, g.K, g.lda,
                       g.ldb, g.ldc, g.ldr, tiles_m, tiles_n, (bf16_t*)nullptr, 0, 0, 0, (const bf16_t*)g.bias, g.out_scale);
    return hipGetLastError();
  }
  static std::once_flag once;       // per instantiation; the attribute is process-wide for the function
  static hipError_t once_status = hipSuccess;
  if (hipError_t e = set_max_dynamic_lds_once(once, once_status, (const void*)gemm_mfma_kernel<A_KC, B_KC, TO, HAS_R>, SMEM_BYTES);
      e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_mfma_kernel<A_KC, B_KC, TO, HAS_R>), dim3(tiles_m * tiles_n), dim3(NTHREADS), SMEM_BYTES, s,
                     (const bf16_t*)g.A, (const bf16_t*)g.B, (TO*)g.C, g.R, g.M, g.N, g.K, g.lda, g.ldb,
                     g.ldc, g.ldr, tiles_m, tiles_n);
  return hipGetLastError();
}

template <bool A_KC, bool B_KC>
hipError_t launch_orient(const GemmArgs& g, hipStream_t s) {
  if (g.out_dtype == F32) return g.R ? launch_one<A_KC, B_KC, float, true>(g, s) : launch_one<A_KC, B_KC, float, false>(g, s);
  return g.R ? launch_one<A_KC, B_KC, bf16_t, true>(g, s) : launch_one<A_KC, B_KC, bf16_t, false>(g, s);
}

}  // namespace

// Fused-activation launch: forward forms are (A K-contiguous, B K-strided), backward forms (both K-contiguous).
template <bool B_KC, int ACT>
hipError_t launch_act(const GemmArgs& g, hipStream_t s) {
  return launch_a_kc<B_KC, bf16_t, false, ACT>(g, s);
}

bool gemm_act_supported(const GemmArgs& g) {
  if (g.act == ACT_NONE) return true;
  if (!gemm_mfma_supports(g) || !direct_ok(g) || g.R || g.out_dtype != BF16 || !g.E || (g.lde & 7) ||
      ((uintptr_t)g.E & 15) || g.transA)
    return false;
  static_assert(dl_wm(true, false) == 2 && dl_wn(true, false) == 4 && dl_wn(true, true) == 4, "epilogue pairing assumes 2x4 wavefronts");
  switch (g.act) {
    case ACT_SWIGLU_FWD: return !g.transB && (g.N % 256) == 0;          // F a multiple of 128: whole paired tiles
    case ACT_GELU_FWD: return !g.transB;
    case ACT_SWIGLU_BWD: case ACT_GELU_BWD: return g.transB;
    default: return false;
  }
}

// How launch_gemm_mfma would cut g (without an activation) on a device with n_cu compute units: the same
// decisions as the launchers above, without touching the device.
GemmPlan gemm_mfma_plan(const GemmArgs& g, int n_cu, bool have_scratch) {
  GemmPlan p{};
  if (!gemm_mfma_supports(g)) return p;
  const bool a_kc = !g.transA, b_kc = g.transB;
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  p.wavefronts = direct_ok(g) ? dl_wm(a_kc, b_kc) * dl_wn(a_kc, b_kc) : NTHREADS / 64;
  p.split_k = 1;
  if (!direct_ok(g)) {
    p.kernel = 2;
    p.main_workgroups = tiles_m * tiles_n;
    return p;
  }
  p.kernel = 1;
  if (a_kc) {
    const int cn = full_tile_columns(tiles_m, tiles_n, n_cu);
    p.main_workgroups = tiles_m * cn;
    p.short_workgroups = ((g.M + 127) / 128) * (tiles_n - cn);
    return p;
  }
  p.main_workgroups = tiles_m * tiles_n;
  if (!b_kc && !g.R && g.out_dtype == F32 && have_scratch) {
    const int S = (g.ldc == g.N && ((size_t)g.M * g.N) % 4 == 0) ? splitk_factor(tiles_m * tiles_n, g.K, n_cu) : 1;
    if (S > 1) {
      const int steps = (g.K + DBK - 1) / DBK, k_split = (steps + S - 1) / S * DBK;
      p.split_k = (g.K + k_split - 1) / k_split;
    } else {
      const int cn = wgrad_full_tile_columns(g, tiles_m, tiles_n, n_cu, true);
      if (cn < tiles_n) {   // plain launch over cn tile columns + a tail launch split along K
        p.main_workgroups = tiles_m * cn;
        p.short_workgroups = tiles_m * (tiles_n - cn) * TAIL_SPLIT;
        p.split_k = TAIL_SPLIT;
      }
    }
  }
  return p;
}

bool gemm_mfma_supports(const GemmArgs& g) {
  if (g.in_dtype != BF16 && g.in_dtype != F16) return false;
  if (g.in_dtype == F16 || g.out_dtype == F16) {
    // half forms: QKV projection (half x half -> half, NN), output projection (half x half -> fp32 + residual, NN)
    // and dO (bf16 x bf16 -> half, NT); direct-load kernel only
    const bool qkv_form = g.in_dtype == F16 && g.out_dtype == F16 && !g.transA && !g.transB && !g.R;
    const bool wo_form = g.in_dtype == F16 && g.out_dtype == F32 && !g.transA && !g.transB && g.R;
    const bool do_form = g.in_dtype == BF16 && g.out_dtype == F16 && !g.transA && g.transB && !g.R;
    if (!(qkv_form || wo_form || do_form) || g.act != ACT_NONE || !direct_ok(g)) return false;
  }
  if (g.bias && (!direct_ok(g) || ((uintptr_t)g.bias & 15))) return false;   // bias lives in the direct-load kernel's epilogue
  if (g.M < 1 || g.N < 1 || g.K < 1) return false;
  if ((g.lda | g.ldb | g.ldc) & 7) return false;
  if (g.R && ((g.ldr & 3) || ((uintptr_t)g.R & 15))) return false;
  if (g.N & 7) return false;
  const bool a_kc = !g.transA, b_kc = g.transB;
  if ((a_kc || b_kc) && (g.K & 7)) return false;      // K-contiguous chunks must be whole
  if (!a_kc && (g.M & 7)) return false;               // K-strided A: rows of C come in chunks of 8
  auto aligned = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  return aligned(g.A) && aligned(g.B) && aligned(g.C);
}

hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s) {
  if (!gemm_mfma_supports(g)) return hipErrorInvalidValue;
  if (g.act != ACT_NONE) {
    if (!gemm_act_supported(g)) return hipErrorInvalidValue;
    switch (g.act) {
      case ACT_SWIGLU_FWD: return launch_act<false, ACT_SWIGLU_FWD>(g, s);
      case ACT_GELU_FWD: return launch_act<false, ACT_GELU_FWD>(g, s);
      case ACT_SWIGLU_BWD: return launch_act<true, ACT_SWIGLU_BWD>(g, s);
      default: return launch_act<true, ACT_GELU_BWD>(g, s);
    }
  }
  const bool a_kc = !g.transA, b_kc = g.transB;
  if (g.in_dtype == F16 && g.out_dtype == F32) return launch_a_kc<false, float, true, ACT_NONE, true>(g, s);
  if (g.in_dtype == F16) return launch_a_kc<false, f16_t, false, ACT_NONE, true>(g, s);
  if (g.out_dtype == F16) return launch_a_kc<true, f16_t, false, ACT_NONE, false>(g, s);
  if (a_kc && !b_kc) return launch_orient<true, false>(g, s);
  if (a_kc && b_kc) return launch_orient<true, true>(g, s);
  if (!a_kc && !b_kc) return launch_orient<false, false>(g, s);
  return launch_orient<false, true>(g, s);
}

}  // namespace rrfp
