// Pieces shared by the MFMA attention kernels (attn_mfma.hip, attn_mfma_dq.hip): vector types,
// fragment reads from LDS tiles, and the global -> register -> LDS tile movers.
//
// Element types.  q, k, v and the kernels' copy of dO are IEEE halves (el_t), and so are the probabilities
// and dS formed in registers: every matrix product here is a v_mfma_f32_32x32x16_f16.  The score S = q k^T
// feeds an exponential, so a relative error e in q or k becomes an error |S| e in log-probability; with
// bf16 operands (e = 2^-9) that is what dominated the error of the whole stage, with halves (2^-12) it does
// not.  The attention OUTPUT and the gradients dq, dk, dv are written in bf16 (they feed bf16 GEMMs against
// bf16 weights and bf16 gradients).
#pragma once

#include "kernels.h"
#include "numeric.h"

#include <type_traits>

namespace rrfp {
namespace {

typedef f16_t el_t;                                            // element type of q, k, v, dO
typedef _Float16 frag_t __attribute__((ext_vector_type(8)));   // eight of them: one MFMA operand fragment per lane
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;

// Eight fp32 values (probabilities or dS, in range by construction) -> one operand fragment; one conversion
// instruction per pair (truncating: a relative error below 2^-11, a quarter of bf16's rounding error).
__device__ __forceinline__ frag_t pack8(const float* p) {
  uint4 w;
  w.x = pack_f16x2_rtz(p[0], p[1]); w.y = pack_f16x2_rtz(p[2], p[3]);
  w.z = pack_f16x2_rtz(p[4], p[5]); w.w = pack_f16x2_rtz(p[6], p[7]);
  return __builtin_bit_cast(frag_t, w);
}
__device__ __forceinline__ floatx16 mfma16(frag_t a, frag_t b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

constexpr int BKV = 64;        // keys per step
constexpr int FWD_Q_ROWS = ATTN_TILE_Q;   // query rows per workgroup of the forward kernel (the dQ kernel uses the same tiles)
constexpr int FWD_NIB = 1;                // 32-query blocks per wavefront: 8 wavefronts, two per SIMD, so that one
                                          // wavefront's softmax arithmetic runs under the other's MFMAs

// Fragment of a tile stored [row][k] (pitch bytes): lane gets row row0 + (lane & 31), k = ks*16 + h*8 .. +8.
__device__ __forceinline__ frag_t frag_rows(const char* tile, int pitch, int row0, int ks, int lane) {
  const uint4 v = *reinterpret_cast<const uint4*>(tile + (row0 + (lane & 31)) * pitch + (ks * 2 + (lane >> 5)) * 16);
  return __builtin_bit_cast(frag_t, v);
}

// Transposed fragment of a tile stored [k][col] (pitch bytes): lane gets column col0 + (lane & 31) and
// the eight k values kstart + {0..3} and kstart + 8 + {0..3}, kstart = k0 + (lane >> 5) * 4.  This is the
// k order in which a 32x32 accumulator block, packed to bf16, serves as the other MFMA operand.
__device__ __forceinline__ frag_t frag_cols_tr(const char* tile, int pitch, int k0, int col0, int lane) {
  const int krow = k0 + (lane >> 5) * 4 + ((lane & 15) >> 2);
  const int col = col0 + ((lane >> 4) & 1) * 16 + (lane & 3) * 4;
  union { short4v hh[2]; frag_t v; } f;
  f.hh[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(tile + krow * pitch + col * 2));
  f.hh[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(tile + (krow + 8) * pitch + col * 2));
  return f.v;
}

// Generic tile movers: ROWS x D bf16 from global rows [row0, row_end) into registers, then into
// LDS with a row pitch of PITCH bytes; columns D .. DPAD-1 are zero-filled.
template <int D, int ROWS, int NT = 256>
struct TileRegs { static constexpr int N = (ROWS * (D / 8) + NT - 1) / NT; };
template <int D, int ROWS, int NT = 256>
using TileArr = uint4[TileRegs<D, ROWS, NT>::N];

template <int D, int ROWS, int NT = 256>
__device__ __forceinline__ void tile_load(TileArr<D, ROWS, NT>& r, const el_t* __restrict__ base, int ld,
                                          int row0, int row_end) {
  constexpr int CH = D / 8;
#pragma unroll
  for (int i = 0; i < TileRegs<D, ROWS, NT>::N; ++i) {
    const int q = i * NT + threadIdx.x;
    const int row = q / CH, c = q - row * CH;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (q < ROWS * CH && row0 + row < row_end) v = *reinterpret_cast<const uint4*>(base + (size_t)(row0 + row) * ld + c * 8);
    r[i] = v;
  }
}

// The same without branches: rows at or past row_end (row_end > row0) re-read row row_end - 1, and a lane
// whose chunk lies past the tile re-reads the tile's last chunk (tile_store drops it).  For tiles whose
// rows past the end only ever meet zero weights.
template <int D, int ROWS, int NT = 256>
__device__ __forceinline__ void tile_load_clamped(TileArr<D, ROWS, NT>& r, const el_t* __restrict__ base, int ld,
                                                  int row0, int row_end) {
  constexpr int CH = D / 8;
#pragma unroll
  for (int i = 0; i < TileRegs<D, ROWS, NT>::N; ++i) {
    const int q = min(i * NT + (int)threadIdx.x, ROWS * CH - 1);
    const int row = q / CH, c = q - row * CH;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // a plain vector load: the register array stays in registers
    r[i] = __builtin_bit_cast(uint4, *reinterpret_cast<const u32x4*>(base + (size_t)min(row0 + row, row_end - 1) * ld + c * 8));
  }
}

// STATIC_FULL: leave out the per-chunk guard where the chunk count is a multiple of the thread count (the guard
// is always true there, but as a run-time test it splits the caller's basic block).
template <int D, int ROWS, int PITCH, int DPAD, int NT = 256, bool STATIC_FULL = false>
__device__ __forceinline__ void tile_store(const TileArr<D, ROWS, NT>& r, char* lds) {
  constexpr int CH = D / 8;
#pragma unroll
  for (int i = 0; i < TileRegs<D, ROWS, NT>::N; ++i) {
    const int q = i * NT + threadIdx.x;
    const int row = q / CH, c = q - row * CH;
    if ((STATIC_FULL && (ROWS * CH) % NT == 0) || q < ROWS * CH) *reinterpret_cast<uint4*>(lds + row * PITCH + c * 16) = r[i];
  }
  if (DPAD != D) {
    constexpr int PADCH = (DPAD - D) / 8;
    for (int q = threadIdx.x; q < ROWS * PADCH; q += NT) {
      const int row = q / PADCH, c = q - row * PADCH;
      *reinterpret_cast<uint4*>(lds + row * PITCH + (CH + c) * 16) = make_uint4(0, 0, 0, 0);
    }
  }
}


// Output of a transposed accumulator block.  A 32x32 accumulator of the kernels here holds 32 consecutive head-dimension
// values (rows) of 32 output rows (one per lane of a half-wavefront): stored from there, every lane writes to a row of
// its own, 8 or 16 bytes at a time, and one store instruction becomes up to 64 separate write requests.  Instead the
// wavefront passes the block through a private LDS area and reads it back with 8 lanes side by side on each output row
// (4 values per lane, 8 rows per sweep), so that a store instruction writes 64 or 128 contiguous bytes per row.
// st: this wavefront's area of OUT_STAGE_BYTES; v = the block times mul; emit(row 0..31, first of 4 head-dimension
// values 0..28, the 4 values).  The area is private to the wavefront and the hardware runs one wavefront's LDS instructions
// in order: the wavefront-scope fences only keep the compiler from reordering the phases.
constexpr int OUT_PITCH = 36;                       // floats per staged row: 32 values + a 16-byte skew
constexpr int OUT_STAGE_BYTES = 32 * OUT_PITCH * 4;
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
template <typename Emit>
__device__ __forceinline__ void emit_block_rows(float* st, const floatx16& acc, float mul, int lane, Emit&& emit) {
  const int h = lane >> 5, li = lane & 31;
  wave_lds_sync();       // the read-back of the block before precedes these writes
#pragma unroll
  for (int g = 0; g < 4; ++g)
    *reinterpret_cast<float4*>(st + li * OUT_PITCH + g * 8 + h * 4) =
        make_float4(acc[g * 4 + 0] * mul, acc[g * 4 + 1] * mul, acc[g * 4 + 2] * mul, acc[g * 4 + 3] * mul);
  wave_lds_sync();
#pragma unroll
  for (int sw = 0; sw < 4; ++sw) {
    const int row = sw * 8 + (lane >> 3), c = (lane & 7) * 4;
    emit(row, c, *reinterpret_cast<const float4*>(st + row * OUT_PITCH + c));
  }
}

}  // namespace
}  // namespace rrfp
