// Internal launcher interface between the stage host code and the gfx950 kernels.
// Every launcher only enqueues on the given stream and returns the launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

namespace rrfp {

// F16 (IEEE half) is internal: the library's own copies of forward activations on the path into the
// attention scores.  It never appears at the C interface (STAGE_DTYPE_* has fp32 and bf16 only).
enum DType : int { F32 = 0, BF16 = 1, F16 = 2 };

static inline size_t dtype_size(int dt) { return dt == F32 ? 4 : 2; }

// Raises a kernel's dynamic LDS limit once per process, safely under concurrent first calls from several
// host threads.  `flag` and `status` are statics of the calling launcher (one pair per kernel instantiation).
static inline hipError_t set_max_dynamic_lds_once(std::once_flag& flag, hipError_t& status, const void* kernel, int bytes) {
  std::call_once(flag, [&] { status = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
  return status;
}

// C[M,N] = A(m,k) * B(k,n) (+ R[M,N]), fp32 accumulation.  R, when present, is always fp32 (the
// residual stream is kept in fp32 between layers whatever the storage type).
//   transA == false: A stored [M,K] (lda), true: stored [K,M] (lda).
//   transB == false: B stored [K,N] (ldb), true: stored [N,K] (ldb).
// in_dtype is the type of A and B; out_dtype the type of C (F32 for weight gradients and for the
// residual stream).
// Optional activation fused into the epilogue (bf16 MFMA kernel only; see gemm_act_supported):
//   ACT_SWIGLU_FWD  N = 2F, B = [K, 2F] (gate columns then up columns).  C [M, 2F] receives gate|up,
//                   E [M, F] (lde) receives m = silu(gate) * up computed from the fp32 accumulators.
//   ACT_GELU_FWD    N = F.  C [M, F] receives u, E [M, F] receives gelu(u).
//   ACT_SWIGLU_BWD  N = F, the product is dm (not stored).  E [M, 2F] (lde) holds gate|up of the forward;
//                   C [M, 2F] receives dgate|dup.
//   ACT_GELU_BWD    N = F.  E [M, F] holds u; C [M, F] receives du = dm * gelu'(u).
enum GemmAct : int { ACT_NONE = 0, ACT_SWIGLU_FWD = 1, ACT_GELU_FWD = 2, ACT_SWIGLU_BWD = 3, ACT_GELU_BWD = 4 };

struct GemmArgs {
  const void* A; const void* B; void* C; const float* R;
  int M, N, K;
  int lda, ldb, ldc, ldr;
  bool transA, transB;
  int in_dtype, out_dtype;
  int act;         // GemmAct
  void* E;         // activation operand (see GemmAct); written for *_FWD, read for *_BWD
  int lde;
  void* ws;        // optional scratch for split-K partial results (fp32), else null
  size_t ws_bytes;
  const void* bias; // optional [N] vector of the storage type added to every row before residual / activation
  const float* out_scale;  // optional device scalar (a power of two) multiplied into a plain 16-bit output before rounding
};
bool gemm_act_supported(const GemmArgs& g);   // true if launch_gemm can run g.act fused for this shape
hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);       // picks the kernel family
hipError_t launch_gemm_simt(const GemmArgs& g, hipStream_t s);  // fp32-FMA tiles, any shape
hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s);  // bf16 MFMA kernels (256-wide tiles)
bool gemm_mfma_supports(const GemmArgs& g);                     // alignment / divisibility rules
// Launch plan of launch_gemm_mfma for a shape (pure host logic): kernel 0 = refused, 1 = direct-to-LDS,
// 2 = register-staged; workgroups of the 256-row launch and of the 128-row launch; split-K ranges.
struct GemmPlan { int kernel, wavefronts, main_workgroups, short_workgroups, split_k; };
GemmPlan gemm_mfma_plan(const GemmArgs& g, int n_cu, bool have_scratch);

// One attention work item: a tile of rows [r0, r1) inside the segment [s0, s1).  kb0 = number of 32-key blocks in
// the segments before this one (each segment rounded up): the segment's first block row in the dS scratch.
struct AttnTile { int32_t r0, r1, s0, s1, kb0; };

constexpr int ATTN_TILE_Q = 256;   // rows per query tile (forward and dQ kernels)
constexpr int ATTN_TILE_KV = 128;  // rows per key tile (dK/dV kernel)

struct AttnArgs {
  const void* qkv;      // [T, (nq + 2 nkv) d]: Q heads, K heads, V heads.  dtype BF16 (the MFMA kernels): IEEE halves,
                        // and so is d_o; the outputs o and dqkv are bf16.  dtype F32: everything fp32.
  void* o;              // [T, nq d]
  float* o32;           // [T, nq d] fp32 copy of o before rounding (bf16 MFMA path; else null): the
                        // backward forms delta from it so that rounding o does not break sum_j dS_ij = 0
  void* o16;            // [T, nq d] optional copy of o as IEEE halves (MFMA path): operand of the output projection
  float* lse;           // [nq, T]   log-sum-exp of the scaled, masked scores (natural log)
  const AttnTile* q_tiles; int n_q_tiles;     // device pointers to the tile lists
  const AttnTile* kv_tiles; int n_kv_tiles;
  int T, nq, nkv, d, causal, dtype;
  // backward only
  const void* d_o;      // [T, nq d]
  void* dqkv;           // [T, (nq + 2 nkv) d]
  float* delta;         // [nq, T]   rowsum(dO * O)
  const float* grad_scale;  // MFMA path, optional: device pair {s, 1/s}; d_o holds s * dO (s a power of two that keeps
                            // the half copy of dO in range), the kernels multiply dq, dk, dv by 1/s before rounding
  void* ds;                 // MFMA path: scratch of attn_ds_bytes(...) bytes.  The dK/dV kernel leaves dS there (IEEE halves,
                            // one 4 KB block per 32 keys x 64 queries of a head) and the dQ kernel contracts it with K
  int ds_rows, ds_nqs;      // its shape: 32-key block rows per head, 64-query steps per block row
  float* dkv_part;          // MFMA path with grouped query heads (nq > nkv): attn_dkv_part_bytes(...) bytes for the partial dK / dV
                            // planes of the head subsets (see attn_dkv_subsets); null = one workgroup walks the whole group
};
// Shape of the dS scratch for up to T tokens in up to n_seg segments, and its size for nq query heads.
inline int attn_ds_rows(int T, int n_seg) { return (T + 31) / 32 + n_seg; }
inline int attn_ds_nqs(int T) { return (T + 63) / 64 + 4; }
inline size_t attn_ds_bytes(int T, int n_seg, int nq) { return (size_t)nq * attn_ds_rows(T, n_seg) * attn_ds_nqs(T) * 4096; }
// Head subsets of the dK/dV kernel (a pure function of shape and CU count).  A workgroup of that kernel owns 128 keys of a
// KV head and walks all query heads of its group; with few KV heads the grid nkv x n_kv_tiles is about one workgroup per CU
// and, under a causal mask, the longest of them sets the time.  The group is then dealt to the smallest number of subsets
// (a divisor of the group size, at most ATTN_DKV_MAX_SUBSETS) that gives two workgroups per CU, each subset summing into
// an fp32 partial plane; the planes are added in subset order.
constexpr int ATTN_DKV_MAX_SUBSETS = 4;
inline int attn_dkv_subsets(int nq, int nkv, int n_kv_tiles, int n_cu) {
  const int G = nq / nkv;
  int best = 1;
  for (int s = 1; s <= G && s <= ATTN_DKV_MAX_SUBSETS; ++s) {
    if (G % s) continue;
    best = s;
    if ((long long)nkv * n_kv_tiles * s >= 2LL * n_cu) break;
  }
  return best;
}
// Bytes of AttnArgs::dkv_part for up to T tokens: room for the most subsets the rule above can pick; 0 without grouped heads.
inline size_t attn_dkv_part_bytes(int T, int nq, int nkv, int d) {
  if (nq == nkv) return 0;
  return (size_t)2 * attn_dkv_subsets(nq, nkv, 1, 1 << 30) * T * nkv * d * 4;
}
hipError_t launch_attn_fwd(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_fwd_simt(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd_simt(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_fwd_mfma(const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_bwd_mfma(const AttnArgs& a, hipStream_t s);
bool attn_mfma_supports(const AttnArgs& a);

// dst[i] = (float)src[i]: storage type -> fp32 (entry of the residual stream).
// copy (optional): also receives src unchanged, in the storage type.
hipError_t launch_widen(const void* src, float* dst, size_t n, int dtype, hipStream_t s, void* copy = nullptr);
// Gradient scale of a microbatch from its output gradient dy [n] (storage type): scale[0] = s = 2^-floor(log2 max|dy|)
// (1 if dy is all zero or not finite), scale[1] = 1/s.  partial: device scratch of grad_scale_partials(n) floats.
int grad_scale_partials(size_t n);
hipError_t launch_grad_scale(const void* dy, size_t n, int dtype, float* partial, float* scale, hipStream_t s);
// Rotary embedding, in place, on the first n_heads heads (head_dim d, even) of every row of a [T, ld]
// tensor: pair (x_i, x_{i+d/2}) turns by sign * pos * base^(-2i/d), pos = row - segment start, rows and
// segment starts taken from the query tile list (the tiles partition the rows).
hipError_t launch_rope(void* x, const AttnTile* q_tiles, int n_q_tiles, int n_heads, int d, int ld, float base,
                       float sign, int dtype, hipStream_t s);

// h = x * r * g, r = rsqrt(mean(x^2) + eps); x fp32, r_out [T] fp32, g and h storage type.
// h16 (optional, bf16 storage only): the same output rounded to IEEE half instead of bf16, [T, H].
hipError_t launch_rmsnorm_fwd(const float* x, const void* g, void* h, float* r_out,
                              int T, int H, float eps, int dtype, hipStream_t s, void* h16 = nullptr);
// dst[i] = (half)src[i] for n bf16 values (n a multiple of 8, 16-byte aligned pointers); saturating.
hipError_t launch_bf16_to_f16(const void* src, void* dst, size_t n, hipStream_t s);

constexpr int NORM_BWD_ROWS = 64;  // rows per partial of the gain-gradient column sum (unfused kernels)
// Number of partial rows launch_rmsnorm_bwd writes for this shape (a pure function of shape and dtype:
// the fused kernel writes one per 8 rows, the unfused pair one per 64).
int norm_bwd_partials(int T, int H, int dtype);
// dx = add_in + r * (w - xhat * mean(w * xhat)), w = dh * g, xhat = x * r; dh, x and add_in fp32.
// dx is written to out32 (fp32) and/or out_t (storage type); either may be null.
// dg_partial [norm_bwd_partials(T, H, dtype), H] fp32 receives per-row-chunk sums of dh * xhat;
// launch_colsum then adds the partials in chunk order into dg [H].
hipError_t launch_rmsnorm_bwd(const float* dh, const float* x, const float* r, const void* g,
                              const float* add_in, float* out32, void* out_t, float* dg_partial,
                              int T, int H, int dtype, hipStream_t s);
hipError_t launch_colsum(const float* partial, int n_partial, int H, float* out, hipStream_t s);
// LayerNorm (model-fidelity variant): forward saves r and mu per row; backward writes dx (+ add_in) and
// the per-chunk partial sums of the gain and bias gradients ([colsum_chunks(T), H] each, for launch_colsum).
int colsum_chunks(int T);
hipError_t launch_layernorm_fwd(const float* x, const void* g, const void* b, void* h, float* r_out, float* mu_out,
                                int T, int H, float eps, int dtype, hipStream_t s, void* h16 = nullptr);
hipError_t launch_layernorm_bwd(const float* dh, const float* x, const float* r, const float* mu, const void* g,
                                const float* add_in, float* out32, void* out_t, float* partial_g, float* partial_b,
                                int T, int H, int dtype, hipStream_t s);
// Head norm (QK-norm variant): RMSNorm over head_dim of the first n_heads heads of every row of a [T, ld]
// tensor, in place; heads [0, nq) use gq, the others gk; xhat [T * n_heads, d] and r [T * n_heads] are saved.
// The backward rewrites the gradient tensor in place and writes headnorm_partials(T, heads of the kind)
// partial rows [d] of each gain gradient (for launch_colsum).
int headnorm_partials(int T, int n_heads_of_kind);
hipError_t launch_headnorm_fwd(void* x, int ld, int nq, int n_heads, int d, const void* gq, const void* gk, void* xhat,
                               float* r_out, int T, float eps, int dtype, hipStream_t s);
hipError_t launch_headnorm_bwd(void* dy, int ld, int nq, int n_heads, int d, const void* gq, const void* gk, const void* xhat,
                               const float* r_in, float* partial_q, float* partial_k, int T, int dtype, hipStream_t s,
                               float* dk32 = nullptr,    // optional fp32 copy [T, n_key_heads * d] of the rewritten key-head gradients
                               int xhat_dtype = -1);     // type of the saved xhat when it differs from dtype (F16: forward ran on a half tensor)
// Per-chunk column sums of a [T, N] tensor of the storage type into partial [colsum_chunks(T), N] (bias gradients).
hipError_t launch_colsum_rows(const void* src, int ld, float* partial, int T, int N, int dtype, hipStream_t s);

// SwiGLU on gu [T, 2F] (gate columns then up columns): m = silu(gate) * up.
hipError_t launch_swiglu_fwd(const void* gu, void* m, int T, int F, int dtype, hipStream_t s);
// dm is fp32 (a GEMM output consumed only by the activation backward).
hipError_t launch_swiglu_bwd(const float* dm, const void* gu, void* dgu, int T, int F, int dtype,
                             hipStream_t s);
// GELU (erf form) on u [T, F].
hipError_t launch_gelu_fwd(const void* u, void* m, int T, int F, int dtype, hipStream_t s);
hipError_t launch_gelu_bwd(const float* dm, const void* u, void* du, int T, int F, int dtype,
                           hipStream_t s);

// out[i] = ((slot_0[i] + slot_1[i]) + ...) + slot_{M-1}[i], slots spaced slot_stride floats apart.
hipError_t launch_grad_reduce(const float* slots, size_t slot_stride, int M, float* out, size_t n,
                              hipStream_t s);

}  // namespace rrfp
