/*
 * rrfp_kernels.h -- kernel-level entry points of librrfp_stage.so.
 *
 * The stage tasks of rrfp_stage.h are built from these kernels.  They are exported one by one
 * so that each can be checked against the oracle and timed against its roofline in isolation
 * (the GEMMs are the a2/a4/a5/a7 forward, a8 input-gradient and a12 weight-gradient steps of
 * the F, B and W tasks; paper Section 7.1 for the B/W decomposition).  Every call only
 * enqueues on `stream` (a hipStream_t, NULL = null stream), allocates nothing, and returns 0 or
 * a negative STAGE_E* code of rrfp_stage.h.
 */
#ifndef RRFP_KERNELS_H
#define RRFP_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { RRFP_GEMM_AUTO = 0, RRFP_GEMM_SIMT = 1, RRFP_GEMM_MFMA = 2 };

/* C[M,N] = A(m,k) B(k,n) (+ R[M,N]) with fp32 accumulation.  All pointers are device pointers.
 * trans_a == 0: A is [M,K] row-major with leading dimension lda; 1: A is stored [K,M].
 * trans_b == 0: B is [K,N] row-major with leading dimension ldb; 1: B is stored [N,K].
 * in_dtype (STAGE_DTYPE_*) is the type of A and B; out_dtype the type of C (fp32 output with bf16
 * inputs is the weight-gradient form and the residual-stream form).  R, the residual, may be NULL and
 * is ALWAYS fp32 [M,N] with leading dimension ldr: the stage keeps its residual stream in fp32.  family picks the kernel:
 * AUTO = what the stage tasks use for this shape; MFMA fails with STAGE_EINVAL when the shape
 * breaks its rules (bf16 inputs, 16-byte aligned pointers, leading dimensions and N multiples
 * of 8 (ldr of 4), K multiple of 8 if an operand is K-contiguous, M multiple of 8 if A is stored [K,M]). */
int rrfp_gemm(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda,
              int ldb, int ldc, int ldr, int trans_a, int trans_b, int in_dtype, int out_dtype,
              int family, void* stream);

/* rrfp_gemm with a caller-owned device workspace (256-byte aligned, contents undefined afterwards), as the W task
 * calls it: with a workspace the weight-gradient form (bf16 inputs, trans_a = 1, trans_b = 0, fp32 output, no
 * residual) may split the contraction into ranges that write partial planes into the workspace and are added in
 * range order (rrfp_gemm_plan with have_scratch = 1 tells which shapes do).  A workspace too small for a shape's
 * split simply disables the split.  The result is bit-identical from call to call for a given shape, workspace
 * size class and device. */
int rrfp_gemm_ws(const void* A, const void* B, void* C, const void* R, int M, int N, int K, int lda, int ldb,
                 int ldc, int ldr, int trans_a, int trans_b, int in_dtype, int out_dtype, int family,
                 void* workspace, size_t workspace_bytes, void* stream);

/* How the bf16 MFMA GEMM cuts a shape into launches on a device with n_cu compute units: host logic only
 * (no GPU call, no pointers; operands are taken as 16-byte aligned).  The cut is a pure function of the
 * shape and n_cu, which is what keeps the summation order of a call fixed (the bit-exactness requirement
 * behind readiness-driven reordering, paper Section 7.1).  out[0] = kernel (0 the MFMA family refuses the
 * shape, 1 direct-to-LDS, 2 register-staged), out[1] = wavefronts per workgroup, out[2] = workgroups of
 * the 256-row-tile launch, out[3] = workgroups of the second launch that finishes a grid whose last round
 * would be nearly empty (128-row tiles when A is K-contiguous; for the weight-gradient form with scratch the
 * trailing tile columns split along K into out[4] ranges), out[4] = split-K ranges (weight-gradient form with
 * scratch: of the whole grid when out[3] = 0, of the tail launch otherwise; 1 = none).
 * Returns STAGE_OK or STAGE_EINVAL. */
int rrfp_gemm_plan(int M, int N, int K, int lda, int ldb, int ldc, int trans_a, int trans_b, int out_dtype,
                   int have_scratch, int n_cu, int32_t out[5]);

/* Launch plan of the attention backward's dK/dV kernel, pure host logic (no HIP call): the number of workgroups that
 * share the query heads of one KV head.  A workgroup of that kernel owns 128 keys of a KV head; with grouped query
 * heads (n_q_heads > n_kv_heads) and few KV heads the grid n_kv_heads x n_kv_tiles under-fills the chip and, under a
 * causal mask, its longest workgroup sets the time, so the group is dealt to the smallest divisor of the group size
 * (at most 4) that gives two workgroups per CU; their partial sums are added in subset order (a pure function of
 * shape and n_cu: the summation order of a call is fixed, paper Section 7.1).  n_kv_tiles = key tiles of 128 rows over
 * all segments.  Returns the count (>= 1), or STAGE_EINVAL for non-positive arguments or n_q_heads not a multiple of
 * n_kv_heads. */
int rrfp_attn_dkv_subsets(int n_q_heads, int n_kv_heads, int n_kv_tiles, int n_cu);

/* ---- HBM-bound kernels of the tasks, one by one (steps a1, a10 and a13 of the F and B tasks and of the
 * gradient reduction; paper Section 3.1 for the tasks, Section 7.1 for the requirement that the result must
 * not depend on the order tasks ran in, which is why every sum here has one fixed order). ---------------- */

/* RMSNorm forward: h[t,:] = x[t,:] * r[t] * g, r[t] = (mean_c x[t,c]^2 + eps)^-1/2.  x: device fp32 [T,H]
 * (the residual stream); g: device [H] storage dtype; h: device [T,H] storage dtype, written; r_out: device
 * fp32 [T], written.  dtype = STAGE_DTYPE_*.  STAGE_EINVAL for NULL pointers or non-positive sizes. */
int rrfp_rmsnorm_fwd(const float* x, const void* g, void* h, float* r_out, int T, int H, float eps, int dtype,
                     void* stream);

/* Bytes of workspace rrfp_rmsnorm_bwd needs for this shape (partial gain-gradient rows); pure host. */
size_t rrfp_rmsnorm_bwd_workspace(int T, int H, int dtype);

/* RMSNorm backward: dx = add_in + r (w - xhat mean_c(w xhat)), w = dh g, xhat = x r; dg[c] = sum_t dh[t,c] xhat[t,c]
 * with the rows added in one fixed order (per-chunk partial rows in `workspace`, then a fixed-order column sum).
 * dh, x, add_in: device fp32 [T,H]; r: device fp32 [T]; g: device [H] storage dtype; out32 (fp32) and out_t
 * (storage dtype): device [T,H], written, either may be NULL; dg: device fp32 [H], written; workspace: device,
 * caller-owned, at least rrfp_rmsnorm_bwd_workspace bytes, 16-byte aligned, contents undefined afterwards.
 * STAGE_EINVAL for NULL inputs, a too small workspace or non-positive sizes. */
int rrfp_rmsnorm_bwd(const float* dh, const float* x, const float* r, const void* g, const float* add_in,
                     float* out32, void* out_t, float* dg, void* workspace, size_t workspace_bytes, int T, int H,
                     int dtype, void* stream);

/* out[i] = ((s_0[i] + s_1[i]) + s_2[i]) + ... + s_{M-1}[i] for i < n, slot j at slots + j * slot_stride floats.
 * All device fp32; n and slot_stride multiples of 4, pointers 16-byte aligned. */
int rrfp_grad_reduce(const float* slots, size_t slot_stride, int M, float* out, size_t n, void* stream);

/* rrfp_rmsnorm_bwd for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results (bit for
 * bit) as rrfp_rmsnorm_bwd minus the workspace: the partial gain-gradient rows go to a 16 MiB array that lives
 * in the library's device image (one copy per GPU, held until the process ends).  Calls no allocating routine.
 * STAGE_ENOMEM when rrfp_rmsnorm_bwd_workspace(T, H, dtype) exceeds rrfp_rmsnorm_bwd_static_limit() (16 MiB:
 * T * H up to 32 Mi elements for the fused kernel, e.g. 8192 x 4096); STAGE_EINVAL / STAGE_EHIP as the other
 * entry points.  All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 * (different streams without ordering) race and give undefined dg; calls ordered on one stream, or by events,
 * are safe, and nothing needs clearing between them (every row read is written first by the same call). */
size_t rrfp_rmsnorm_bwd_static_limit(void);
int rrfp_rmsnorm_bwd_static(const float* dh, const float* x, const float* r, const void* g, const float* add_in,
                            float* out32, void* out_t, float* dg, int T, int H, int dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RRFP_KERNELS_H */
