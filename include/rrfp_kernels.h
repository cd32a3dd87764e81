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

/* How the bf16 MFMA GEMM cuts a shape into launches on a device with n_cu compute units: host logic only
 * (no GPU call, no pointers; operands are taken as 16-byte aligned).  The cut is a pure function of the
 * shape and n_cu, which is what keeps the summation order of a call fixed (the bit-exactness requirement
 * behind readiness-driven reordering, paper Section 7.1).  out[0] = kernel (0 the MFMA family refuses the
 * shape, 1 direct-to-LDS, 2 register-staged), out[1] = wavefronts per workgroup, out[2] = workgroups of
 * the 256-row-tile launch, out[3] = workgroups of the 128-row-tile launch that finishes a grid whose last
 * round would be nearly empty, out[4] = split-K ranges (weight-gradient form with scratch; 1 = none).
 * Returns STAGE_OK or STAGE_EINVAL. */
int rrfp_gemm_plan(int M, int N, int K, int lda, int ldb, int ldc, int trans_a, int trans_b, int out_dtype,
                   int have_scratch, int n_cu, int32_t out[5]);

#ifdef __cplusplus
}
#endif
#endif /* RRFP_KERNELS_H */
