/*
 * rrfp_stage.h -- C ABI of the per-microbatch stage tasks F, B and W on one MI355X.
 *
 * Task model (paper, Section 3.1 "Execution Model and Constraints", Section 4.1
 * "Message-Driven Asynchronous Communication", Section 7.1 "Baselines", Appendix C.1
 * "Buffer Implementation Details"):
 *   - a task is identified by (microbatch id, direction);
 *   - F_j consumes the activation of microbatch j and produces the stage's output;
 *   - the backward of j needs the local F_j and the gradient from the next stage;
 *   - under the B/F/W hint the backward is decomposed: B_j produces the input
 *     gradient, W_j the weight gradients, and W_j may run whenever it is convenient
 *     after B_j;
 *   - the forward input is retained until the backward side has consumed it;
 *   - a stage may run its ready tasks in ANY order, and the order must not change
 *     the training result.
 * The layer math is an ordinary pre-norm transformer layer:
 *     h1 = RMSNorm(x; g1);  [q|k|v] = h1 Wqkv;  o = attention(q,k,v);  x1 = x + o Wo;
 *     h2 = RMSNorm(x1; g2); m = silu(h2 Wg) * (h2 Wu)  or  gelu_erf(h2 W1);  y = x1 + m Wd.
 *
 * Conventions for every entry point
 *   - returns 0 (STAGE_OK) or a negative STAGE_E* code; the message is available from
 *     stage_last_error();
 *   - "host" / "device" is stated for every pointer.  The library never allocates or
 *     frees device memory and never synchronises the device; every task call only
 *     enqueues work on the given HIP stream and returns.  One exception: stage_F copies the
 *     attention tile lists of the microbatch from a pinned host buffer owned by the slot;
 *     if the copy the SAME slot enqueued in the previous iteration has not completed yet,
 *     stage_F waits for that one copy on the host first (it precedes all kernels of that
 *     earlier task on its stream, so in steady state the wait returns at once);
 *   - all argument validation and all dependency checks happen BEFORE the first HIP call
 *     of an entry point; a call that fails validation (STAGE_EINVAL, STAGE_ENOTREADY,
 *     STAGE_ENOMEM) has no side effect.  A HIP runtime failure (STAGE_EHIP) in the middle of
 *     a task is different: part of the task may already be enqueued, so the slot is marked
 *     POISONED and every later task on it (and stage_grad_reduce) returns STAGE_EHIP, with
 *     the reason in stage_last_error, until the stage is destroyed;
 *   - calls on one stage_t must come from one host thread at a time (the arbiter thread).
 *     Tasks of different microbatches may be put on different streams; the device-side
 *     order F_j -> B_j -> W_j -> grad_reduce is enforced with library-owned events;
 *   - tensors are row-major.  Activations are [T, hidden] with the T tokens of a
 *     microbatch packed; segment s is rows cu_seqlens[s] .. cu_seqlens[s+1]-1 and attention
 *     never crosses a segment boundary.  Storage dtype is fp32 or bf16 (config); every
 *     gradient slot and grad_out are fp32;
 *   - on the bf16 path the library keeps its OWN copies of the forward activations that lead into
 *     the attention scores (first norm output, q, k, v) and of Wqkv as IEEE halves (11-bit
 *     significand), because the softmax amplifies their rounding error; interface tensors,
 *     parameters and gradients stay bf16.  The half copy of Wqkv is refreshed by the first
 *     stage_F after stage_create / stage_grad_reduce: the caller may change the parameters only
 *     between stage_grad_reduce and the next stage_F.
 */
#ifndef RRFP_STAGE_H
#define RRFP_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  STAGE_OK = 0,
  STAGE_EINVAL = -1,    /* bad config / argument / cu_seqlens / T > max_tokens / mb out of range */
  STAGE_ENOTREADY = -2, /* dependency violated: B before F, W before B, reduce before all W, F on a busy slot */
  STAGE_ENOMEM = -3,    /* arena smaller than stage_query reports */
  STAGE_EHIP = -4       /* a HIP runtime call failed; text in stage_last_error */
};

enum { STAGE_DTYPE_FP32 = 0, STAGE_DTYPE_BF16 = 1 };
enum { STAGE_MLP_SWIGLU = 0, STAGE_MLP_GELU = 1 };

/* Parameter tensors of one layer, all stored as y = x @ W with W [in, out] row-major. */
enum {
  STAGE_P_G1 = 0,   /* [hidden]                       gain of the first RMSNorm            */
  STAGE_P_WQKV = 1, /* [hidden, (n_q + 2 n_kv) d]     columns: Q heads, then K, then V     */
  STAGE_P_WO = 2,   /* [n_q d, hidden]                                                      */
  STAGE_P_G2 = 3,   /* [hidden]                       gain of the second RMSNorm           */
  STAGE_P_WUP = 4,  /* SwiGLU: [hidden, 2 ffn] gate columns then up columns; GELU: [hidden, ffn] */
  STAGE_P_WD = 5,   /* [ffn, hidden]                                                        */
  /* Vectors of the model-fidelity variants; zero-sized (shape [0, 1]) when their variant is off. */
  STAGE_P_B1 = 6,   /* [hidden]                       bias of the first LayerNorm  (norm_kind 1)  */
  STAGE_P_BQKV = 7, /* [(n_q + 2 n_kv) d]             bias of the QKV projection   (bias 1)       */
  STAGE_P_BO = 8,   /* [hidden]                       bias of the output projection (bias 1)      */
  STAGE_P_B2 = 9,   /* [hidden]                       bias of the second LayerNorm (norm_kind 1)  */
  STAGE_P_BUP = 10, /* [2 ffn] gate then up, or [ffn] bias of the up projection    (bias 1)       */
  STAGE_P_BD = 11,  /* [hidden]                       bias of the down projection  (bias 1)       */
  STAGE_P_GQ = 12,  /* [head_dim]                     gain of the query head norm  (qk_norm 1)    */
  STAGE_P_GK = 13,  /* [head_dim]                     gain of the key head norm    (qk_norm 1)    */
  STAGE_P_COUNT = 14
};

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn;
  int32_t max_tokens;     /* largest T of any microbatch                                  */
  int32_t n_microbatches; /* M: number of microbatch slots per iteration                  */
  int32_t max_segments;   /* largest number of segments in one microbatch                 */
  int32_t dtype;          /* STAGE_DTYPE_*: storage type; accumulation is always fp32     */
  int32_t mlp_kind;       /* STAGE_MLP_*                                                  */
  int32_t causal;         /* 1: key j <= query i inside a segment; 0: whole segment       */
  int32_t norm_kind;      /* 0 = RMSNorm; 1 = LayerNorm with gain and bias (model-fidelity variant):
                             h = (x - mean) * (var + eps)^-1/2 * g + b, biased variance      */
  float norm_eps;         /* added to the mean of squares inside the square root          */
  int32_t rope;           /* 0 = none; 1 = rotary position embedding on q and k (model-fidelity
                             variant; split-half pairs (x_i, x_{i+d/2}), angle pos * rope_base^(-2i/d),
                             pos = index of the token inside its own segment)              */
  float rope_base;        /* > 1 when rope = 1 (10000 in the usual models); ignored otherwise */
  int32_t bias;           /* 1 = a bias vector on each of the four projections (model-fidelity
                             variant); their gradients are column sums of the projections'
                             output-gradients, produced by stage_B like the norm gradients   */
  int32_t qk_norm;        /* 1 = RMSNorm over head_dim (same eps) on every query and key head after
                             the QKV projection and before the rotary embedding, gains STAGE_P_GQ /
                             STAGE_P_GK shared by all heads (model-fidelity variant)          */
} stage_config;

typedef struct stage_s stage_t;

/* Sizes the caller must provide (pure host computation, no HIP call).
 *   param_bytes: the parameter buffer in the storage dtype, laid out per stage_param_layout;
 *   grad_bytes:  grad_out of stage_grad_reduce (fp32, same element offsets as the parameters);
 *   arena_bytes: the work arena (activation stashes, per-microbatch gradient slots, scratch).
 * Any of the three output pointers may be NULL.  STAGE_EINVAL for an unsupported config:
 * n_q_heads not a multiple of n_kv_heads, non-positive sizes, head_dim not a multiple of 16
 * or above 128; fp32: ffn not a multiple of 4; bf16: head_dim not in {64, 80, 128}, or
 * hidden, ffn, n_q*d, n_kv*d not multiples of 64. */
int stage_query(const stage_config* cfg /*host*/, size_t* param_bytes /*host*/,
                size_t* grad_bytes /*host*/, size_t* arena_bytes /*host*/);

/* Where tensor `which` (STAGE_P_*) of `layer` lives: offset in ELEMENTS from the start of
 * the parameter buffer (storage dtype) and equally of every fp32 gradient buffer, and its
 * logical shape ([n, 1] for gains).  Pure host. */
int stage_param_layout(const stage_config* cfg /*host*/, int layer, int which,
                       size_t* offset_elems /*host*/, int64_t shape[2] /*host*/);

/* Creates a stage.  params_dev: device, param_bytes, caller-owned, read-only to the library
 * and must stay valid and unchanged while tasks are in flight.  arena_dev: device, at least
 * arena_bytes (STAGE_ENOMEM otherwise), 256-byte aligned, caller-owned, contents managed by
 * the library.  The device current at this call is the stage's device.  Creates HIP events;
 * allocates no device memory.  *out receives the handle. */
int stage_create(const stage_config* cfg /*host*/, const void* params_dev /*device*/,
                 void* arena_dev /*device*/, size_t arena_bytes, stage_t** out /*host*/);

/* Same validation, layout and dependency state machine as stage_create but no device: task
 * calls check their arguments and dependencies, update the state, and launch nothing.  For
 * schedulers, simulators and tests on machines without a GPU.  Makes no HIP call. */
int stage_create_dry(const stage_config* cfg /*host*/, stage_t** out /*host*/);

/* F task of microbatch mb (Section 3.1; Section 4.1: ready once its activation arrived).
 * x_dev: device [T, hidden] storage dtype, read during the task only (the library keeps its
 * own copy for B, so x may be reused once the stream has passed this task).
 * cu_seqlens_host: host, n_seg + 1 int32, cu[0] = 0, strictly increasing, T = cu[n_seg]
 * (1 <= T <= max_tokens, 1 <= n_seg <= max_segments); copied during the call.
 * y_dev: device [T, hidden] storage dtype, written.  stream: a hipStream_t (NULL = null stream).
 * STAGE_ENOTREADY if slot mb is still busy (F already issued in this iteration). */
int stage_F(stage_t* st, int mb, const void* x_dev /*device*/,
            const int32_t* cu_seqlens_host /*host*/, int n_seg, void* y_dev /*device*/,
            void* stream);

/* B task of microbatch mb: backward to the stage input (Section 4.1: ready after local F_j
 * and the gradient from the next stage; Section 7.1 for the B/W decomposition).
 * dy_dev: device [T, hidden], gradient of the loss w.r.t. y; read during the task only.
 * dx_dev: device [T, hidden], written.  Also produces the two norm-gain gradients of every
 * layer into gradient slot mb and keeps the GEMM output-gradients W needs.
 * STAGE_ENOTREADY unless F(mb) was issued and B(mb) was not. */
int stage_B(stage_t* st, int mb, const void* dy_dev /*device*/, void* dx_dev /*device*/,
            void* stream);

/* W task of microbatch mb: every GEMM-shaped weight gradient dW = input^T dOut of every
 * layer, written (not accumulated) to gradient slot mb in fp32 (Section 7.1: may be issued
 * at any time after B_j, including after other microbatches' F and B).  After it the
 * activation stash of mb is released (Appendix C.1 release rule, extended to W).
 * STAGE_ENOTREADY unless B(mb) was issued and W(mb) was not. */
int stage_W(stage_t* st, int mb, void* stream);

/* Ends the iteration: grad_out = ((s_0 + s_1) + s_2) + ... + s_{M-1} in fp32, in microbatch
 * INDEX order whatever order the tasks ran in, so the result is bit-identical under every
 * dispatch order.  grad_out_dev: device, grad_bytes, written.  STAGE_ENOTREADY unless W was
 * issued for all M microbatches.  Frees all M slots for the next iteration. */
int stage_grad_reduce(stage_t* st, void* grad_out_dev /*device*/, void* stream);

/* Device pointer of gradient slot mb (fp32, parameter element offsets); valid to read once
 * the stream of W(mb) has passed it and until the slot's next F.  For tests and tools. */
int stage_grad_slot(stage_t* st, int mb, void** slot_dev /*host*/);

/* Intermediate tensors the tasks keep per microbatch and layer (for tests and tools: lets every
 * kernel of a task be compared with the oracle's value of the same tensor). */
enum {
  STAGE_T_X = 0,      /* fp32 [T, hidden]   layer input (residual stream)           */
  STAGE_T_H1 = 1,     /* storage [T, hidden] first RMSNorm output                   */
  STAGE_T_QKV = 2,    /* [T, (n_q + 2 n_kv) d]; fp32 path: fp32; bf16 path: IEEE half */
  STAGE_T_O = 3,      /* storage [T, n_q d]  attention output                       */
  STAGE_T_X1 = 4,     /* fp32 [T, hidden]   x + o Wo                                */
  STAGE_T_H2 = 5,     /* storage [T, hidden] second RMSNorm output                  */
  STAGE_T_UP = 6,     /* storage [T, 2 ffn] (gate|up) or [T, ffn]                   */
  STAGE_T_M = 7,      /* storage [T, ffn]   activation output                       */
  STAGE_T_DY = 8,     /* storage [T, hidden] gradient w.r.t. the layer output       */
  STAGE_T_DUP = 9,    /* storage, shape of STAGE_T_UP                               */
  STAGE_T_DX1 = 10,   /* storage [T, hidden] gradient w.r.t. x1                     */
  STAGE_T_DQKV = 11,  /* storage, shape of STAGE_T_QKV                              */
  STAGE_T_LSE = 12,   /* fp32 [n_q, T]      log-sum-exp of the attention scores     */
  STAGE_T_H1_HALF = 13, /* bf16 path only: IEEE half [T, hidden], the first norm output as the QKV projection reads it */
  STAGE_T_COUNT = 14
};

/* Device pointer of intermediate tensor `which` (STAGE_T_*) of `layer` for microbatch mb; valid to
 * read after the task that writes it has completed and until the slot's next F. */
int stage_intermediate(stage_t* st, int mb, int layer, int which, void** ptr_dev /*host*/);

/* Destroys events and the handle.  The caller must have synchronised the streams used.  */
int stage_destroy(stage_t* st);

/* Last error text of this handle, or (st == NULL) of the calling thread's last failed
 * stage_query / stage_param_layout / stage_create*.  Never NULL. */
const char* stage_last_error(const stage_t* st);

#ifdef __cplusplus
}
#endif
#endif /* RRFP_STAGE_H */
