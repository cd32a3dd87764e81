// Host side of the stage library: configuration checks, memory plan, the per-microbatch
// dependency state machine, and the F / B / W / grad_reduce task bodies that enqueue the
// kernels.  Task model: paper Section 3.1 (precedence), Section 4.1 (readiness), Section 7.1
// (B/W decomposition), Appendix C.1 (retain until the backward side is done).
#include "../../include/rrfp_stage.h"
#include "kernels.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace rrfp;

namespace {

thread_local char g_tls_error[512] = "";

void set_tls_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_tls_error, sizeof(g_tls_error), fmt, ap);
  va_end(ap);
}

constexpr size_t ALIGN = 256;
size_t align_up(size_t v, size_t a = ALIGN) { return (v + a - 1) / a * a; }

// Byte offsets inside one microbatch region.  The residual stream (x, x1 and the gradients dy, dx1
// that flow along it) is kept in fp32 between layers; GEMM operands are in the storage type, so the
// two residual gradients exist twice: fp32 for the chain, storage type for the GEMMs and for W.
struct LayerStash {
  size_t x, r1, h1, qkv, lse, o, x1, r2, h2, up, m;   // written by F (x and x1 fp32)
  size_t dy, dup, dx1, dqkv;                          // written by B, read by W (storage type)
  size_t dy32, dx1_32;                                // written by B, fp32 residual-gradient chain
  size_t o32;                                         // written by F: attention output before rounding (bf16 path)
  size_t mu1, mu2;                                    // written by F: row means (LayerNorm variant)
  size_t qk_hat, qk_r;                                // written by F: normalised q, k heads and their 1/rms (QK-norm variant)
  size_t h1_16;                                       // written by F (bf16 path): first norm output as IEEE halves, operand of the QKV projection
  size_t o16;                                         // written by F (bf16 path): attention output as IEEE halves, operand of the output projection
};

struct Plan {
  stage_config c;
  int n_qkv, n_up;                  // widths of the fused projections
  size_t esz;                       // storage element size
  size_t p_off[64][STAGE_P_COUNT];  // element offsets (layers capped at 64)
  int64_t p_shape[STAGE_P_COUNT][2];
  size_t param_elems;
  std::vector<LayerStash> layer;
  size_t t_dm, t_dh, t_do, t_delta, t_dgp, t_dbp, t_qtiles, t_kvtiles;  // per-microbatch temporaries
  size_t t_ds;               // dS scratch of the MFMA attention backward (0 when that path cannot run)
  int ds_rows, ds_nqs;
  size_t t_dkvp;             // partial dK / dV planes of its head subsets (0 without grouped query heads)
  size_t t_dk32;                    // fp32 key-head gradients behind the head norm (QK-norm with biases only)
  size_t t_gscale, t_gpart;         // bf16 path: {s, 1/s} of the microbatch's gradient scale, and the partial maxima behind it
  int max_tiles;
  size_t mb_bytes;                  // one microbatch region
  size_t slots_off;                 // start of the M gradient slots
  size_t slot_floats;               // floats per slot (= param_elems)
  size_t w16_off[64];               // bf16 path: IEEE-half copy of every layer's Wqkv (byte offsets in the arena), refreshed once per iteration
  size_t w16o_off[64];              // the same for Wo
  size_t arena_bytes;
};

int check_config(const stage_config* c) {
  if (!c) { set_tls_error("config is NULL"); return STAGE_EINVAL; }
  if (c->n_layers < 1 || c->n_layers > 64) { set_tls_error("n_layers must be in [1, 64]"); return STAGE_EINVAL; }
  if (c->hidden < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1 || c->ffn < 1 ||
      c->max_tokens < 1 || c->n_microbatches < 1 || c->max_segments < 1) {
    set_tls_error("all sizes must be positive"); return STAGE_EINVAL;
  }
  if (c->n_microbatches > 4096) { set_tls_error("n_microbatches must be <= 4096"); return STAGE_EINVAL; }
  if (c->n_q_heads % c->n_kv_heads != 0) {
    set_tls_error("n_q_heads (%d) must be a multiple of n_kv_heads (%d)", c->n_q_heads, c->n_kv_heads);
    return STAGE_EINVAL;
  }
  if (c->dtype != STAGE_DTYPE_FP32 && c->dtype != STAGE_DTYPE_BF16) { set_tls_error("unknown dtype %d", c->dtype); return STAGE_EINVAL; }
  if (c->mlp_kind != STAGE_MLP_SWIGLU && c->mlp_kind != STAGE_MLP_GELU) { set_tls_error("unknown mlp_kind %d", c->mlp_kind); return STAGE_EINVAL; }
  if (c->causal != 0 && c->causal != 1) { set_tls_error("causal must be 0 or 1"); return STAGE_EINVAL; }
  if (c->norm_kind != 0 && c->norm_kind != 1) { set_tls_error("norm_kind must be 0 (RMSNorm) or 1 (LayerNorm)"); return STAGE_EINVAL; }
  if (c->bias != 0 && c->bias != 1) { set_tls_error("bias must be 0 or 1"); return STAGE_EINVAL; }
  if (c->qk_norm != 0 && c->qk_norm != 1) { set_tls_error("qk_norm must be 0 or 1"); return STAGE_EINVAL; }
  if (!(c->norm_eps >= 0.0f) || !(c->norm_eps < 1.0f)) { set_tls_error("norm_eps must be in [0, 1)"); return STAGE_EINVAL; }
  if (c->rope != 0 && c->rope != 1) { set_tls_error("rope must be 0 or 1"); return STAGE_EINVAL; }
  if (c->rope == 1 && !(c->rope_base > 1.0f)) { set_tls_error("rope_base must be > 1"); return STAGE_EINVAL; }
  if (c->head_dim % 16 != 0 || c->head_dim > 128) { set_tls_error("head_dim must be a multiple of 16, at most 128"); return STAGE_EINVAL; }
  if (c->dtype == STAGE_DTYPE_FP32 && c->ffn % 4 != 0) { set_tls_error("fp32: ffn must be a multiple of 4"); return STAGE_EINVAL; }
  if (c->dtype == STAGE_DTYPE_BF16) {
    if (c->head_dim != 64 && c->head_dim != 80 && c->head_dim != 128) { set_tls_error("bf16: head_dim must be 64, 80 or 128"); return STAGE_EINVAL; }
    if (c->hidden % 64 || c->ffn % 64 || (c->n_q_heads * c->head_dim) % 64 || (c->n_kv_heads * c->head_dim) % 64) {
      set_tls_error("bf16: hidden, ffn, n_q*head_dim and n_kv*head_dim must be multiples of 64"); return STAGE_EINVAL;
    }
  }
  if ((int64_t)c->max_tokens * std::max(c->hidden, 2 * c->ffn) >= ((int64_t)1 << 40)) { set_tls_error("max_tokens too large"); return STAGE_EINVAL; }
  return STAGE_OK;
}

int make_plan(const stage_config* c, Plan* p) {
  int rc = check_config(c);
  if (rc) return rc;
  p->c = *c;
  const size_t H = c->hidden, d = c->head_dim, F = c->ffn, T = c->max_tokens;
  const size_t nq = c->n_q_heads, nkv = c->n_kv_heads;
  p->n_qkv = (int)((nq + 2 * nkv) * d);
  p->n_up = (int)(c->mlp_kind == STAGE_MLP_SWIGLU ? 2 * F : F);
  p->esz = dtype_size(c->dtype);
  const int64_t ln = c->norm_kind == 1 ? 1 : 0, bs = c->bias ? 1 : 0;   // zero-sized vectors when a variant is off
  const int64_t shapes[STAGE_P_COUNT][2] = {
      {(int64_t)H, 1}, {(int64_t)H, p->n_qkv}, {(int64_t)(nq * d), (int64_t)H},
      {(int64_t)H, 1}, {(int64_t)H, p->n_up}, {(int64_t)F, (int64_t)H},
      {ln * (int64_t)H, 1}, {bs * (int64_t)p->n_qkv, 1}, {bs * (int64_t)H, 1},
      {ln * (int64_t)H, 1}, {bs * (int64_t)p->n_up, 1}, {bs * (int64_t)H, 1},
      {(c->qk_norm ? 1 : 0) * (int64_t)d, 1}, {(c->qk_norm ? 1 : 0) * (int64_t)d, 1}};
  memcpy(p->p_shape, shapes, sizeof(shapes));
  size_t off = 0;
  for (int l = 0; l < c->n_layers; ++l)
    for (int w = 0; w < STAGE_P_COUNT; ++w) {
      p->p_off[l][w] = off;
      off += align_up((size_t)(shapes[w][0] * shapes[w][1]), 128);  // 128 elements: 256 B bf16, 512 B fp32
    }
  p->param_elems = off;
  p->slot_floats = off;

  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += align_up(bytes); return r; };
  const size_t e = p->esz;
  p->layer.resize(c->n_layers);
  for (auto& s : p->layer) {
    s.x = take(T * H * 4);   s.r1 = take(T * 4);        s.h1 = take(T * H * e);
    s.qkv = take(T * p->n_qkv * e);  s.lse = take(nq * T * 4);  s.o = take(T * nq * d * e);
    s.x1 = take(T * H * 4);  s.r2 = take(T * 4);        s.h2 = take(T * H * e);
    s.up = take(T * p->n_up * e);    s.m = take(T * F * e);
    s.dy = take(T * H * e);  s.dup = take(T * p->n_up * e);
    s.dx1 = take(T * H * e); s.dqkv = take(T * p->n_qkv * e);
    s.dy32 = take(T * H * 4); s.dx1_32 = take(T * H * 4);
    s.o32 = c->dtype == STAGE_DTYPE_BF16 ? take(T * nq * d * 4) : 0;
    s.mu1 = c->norm_kind == 1 ? take(T * 4) : 0;
    s.mu2 = c->norm_kind == 1 ? take(T * 4) : 0;
    s.qk_hat = c->qk_norm ? take(T * (nq + nkv) * d * e) : 0;
    s.qk_r = c->qk_norm ? take(T * (nq + nkv) * 4) : 0;
    s.h1_16 = c->dtype == STAGE_DTYPE_BF16 ? take(T * H * 2) : 0;
    s.o16 = c->dtype == STAGE_DTYPE_BF16 ? take(T * nq * d * 2) : 0;
  }
  p->t_dm = take(T * F * 4);     // fp32: GEMM outputs that only an elementwise kernel consumes are not rounded
  p->t_dh = take(T * H * 4);
  p->t_do = take(T * nq * d * e);
  p->t_delta = take(nq * T * 4);
  size_t dgp = (size_t)std::max(norm_bwd_partials((int)T, (int)H, c->dtype), colsum_chunks((int)T)) * H * 4;
  if (c->qk_norm) dgp = std::max(dgp, (size_t)headnorm_partials((int)T, (int)nq) * d * 4);
  p->t_dgp = take(dgp);
  // second partial array: LayerNorm bias gradient, and the projection-bias gradients (widest tensor)
  const size_t wide = std::max((size_t)H, (size_t)std::max(p->n_qkv, p->n_up));
  size_t dbp = (c->norm_kind == 1 || c->bias) ? (size_t)colsum_chunks((int)T) * wide * 4 : 0;
  if (c->qk_norm) dbp = std::max(dbp, (size_t)headnorm_partials((int)T, (int)nkv) * d * 4);
  p->t_dbp = dbp ? take(dbp) : 0;
  p->t_dk32 = (c->qk_norm && c->bias) ? take(T * nkv * d * 4) : 0;
  p->t_gscale = take(256);
  p->t_gpart = take((size_t)grad_scale_partials(T * H) * 4);
  const int tile = std::min(ATTN_TILE_Q, ATTN_TILE_KV);
  p->max_tiles = (int)((T + tile - 1) / tile) + c->max_segments;
  p->t_qtiles = take((size_t)p->max_tiles * sizeof(AttnTile));
  p->t_kvtiles = take((size_t)p->max_tiles * sizeof(AttnTile));
  // The MFMA attention backward forms dS once, in the dK/dV kernel, and hands it to the dQ kernel through this
  // scratch (per microbatch: B tasks of different microbatches may run side by side on different streams).
  {
    AttnArgs probe{};
    probe.dtype = c->dtype; probe.d = c->head_dim; probe.n_q_tiles = 1;
    p->ds_rows = attn_ds_rows((int)T, c->max_segments);
    p->ds_nqs = attn_ds_nqs((int)T);
    p->t_ds = attn_mfma_supports(probe) ? take(attn_ds_bytes((int)T, c->max_segments, (int)nq)) : 0;
    const size_t part = attn_dkv_part_bytes((int)T, (int)nq, (int)nkv, (int)d);
    p->t_dkvp = (attn_mfma_supports(probe) && part) ? take(part) : 0;
  }
  p->mb_bytes = o;
  p->slots_off = p->mb_bytes * (size_t)c->n_microbatches;
  p->arena_bytes = p->slots_off + align_up(p->slot_floats * 4) * (size_t)c->n_microbatches;
  for (int l = 0; l < c->n_layers; ++l) {
    p->w16_off[l] = p->arena_bytes;
    if (c->dtype == STAGE_DTYPE_BF16) p->arena_bytes += align_up(H * (size_t)p->n_qkv * 2);
    p->w16o_off[l] = p->arena_bytes;
    if (c->dtype == STAGE_DTYPE_BF16) p->arena_bytes += align_up(nq * d * H * 2);
  }
  return STAGE_OK;
}

// MB_POISONED: a HIP call failed in the middle of a task of this slot, so part of the task is enqueued and the
// slot's memory is in an unknown state; every later task on the slot is refused until the stage is destroyed.
enum MbState { MB_FREE = 0, MB_F = 1, MB_B = 2, MB_W = 3, MB_POISONED = 4 };

struct MbSlot {
  int state = MB_FREE;
  int T = 0, n_seg = 0, n_q_tiles = 0, n_kv_tiles = 0;
  hipEvent_t ev_F = nullptr, ev_B = nullptr, ev_W = nullptr, ev_copy = nullptr;
  bool copy_pending = false;
  AttnTile* staging = nullptr;   // pinned host, 2 * max_tiles entries
};

}  // namespace

struct stage_s {
  Plan plan;
  bool dry = false;
  int device = 0;
  const char* params = nullptr;
  char* arena = nullptr;
  std::vector<MbSlot> mb;
  hipEvent_t ev_reduce = nullptr;
  bool reduce_recorded = false;
  hipEvent_t ev_w16 = nullptr;      // the half copies of Wqkv of this iteration are complete
  bool w16_valid = false;           // false from stage_create / stage_grad_reduce until the next stage_F
  char err[512] = "";
};

namespace {

void set_error(stage_t* st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(st->err, sizeof(st->err), fmt, ap);
  va_end(ap);
}

// A HIP failure inside a task body: the slot named by the enclosing scope's `poison` (an int*, or nullptr
// outside task bodies) is marked poisoned, because kernels of the task may already be enqueued.
#define HIP_TRY(st, expr)                                                              \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess) {                                                            \
      set_error(st, "%s failed: %s%s", #expr, hipGetErrorString(e_),                   \
                poison ? "; the microbatch slot is poisoned: its tasks are refused until stage_destroy" : ""); \
      if (poison) *poison = MB_POISONED;                                               \
      return STAGE_EHIP;                                                               \
    }                                                                                  \
  } while (0)

int refuse_poisoned(stage_t* st, int mb, const char* task);

// Tiles of `rows` rows carved inside each segment, heaviest first (more keys first under a
// causal mask) so that long tiles start early.  A pure function of cu_seqlens.
int build_tiles(const int32_t* cu, int n_seg, int rows, bool causal, bool kv_side, AttnTile* out) {
  int n = 0, kb0 = 0;
  for (int s = 0; s < n_seg; ++s) {
    for (int r = cu[s]; r < cu[s + 1]; r += rows)
      out[n++] = AttnTile{r, std::min(r + rows, cu[s + 1]), cu[s], cu[s + 1], kb0};
    kb0 += (cu[s + 1] - cu[s] + 31) / 32;
  }
  auto work = [&](const AttnTile& t) {
    if (!causal) return t.s1 - t.s0;
    return kv_side ? t.s1 - t.r0 : t.r1 - t.s0;
  };
  std::stable_sort(out, out + n, [&](const AttnTile& a, const AttnTile& b) { return work(a) > work(b); });
  return n;
}

int refuse_poisoned(stage_t* st, int mb, const char* task) {
  set_error(st, "%s(%d): the slot is poisoned by an earlier HIP failure in one of its tasks; destroy the stage", task, mb);
  return STAGE_EHIP;
}

char* mb_base(stage_t* st, int mb) { return st->arena + st->plan.mb_bytes * (size_t)mb; }
float* slot_base(stage_t* st, int mb) {
  return (float*)(st->arena + st->plan.slots_off + align_up(st->plan.slot_floats * 4) * (size_t)mb);
}
const char* param_ptr(stage_t* st, int l, int w) { return st->params + st->plan.p_off[l][w] * st->plan.esz; }

int check_handle_mb(stage_t* st, int mb) {
  if (!st) { set_tls_error("stage handle is NULL"); return STAGE_EINVAL; }
  if (mb < 0 || mb >= st->plan.c.n_microbatches) {
    set_error(st, "microbatch index %d out of range [0, %d)", mb, st->plan.c.n_microbatches);
    return STAGE_EINVAL;
  }
  return STAGE_OK;
}

int create_common(const stage_config* cfg, stage_t** out, stage_t** made) {
  if (!out) { set_tls_error("out is NULL"); return STAGE_EINVAL; }
  *out = nullptr;
  Plan plan;
  int rc = make_plan(cfg, &plan);
  if (rc) return rc;
  stage_t* st = new (std::nothrow) stage_s();
  if (!st) { set_tls_error("host allocation failed"); return STAGE_ENOMEM; }
  st->plan = plan;
  st->mb.resize(cfg->n_microbatches);
  *made = st;
  return STAGE_OK;
}

}  // namespace

extern "C" {

int stage_query(const stage_config* cfg, size_t* param_bytes, size_t* grad_bytes, size_t* arena_bytes) {
  Plan p;
  int rc = make_plan(cfg, &p);
  if (rc) return rc;
  if (param_bytes) *param_bytes = p.param_elems * p.esz;
  if (grad_bytes) *grad_bytes = p.param_elems * 4;
  if (arena_bytes) *arena_bytes = p.arena_bytes;
  return STAGE_OK;
}

int stage_param_layout(const stage_config* cfg, int layer, int which, size_t* offset_elems, int64_t shape[2]) {
  Plan p;
  int rc = make_plan(cfg, &p);
  if (rc) return rc;
  if (layer < 0 || layer >= cfg->n_layers || which < 0 || which >= STAGE_P_COUNT) {
    set_tls_error("layer %d / tensor %d out of range", layer, which);
    return STAGE_EINVAL;
  }
  if (offset_elems) *offset_elems = p.p_off[layer][which];
  if (shape) { shape[0] = p.p_shape[which][0]; shape[1] = p.p_shape[which][1]; }
  return STAGE_OK;
}

int stage_create_dry(const stage_config* cfg, stage_t** out) {
  stage_t* st = nullptr;
  int rc = create_common(cfg, out, &st);
  if (rc) return rc;
  st->dry = true;
  *out = st;
  return STAGE_OK;
}

int stage_create(const stage_config* cfg, const void* params_dev, void* arena_dev, size_t arena_bytes,
                 stage_t** out) {
  stage_t* st = nullptr;
  int rc = create_common(cfg, out, &st);
  if (rc) return rc;
  auto fail = [&](int code, const char* msg) { set_tls_error("%s", msg); delete st; return code; };
  if (!params_dev || !arena_dev) return fail(STAGE_EINVAL, "params_dev and arena_dev must not be NULL");
  if (((uintptr_t)arena_dev % ALIGN) || ((uintptr_t)params_dev % ALIGN)) return fail(STAGE_EINVAL, "params_dev and arena_dev must be 256-byte aligned");
  if (arena_bytes < st->plan.arena_bytes) return fail(STAGE_ENOMEM, "arena smaller than stage_query reports");
  st->params = (const char*)params_dev;
  st->arena = (char*)arena_dev;
  hipError_t e = hipGetDevice(&st->device);
  for (auto& m : st->mb) {
    if (e == hipSuccess) e = hipEventCreateWithFlags(&m.ev_F, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&m.ev_B, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&m.ev_W, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&m.ev_copy, hipEventDisableTiming);
    if (e == hipSuccess) e = hipHostMalloc((void**)&m.staging, 2 * (size_t)st->plan.max_tiles * sizeof(AttnTile), hipHostMallocDefault);
  }
  if (e == hipSuccess) e = hipEventCreateWithFlags(&st->ev_reduce, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&st->ev_w16, hipEventDisableTiming);
  if (e != hipSuccess) {
    set_tls_error("HIP set-up failed: %s", hipGetErrorString(e));
    stage_destroy(st);
    return STAGE_EHIP;
  }
  *out = st;
  return STAGE_OK;
}

int stage_destroy(stage_t* st) {
  if (!st) return STAGE_OK;
  if (!st->dry) {
    for (auto& m : st->mb) {
      if (m.ev_F) (void)hipEventDestroy(m.ev_F);
      if (m.ev_B) (void)hipEventDestroy(m.ev_B);
      if (m.ev_W) (void)hipEventDestroy(m.ev_W);
      if (m.ev_copy) (void)hipEventDestroy(m.ev_copy);
      if (m.staging) (void)hipHostFree(m.staging);
    }
    if (st->ev_reduce) (void)hipEventDestroy(st->ev_reduce);
    if (st->ev_w16) (void)hipEventDestroy(st->ev_w16);
  }
  delete st;
  return STAGE_OK;
}

const char* stage_last_error(const stage_t* st) { return st ? st->err : g_tls_error; }

int stage_grad_slot(stage_t* st, int mb, void** slot_dev) {
  int rc = check_handle_mb(st, mb);
  if (rc) return rc;
  if (!slot_dev) { set_error(st, "slot_dev is NULL"); return STAGE_EINVAL; }
  *slot_dev = st->dry ? nullptr : (void*)slot_base(st, mb);
  return STAGE_OK;
}

int stage_intermediate(stage_t* st, int mb, int layer, int which, void** ptr_dev) {
  int rc = check_handle_mb(st, mb);
  if (rc) return rc;
  if (!ptr_dev || layer < 0 || layer >= st->plan.c.n_layers || which < 0 || which >= STAGE_T_COUNT) {
    set_error(st, "stage_intermediate: bad layer %d / tensor %d / NULL output", layer, which);
    return STAGE_EINVAL;
  }
  const LayerStash& L = st->plan.layer[layer];
  const size_t off[STAGE_T_COUNT] = {L.x, L.h1, L.qkv, L.o, L.x1, L.h2, L.up, L.m, L.dy, L.dup, L.dx1, L.dqkv, L.lse, L.h1_16};
  if (which == STAGE_T_H1_HALF && st->plan.c.dtype != STAGE_DTYPE_BF16) {
    set_error(st, "stage_intermediate: the half copy of h1 exists on the bf16 path only");
    return STAGE_EINVAL;
  }
  *ptr_dev = st->dry ? nullptr : (void*)(mb_base(st, mb) + off[which]);
  return STAGE_OK;
}

int stage_F(stage_t* st, int mb, const void* x_dev, const int32_t* cu, int n_seg, void* y_dev, void* stream) {
  int rc = check_handle_mb(st, mb);
  if (rc) return rc;
  const Plan& P = st->plan;
  const stage_config& c = P.c;
  if (!cu) { set_error(st, "cu_seqlens_host is NULL"); return STAGE_EINVAL; }
  if (n_seg < 1 || n_seg > c.max_segments) { set_error(st, "n_seg %d outside [1, max_segments=%d]", n_seg, c.max_segments); return STAGE_EINVAL; }
  if (cu[0] != 0) { set_error(st, "cu_seqlens[0] must be 0"); return STAGE_EINVAL; }
  for (int s = 0; s < n_seg; ++s)
    if (cu[s + 1] <= cu[s]) { set_error(st, "cu_seqlens must be strictly increasing (entry %d)", s + 1); return STAGE_EINVAL; }
  const int T = cu[n_seg];
  if (T > c.max_tokens) { set_error(st, "T = %d exceeds max_tokens = %d", T, c.max_tokens); return STAGE_EINVAL; }
  if (!st->dry && (!x_dev || !y_dev)) { set_error(st, "x_dev and y_dev must not be NULL"); return STAGE_EINVAL; }
  MbSlot& m = st->mb[mb];
  if (m.state == MB_POISONED) return refuse_poisoned(st, mb, "F");
  if (m.state != MB_FREE) { set_error(st, "F(%d): slot is busy until stage_grad_reduce", mb); return STAGE_ENOTREADY; }

  m.T = T;
  m.n_seg = n_seg;
  if (st->dry) {
    m.state = MB_F;
    return STAGE_OK;
  }
  int* poison = &m.state;
  hipStream_t s = (hipStream_t)stream;
  // The pinned tile lists of this slot may still be the source of the previous iteration's copy: the one
  // place where a task call can wait on the host (documented in the header).  The copy was enqueued before
  // the previous iteration's kernels of this slot, so in steady state it has long completed.
  if (m.copy_pending) { HIP_TRY(st, hipEventSynchronize(m.ev_copy)); m.copy_pending = false; }
  AttnTile* qt = m.staging;
  AttnTile* kt = m.staging + P.max_tiles;
  m.n_q_tiles = build_tiles(cu, n_seg, ATTN_TILE_Q, c.causal != 0, false, qt);
  m.n_kv_tiles = build_tiles(cu, n_seg, ATTN_TILE_KV, c.causal != 0, true, kt);

  char* base = mb_base(st, mb);
  if (st->reduce_recorded) HIP_TRY(st, hipStreamWaitEvent(s, st->ev_reduce, 0));
  if (c.dtype == STAGE_DTYPE_BF16) {
    // The QKV and output projections run on IEEE-half operands.  The first F of an iteration converts every
    // layer's Wqkv and Wo (the caller may have changed the parameters since the last stage_grad_reduce) on its own
    // stream, behind the previous reduce and so behind every earlier reader of the copies; every F waits for
    // that conversion.
    if (!st->w16_valid) {
      for (int l = 0; l < c.n_layers; ++l) {
        HIP_TRY(st, launch_bf16_to_f16(param_ptr(st, l, STAGE_P_WQKV), st->arena + P.w16_off[l], (size_t)c.hidden * P.n_qkv, s));
        HIP_TRY(st, launch_bf16_to_f16(param_ptr(st, l, STAGE_P_WO), st->arena + P.w16o_off[l],
                                       (size_t)c.n_q_heads * c.head_dim * c.hidden, s));
      }
      HIP_TRY(st, hipEventRecord(st->ev_w16, s));
      st->w16_valid = true;
    } else {
      HIP_TRY(st, hipStreamWaitEvent(s, st->ev_w16, 0));
    }
  }
  HIP_TRY(st, hipMemcpyAsync(base + P.t_qtiles, qt, (size_t)m.n_q_tiles * sizeof(AttnTile), hipMemcpyHostToDevice, s));
  HIP_TRY(st, hipMemcpyAsync(base + P.t_kvtiles, kt, (size_t)m.n_kv_tiles * sizeof(AttnTile), hipMemcpyHostToDevice, s));
  HIP_TRY(st, hipEventRecord(m.ev_copy, s));
  m.copy_pending = true;

  const int H = c.hidden, F = c.ffn, dt = c.dtype, nqd = c.n_q_heads * c.head_dim;
  const bool half_path = dt == BF16;            // h1 -> QKV projection -> attention run on IEEE halves
  const int qdt = half_path ? (int)F16 : dt;    // element type of the q|k|v stash
  HIP_TRY(st, launch_widen(x_dev, (float*)(base + P.layer[0].x), (size_t)T * H, dt, s));
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerStash& L = P.layer[l];
    const bool last = l == c.n_layers - 1;
    void* y_out = last ? y_dev : (void*)(base + P.layer[l + 1].x);
    if (c.norm_kind == 1)
      HIP_TRY(st, launch_layernorm_fwd((const float*)(base + L.x), param_ptr(st, l, STAGE_P_G1), param_ptr(st, l, STAGE_P_B1), base + L.h1,
                                       (float*)(base + L.r1), (float*)(base + L.mu1), T, H, c.norm_eps, dt, s, half_path ? base + L.h1_16 : nullptr));
    else
      HIP_TRY(st, launch_rmsnorm_fwd((const float*)(base + L.x), param_ptr(st, l, STAGE_P_G1), base + L.h1, (float*)(base + L.r1), T, H, c.norm_eps, dt, s,
                                     half_path ? base + L.h1_16 : nullptr));
    GemmArgs g{};
    g.in_dtype = dt; g.out_dtype = dt; g.transA = false; g.transB = false; g.M = T;
    g.A = base + L.h1; g.lda = H; g.B = param_ptr(st, l, STAGE_P_WQKV); g.ldb = P.n_qkv;
    if (half_path) { g.in_dtype = F16; g.out_dtype = F16; g.A = base + L.h1_16; g.B = st->arena + P.w16_off[l]; }
    g.C = base + L.qkv; g.ldc = P.n_qkv; g.R = nullptr; g.N = P.n_qkv; g.K = H;
    g.bias = c.bias ? param_ptr(st, l, STAGE_P_BQKV) : nullptr;
    HIP_TRY(st, launch_gemm(g, s));
    g.in_dtype = dt; g.out_dtype = dt;
    if (c.qk_norm)   // normalise every q and k head in place (before the rotation)
      HIP_TRY(st, launch_headnorm_fwd(base + L.qkv, P.n_qkv, c.n_q_heads, c.n_q_heads + c.n_kv_heads, c.head_dim,
                                      param_ptr(st, l, STAGE_P_GQ), param_ptr(st, l, STAGE_P_GK), base + L.qk_hat,
                                      (float*)(base + L.qk_r), T, c.norm_eps, qdt, s));
    if (c.rope)   // rotate q and k in place: the stash then holds what the attention (and its backward) reads
      HIP_TRY(st, launch_rope(base + L.qkv, (const AttnTile*)(base + P.t_qtiles), m.n_q_tiles, c.n_q_heads + c.n_kv_heads,
                              c.head_dim, P.n_qkv, c.rope_base, 1.0f, qdt, s));
    AttnArgs a{};
    a.qkv = base + L.qkv; a.o = base + L.o; a.lse = (float*)(base + L.lse);
    a.o32 = dt == BF16 ? (float*)(base + L.o32) : nullptr;
    a.o16 = half_path ? base + L.o16 : nullptr;
    a.q_tiles = (const AttnTile*)(base + P.t_qtiles); a.n_q_tiles = m.n_q_tiles;
    a.kv_tiles = (const AttnTile*)(base + P.t_kvtiles); a.n_kv_tiles = m.n_kv_tiles;
    a.T = T; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads; a.d = c.head_dim; a.causal = c.causal; a.dtype = dt;
    HIP_TRY(st, launch_attn_fwd(a, s));
    g.A = base + L.o; g.lda = nqd; g.B = param_ptr(st, l, STAGE_P_WO); g.ldb = H;
    if (half_path) { g.in_dtype = F16; g.A = base + L.o16; g.B = st->arena + P.w16o_off[l]; }
    g.C = base + L.x1; g.ldc = H; g.R = (const float*)(base + L.x); g.ldr = H; g.N = H; g.K = nqd;
    g.out_dtype = F32;                       // x1 stays in the fp32 residual stream
    g.bias = c.bias ? param_ptr(st, l, STAGE_P_BO) : nullptr;
    HIP_TRY(st, launch_gemm(g, s));
    g.out_dtype = dt; g.in_dtype = dt;
    if (c.norm_kind == 1)
      HIP_TRY(st, launch_layernorm_fwd((const float*)(base + L.x1), param_ptr(st, l, STAGE_P_G2), param_ptr(st, l, STAGE_P_B2), base + L.h2,
                                       (float*)(base + L.r2), (float*)(base + L.mu2), T, H, c.norm_eps, dt, s));
    else
      HIP_TRY(st, launch_rmsnorm_fwd((const float*)(base + L.x1), param_ptr(st, l, STAGE_P_G2), base + L.h2, (float*)(base + L.r2), T, H, c.norm_eps, dt, s));
    g.A = base + L.h2; g.lda = H; g.B = param_ptr(st, l, STAGE_P_WUP); g.ldb = P.n_up;
    g.C = base + L.up; g.ldc = P.n_up; g.R = nullptr; g.N = P.n_up; g.K = H;
    g.bias = c.bias ? param_ptr(st, l, STAGE_P_BUP) : nullptr;
    // the activation runs in the GEMM epilogue on the fp32 accumulators when the shape allows it
    g.act = c.mlp_kind == STAGE_MLP_SWIGLU ? ACT_SWIGLU_FWD : ACT_GELU_FWD; g.E = base + L.m; g.lde = F;
    if (gemm_act_supported(g)) {
      HIP_TRY(st, launch_gemm(g, s));
      g.act = ACT_NONE; g.E = nullptr;
    } else {
      g.act = ACT_NONE; g.E = nullptr;
      HIP_TRY(st, launch_gemm(g, s));
      if (c.mlp_kind == STAGE_MLP_SWIGLU) HIP_TRY(st, launch_swiglu_fwd(base + L.up, base + L.m, T, F, dt, s));
      else HIP_TRY(st, launch_gelu_fwd(base + L.up, base + L.m, T, F, dt, s));
    }
    g.A = base + L.m; g.lda = F; g.B = param_ptr(st, l, STAGE_P_WD); g.ldb = H;
    g.C = y_out; g.ldc = H; g.R = (const float*)(base + L.x1); g.ldr = H; g.N = H; g.K = F;
    g.out_dtype = last ? dt : (int)F32;      // the stage output is rounded once; between layers fp32
    g.bias = c.bias ? param_ptr(st, l, STAGE_P_BD) : nullptr;
    HIP_TRY(st, launch_gemm(g, s));
    g.out_dtype = dt; g.bias = nullptr;
  }
  HIP_TRY(st, hipEventRecord(m.ev_F, s));
  m.state = MB_F;
  return STAGE_OK;
}

int stage_B(stage_t* st, int mb, const void* dy_dev, void* dx_dev, void* stream) {
  int rc = check_handle_mb(st, mb);
  if (rc) return rc;
  const Plan& P = st->plan;
  const stage_config& c = P.c;
  if (!st->dry && (!dy_dev || !dx_dev)) { set_error(st, "dy_dev and dx_dev must not be NULL"); return STAGE_EINVAL; }
  MbSlot& m = st->mb[mb];
  if (m.state == MB_POISONED) return refuse_poisoned(st, mb, "B");
  if (m.state != MB_F) {
    set_error(st, m.state == MB_FREE ? "B(%d) before F(%d)" : "B(%d) already issued", mb, mb);
    return STAGE_ENOTREADY;
  }
  if (st->dry) { m.state = MB_B; return STAGE_OK; }
  int* poison = &m.state;
  hipStream_t s = (hipStream_t)stream;
  HIP_TRY(st, hipStreamWaitEvent(s, m.ev_F, 0));
  char* base = mb_base(st, mb);
  float* slot = slot_base(st, mb);
  const int T = m.T, H = c.hidden, F = c.ffn, dt = c.dtype, nqd = c.n_q_heads * c.head_dim;
  const int n_part = norm_bwd_partials(T, H, dt);
  // one pass over dy: the fp32 head of the residual-gradient chain and the library's own copy for the GEMMs and W
  HIP_TRY(st, launch_widen(dy_dev, (float*)(base + P.layer[c.n_layers - 1].dy32), (size_t)T * H, dt, s,
                           base + P.layer[c.n_layers - 1].dy));
  // bf16 path: the attention backward keeps its copy of dO as IEEE halves; s = 2^-floor(log2 max|dy|) brings it
  // into their range whatever the scale of the loss (dO is linear in dy), and dq, dk, dv are multiplied by 1/s
  const float* gscale = nullptr;
  if (dt == BF16) {
    HIP_TRY(st, launch_grad_scale(dy_dev, (size_t)T * H, dt, (float*)(base + P.t_gpart), (float*)(base + P.t_gscale), s));
    gscale = (const float*)(base + P.t_gscale);
  }
  const int n_chunk = colsum_chunks(T);
  // bias gradient = column sum of a projection's output-gradient (storage type), in a fixed order
  auto bias_grad = [&](const void* src, int n, size_t slot_off) -> int {
    HIP_TRY(st, launch_colsum_rows(src, n, (float*)(base + P.t_dbp), T, n, dt, s));
    HIP_TRY(st, launch_colsum((const float*)(base + P.t_dbp), n_chunk, n, slot + slot_off, s));
    return STAGE_OK;
  };
  // backward of one norm: dx (+ add_in) and the vector gradients into the slot
  auto norm_bwd = [&](int l, bool first, const float* dh, const float* x, const float* r, const float* mu, const float* add_in,
                      float* out32, void* out_t) -> int {
    const int pg = first ? STAGE_P_G1 : STAGE_P_G2, pb = first ? STAGE_P_B1 : STAGE_P_B2;
    if (c.norm_kind == 1) {
      HIP_TRY(st, launch_layernorm_bwd(dh, x, r, mu, param_ptr(st, l, pg), add_in, out32, out_t, (float*)(base + P.t_dgp),
                                       (float*)(base + P.t_dbp), T, H, dt, s));
      HIP_TRY(st, launch_colsum((const float*)(base + P.t_dgp), n_chunk, H, slot + P.p_off[l][pg], s));
      HIP_TRY(st, launch_colsum((const float*)(base + P.t_dbp), n_chunk, H, slot + P.p_off[l][pb], s));
    } else {
      HIP_TRY(st, launch_rmsnorm_bwd(dh, x, r, param_ptr(st, l, pg), add_in, out32, out_t, (float*)(base + P.t_dgp), T, H, dt, s));
      HIP_TRY(st, launch_colsum((const float*)(base + P.t_dgp), n_part, H, slot + P.p_off[l][pg], s));
    }
    return STAGE_OK;
  };
  for (int l = c.n_layers - 1; l >= 0; --l) {
    const LayerStash& L = P.layer[l];
    if (c.bias) { rc = bias_grad(base + L.dy, H, P.p_off[l][STAGE_P_BD]); if (rc) return rc; }
    void* dx_out = (l == 0) ? dx_dev : (void*)(base + P.layer[l - 1].dy);
    float* dx_out32 = (l == 0) ? nullptr : (float*)(base + P.layer[l - 1].dy32);
    GemmArgs g{};
    g.in_dtype = dt; g.out_dtype = dt; g.transA = false; g.transB = true; g.M = T; g.R = nullptr;
    // dm = dy Wd^T
    g.A = base + L.dy; g.lda = H; g.B = param_ptr(st, l, STAGE_P_WD); g.ldb = H;
    // dm = dy Wd^T feeds only the activation backward: fused into the epilogue when the shape allows it
    g.C = base + L.dup; g.ldc = P.n_up; g.N = F; g.K = H; g.out_dtype = dt;
    g.act = c.mlp_kind == STAGE_MLP_SWIGLU ? ACT_SWIGLU_BWD : ACT_GELU_BWD; g.E = base + L.up; g.lde = P.n_up;
    if (gemm_act_supported(g)) {
      HIP_TRY(st, launch_gemm(g, s));
      g.act = ACT_NONE; g.E = nullptr;
    } else {
      g.act = ACT_NONE; g.E = nullptr;
      g.C = base + P.t_dm; g.ldc = F; g.out_dtype = F32;
      HIP_TRY(st, launch_gemm(g, s));
      if (c.mlp_kind == STAGE_MLP_SWIGLU) HIP_TRY(st, launch_swiglu_bwd((const float*)(base + P.t_dm), base + L.up, base + L.dup, T, F, dt, s));
      else HIP_TRY(st, launch_gelu_bwd((const float*)(base + P.t_dm), base + L.up, base + L.dup, T, F, dt, s));
    }
    // dh2 = [dgate|dup] Wup^T
    g.A = base + L.dup; g.lda = P.n_up; g.B = param_ptr(st, l, STAGE_P_WUP); g.ldb = P.n_up;
    g.C = base + P.t_dh; g.ldc = H; g.N = H; g.K = P.n_up; g.out_dtype = F32;
    HIP_TRY(st, launch_gemm(g, s));
    if (c.bias) { rc = bias_grad(base + L.dup, P.n_up, P.p_off[l][STAGE_P_BUP]); if (rc) return rc; }
    rc = norm_bwd(l, false, (const float*)(base + P.t_dh), (const float*)(base + L.x1), (const float*)(base + L.r2),
                  (const float*)(base + L.mu2), (const float*)(base + L.dy32), (float*)(base + L.dx1_32), base + L.dx1);
    if (rc) return rc;
    if (c.bias) { rc = bias_grad(base + L.dx1, H, P.p_off[l][STAGE_P_BO]); if (rc) return rc; }
    // do = dx1 Wo^T
    g.A = base + L.dx1; g.lda = H; g.B = param_ptr(st, l, STAGE_P_WO); g.ldb = H;
    g.C = base + P.t_do; g.ldc = nqd; g.N = nqd; g.K = H;
    g.out_dtype = dt == BF16 ? (int)F16 : dt;      // bf16 path: the attention backward reads s * dO as IEEE halves
    g.out_scale = gscale;
    HIP_TRY(st, launch_gemm(g, s));
    g.out_dtype = dt; g.out_scale = nullptr;
    AttnArgs a{};
    a.qkv = base + L.qkv; a.o = base + L.o; a.lse = (float*)(base + L.lse);
    a.o32 = dt == BF16 ? (float*)(base + L.o32) : nullptr;
    a.q_tiles = (const AttnTile*)(base + P.t_qtiles); a.n_q_tiles = m.n_q_tiles;
    a.kv_tiles = (const AttnTile*)(base + P.t_kvtiles); a.n_kv_tiles = m.n_kv_tiles;
    a.T = T; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads; a.d = c.head_dim; a.causal = c.causal; a.dtype = dt;
    a.d_o = base + P.t_do; a.dqkv = base + L.dqkv; a.delta = (float*)(base + P.t_delta);
    a.grad_scale = gscale;
    a.ds = P.t_ds ? base + P.t_ds : nullptr; a.ds_rows = P.ds_rows; a.ds_nqs = P.ds_nqs;
    a.dkv_part = P.t_dkvp ? (float*)(base + P.t_dkvp) : nullptr;
    HIP_TRY(st, launch_attn_bwd(a, s));
    if (c.rope)   // gradients w.r.t. the rotated q, k -> w.r.t. the projection outputs (inverse rotation)
      HIP_TRY(st, launch_rope(base + L.dqkv, (const AttnTile*)(base + P.t_qtiles), m.n_q_tiles, c.n_q_heads + c.n_kv_heads,
                              c.head_dim, P.n_qkv, c.rope_base, -1.0f, dt, s));
    if (c.qk_norm) {   // gradients w.r.t. the normalised heads -> w.r.t. the projection outputs, gain gradients to the slot
      HIP_TRY(st, launch_headnorm_bwd(base + L.dqkv, P.n_qkv, c.n_q_heads, c.n_q_heads + c.n_kv_heads, c.head_dim,
                                      param_ptr(st, l, STAGE_P_GQ), param_ptr(st, l, STAGE_P_GK), base + L.qk_hat,
                                      (const float*)(base + L.qk_r), (float*)(base + P.t_dgp), (float*)(base + P.t_dbp), T, dt, s,
                                      c.bias ? (float*)(base + P.t_dk32) : nullptr, dt == BF16 ? (int)F16 : -1));
      HIP_TRY(st, launch_colsum((const float*)(base + P.t_dgp), headnorm_partials(T, c.n_q_heads), c.head_dim, slot + P.p_off[l][STAGE_P_GQ], s));
      HIP_TRY(st, launch_colsum((const float*)(base + P.t_dbp), headnorm_partials(T, c.n_kv_heads), c.head_dim, slot + P.p_off[l][STAGE_P_GK], s));
    }
    if (c.bias) {
      rc = bias_grad(base + L.dqkv, P.n_qkv, P.p_off[l][STAGE_P_BQKV]);
      if (rc) return rc;
      if (c.qk_norm) {   // the key block again, from the un-rounded gradients (a sum of cancelling terms)
        const int nk = c.n_kv_heads * c.head_dim;
        HIP_TRY(st, launch_colsum_rows(base + P.t_dk32, nk, (float*)(base + P.t_dbp), T, nk, F32, s));
        HIP_TRY(st, launch_colsum((const float*)(base + P.t_dbp), n_chunk, nk, slot + P.p_off[l][STAGE_P_BQKV] + c.n_q_heads * c.head_dim, s));
      }
    }
    // dh1 = [dq|dk|dv] Wqkv^T
    g.A = base + L.dqkv; g.lda = P.n_qkv; g.B = param_ptr(st, l, STAGE_P_WQKV); g.ldb = P.n_qkv;
    g.C = base + P.t_dh; g.ldc = H; g.N = H; g.K = P.n_qkv; g.out_dtype = F32;
    HIP_TRY(st, launch_gemm(g, s));
    rc = norm_bwd(l, true, (const float*)(base + P.t_dh), (const float*)(base + L.x), (const float*)(base + L.r1),
                  (const float*)(base + L.mu1), (const float*)(base + L.dx1_32), dx_out32, dx_out);
    if (rc) return rc;
  }
  HIP_TRY(st, hipEventRecord(m.ev_B, s));
  m.state = MB_B;
  return STAGE_OK;
}

int stage_W(stage_t* st, int mb, void* stream) {
  int rc = check_handle_mb(st, mb);
  if (rc) return rc;
  const Plan& P = st->plan;
  const stage_config& c = P.c;
  MbSlot& m = st->mb[mb];
  if (m.state == MB_POISONED) return refuse_poisoned(st, mb, "W");
  if (m.state != MB_B) {
    set_error(st, m.state == MB_W ? "W(%d) already issued" : "W(%d) before B(%d)", mb, mb);
    return STAGE_ENOTREADY;
  }
  if (st->dry) { m.state = MB_W; return STAGE_OK; }
  int* poison = &m.state;
  hipStream_t s = (hipStream_t)stream;
  HIP_TRY(st, hipStreamWaitEvent(s, m.ev_B, 0));
  char* base = mb_base(st, mb);
  float* slot = slot_base(st, mb);
  const int T = m.T, H = c.hidden, F = c.ffn, dt = c.dtype, nqd = c.n_q_heads * c.head_dim;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerStash& L = P.layer[l];
    GemmArgs g{};
    g.in_dtype = dt; g.out_dtype = F32; g.transA = true; g.transB = false; g.K = T; g.R = nullptr;
    g.ws = base + P.t_dm; g.ws_bytes = (size_t)c.max_tokens * F * 4;   // B's fp32 temporary is idle during W
    g.A = base + L.h1; g.lda = H; g.B = base + L.dqkv; g.ldb = P.n_qkv;
    g.C = slot + P.p_off[l][STAGE_P_WQKV]; g.ldc = P.n_qkv; g.M = H; g.N = P.n_qkv;
    HIP_TRY(st, launch_gemm(g, s));
    g.A = base + L.o; g.lda = nqd; g.B = base + L.dx1; g.ldb = H;
    g.C = slot + P.p_off[l][STAGE_P_WO]; g.ldc = H; g.M = nqd; g.N = H;
    HIP_TRY(st, launch_gemm(g, s));
    g.A = base + L.h2; g.lda = H; g.B = base + L.dup; g.ldb = P.n_up;
    g.C = slot + P.p_off[l][STAGE_P_WUP]; g.ldc = P.n_up; g.M = H; g.N = P.n_up;
    HIP_TRY(st, launch_gemm(g, s));
    g.A = base + L.m; g.lda = F; g.B = base + L.dy; g.ldb = H;
    g.C = slot + P.p_off[l][STAGE_P_WD]; g.ldc = H; g.M = F; g.N = H;
    HIP_TRY(st, launch_gemm(g, s));
  }
  HIP_TRY(st, hipEventRecord(m.ev_W, s));
  m.state = MB_W;
  return STAGE_OK;
}

int stage_grad_reduce(stage_t* st, void* grad_out_dev, void* stream) {
  if (!st) { set_tls_error("stage handle is NULL"); return STAGE_EINVAL; }
  const Plan& P = st->plan;
  if (!st->dry && !grad_out_dev) { set_error(st, "grad_out_dev is NULL"); return STAGE_EINVAL; }
  for (int j = 0; j < P.c.n_microbatches; ++j) {
    if (st->mb[j].state == MB_POISONED) return refuse_poisoned(st, j, "grad_reduce: slot");
    if (st->mb[j].state != MB_W) { set_error(st, "grad_reduce: W(%d) not issued", j); return STAGE_ENOTREADY; }
  }
  if (!st->dry) {
    int* poison = &st->mb[0].state;   // a failed reduce leaves grad_out undefined: the iteration cannot be completed
    hipStream_t s = (hipStream_t)stream;
    for (auto& m : st->mb) HIP_TRY(st, hipStreamWaitEvent(s, m.ev_W, 0));
    HIP_TRY(st, launch_grad_reduce(slot_base(st, 0), align_up(P.slot_floats * 4) / 4, P.c.n_microbatches,
                                   (float*)grad_out_dev, P.slot_floats, s));
    HIP_TRY(st, hipEventRecord(st->ev_reduce, s));
    st->reduce_recorded = true;
  }
  for (auto& m : st->mb) m.state = MB_FREE;
  st->w16_valid = false;    // the caller may change the parameters now: the next F converts Wqkv again
  return STAGE_OK;
}

}  // extern "C"
