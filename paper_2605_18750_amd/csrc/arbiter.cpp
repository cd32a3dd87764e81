// Ready-set arbiter (App. A, Algorithm 1; hint orders of Sec. 7.1 and 7.7; backpressure of App. C.2)
// and a discrete-event pipeline simulator (setting of Sec. 6 plus message latency and the jitter model
// of Sec. 7.6).  Host code; no GPU calls.
//
// Ready buffers are bitmaps, one per (direction, chunk): NextByPriority is a find-first-set over at
// most C words groups, so an arbitration costs O(C * M / 64) with no allocation and no locking.
#include "../../include/rrfp_arbiter.h"

// Simulated times must be reproducible bit for bit by an independent implementation: no fused
// multiply-adds in this file.
#pragma clang fp contract(off)

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <queue>
#include <string>
#include <vector>

namespace {

thread_local std::string g_tls_error;

struct Bits {
  std::vector<uint64_t> w;
  int n = 0;
  void init(int bits) { n = bits; w.assign((bits + 63) / 64, 0); }
  void clear() { std::fill(w.begin(), w.end(), 0); }
  bool test(int i) const { return (w[i >> 6] >> (i & 63)) & 1; }
  void set(int i) { w[i >> 6] |= (uint64_t)1 << (i & 63); }
  void reset(int i) { w[i >> 6] &= ~((uint64_t)1 << (i & 63)); }
  int first() const {
    for (size_t k = 0; k < w.size(); ++k)
      if (w[k]) return (int)(k * 64 + __builtin_ctzll(w[k]));
    return -1;
  }
};

}  // namespace

struct arbiter {
  arbiter_config c;
  // ready[dir][chunk], done[dir][chunk]: bit j = microbatch j
  std::vector<Bits> ready[3], done[3];
  int64_t count[3] = {0, 0, 0};     // n_f, n_b, n_w
  int64_t n_ready[3] = {0, 0, 0};
  int phase = 0;                    // position inside the current round of BF / FB / BFW
  bool in_flight = false;
  arbiter_task flight{};
  std::vector<arbiter_task> fixed;  // binding sequence (FIXED_1F1B)
  size_t fixed_pos = 0;
  std::string error;

  int64_t target() const { return (int64_t)(c.hint == ARB_HINT_BFW ? 3 : 2) * c.n_microbatches * c.n_chunks; }
  int64_t completed() const { return count[0] + count[1] + count[2]; }
  bool backpressure() const { return c.buffer_limit > 0 && count[ARB_F] - count[ARB_B] >= c.buffer_limit; }
};

namespace {

int fail(arbiter* a, int code, const char* fmt, ...) {
  char buf[256];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (a) a->error = buf; else g_tls_error = buf;
  return code;
}

// NextByPriority: forward - smallest chunk, backward and W - largest chunk; ties - smallest microbatch.
bool pick(arbiter* a, int dir, arbiter_task* out) {
  if (a->n_ready[dir] == 0) return false;
  const int C = a->c.n_chunks;
  for (int k = 0; k < C; ++k) {
    const int c = dir == ARB_F ? k : C - 1 - k;
    const int j = a->ready[dir][c].first();
    if (j >= 0) {
      a->ready[dir][c].reset(j);
      --a->n_ready[dir];
      *out = arbiter_task{dir, j, c};
      return true;
    }
  }
  return false;
}

bool take_exact(arbiter* a, int dir, int j, int c, arbiter_task* out) {
  if (!a->ready[dir][c].test(j)) return false;
  a->ready[dir][c].reset(j);
  --a->n_ready[dir];
  *out = arbiter_task{dir, j, c};
  return true;
}

void build_1f1b(arbiter* a) {
  const int M = a->c.n_microbatches;
  const int warm = std::min(a->c.n_stages - 1 - a->c.stage, M);
  a->fixed.clear();
  for (int j = 0; j < warm; ++j) a->fixed.push_back(arbiter_task{ARB_F, j, 0});
  int nf = warm, nb = 0;
  while (nb < M) {
    if (nf < M) a->fixed.push_back(arbiter_task{ARB_F, nf++, 0});
    a->fixed.push_back(arbiter_task{ARB_B, nb++, 0});
  }
}

bool arbitrate(arbiter* a, arbiter_task* out) {
  const arbiter_config& c = a->c;
  const bool bfw = c.hint == ARB_HINT_BFW;
  if (c.hint == ARB_HINT_FIXED_1F1B) {
    const arbiter_task& want = a->fixed[a->fixed_pos];
    if (take_exact(a, want.dir, want.microbatch, want.chunk, out)) { ++a->fixed_pos; return true; }
    return false;
  }
  if (a->backpressure()) {
    if (c.n_chunks == 1) {
      if (pick(a, ARB_B, out)) return true;
      return bfw && pick(a, ARB_W, out);
    }
    // interleaved drain order: first unfinished microbatch, its next required task, else wait
    for (int j = 0; j < c.n_microbatches; ++j) {
      int dir = -1, ch = -1;
      for (int k = 0; k < c.n_chunks && dir < 0; ++k)
        if (!a->done[ARB_F][k].test(j)) { dir = ARB_F; ch = k; }
      for (int k = c.n_chunks - 1; k >= 0 && dir < 0; --k)
        if (!a->done[ARB_B][k].test(j)) { dir = ARB_B; ch = k; }
      if (dir < 0) continue;
      if (take_exact(a, dir, j, ch, out)) return true;
      return bfw && pick(a, ARB_W, out);
    }
    return bfw && pick(a, ARB_W, out);
  }
  if (c.hint == ARB_HINT_B_PRIO) return pick(a, ARB_B, out) || pick(a, ARB_F, out);
  if (c.hint == ARB_HINT_F_PRIO) return pick(a, ARB_F, out) || pick(a, ARB_B, out);
  // rounds: BF and BFW check backward then forward, FB forward then backward
  const int order[2] = {c.hint == ARB_HINT_FB ? ARB_F : ARB_B, c.hint == ARB_HINT_FB ? ARB_B : ARB_F};
  for (int k = 0; k < 2; ++k) {
    const int d = order[a->phase];
    a->phase ^= 1;
    if (pick(a, d, out)) return true;
  }
  a->phase = 0;   // neither direction ready: the next round starts from its first direction
  return bfw && pick(a, ARB_W, out);
}

bool valid_cfg(const arbiter_config* c) {
  if (!c) return false;
  if (c->n_microbatches < 1 || c->n_chunks < 1 || c->n_stages < 1 || c->stage < 0 || c->stage >= c->n_stages) return false;
  if (c->hint < ARB_HINT_BF || c->hint > ARB_HINT_FIXED_1F1B || c->buffer_limit < 0) return false;
  if (c->hint == ARB_HINT_FIXED_1F1B && c->n_chunks != 1) return false;
  return true;
}

}  // namespace

extern "C" {

arbiter_t* arbiter_create(const arbiter_config* cfg) {
  if (!valid_cfg(cfg)) { fail(nullptr, ARB_EINVAL, "arbiter_create: invalid configuration"); return nullptr; }
  arbiter* a = new (std::nothrow) arbiter();
  if (!a) { fail(nullptr, ARB_EINVAL, "arbiter_create: out of memory"); return nullptr; }
  a->c = *cfg;
  for (int d = 0; d < 3; ++d) {
    a->ready[d].resize(cfg->n_chunks);
    a->done[d].resize(cfg->n_chunks);
    for (int k = 0; k < cfg->n_chunks; ++k) { a->ready[d][k].init(cfg->n_microbatches); a->done[d][k].init(cfg->n_microbatches); }
  }
  if (cfg->hint == ARB_HINT_FIXED_1F1B) build_1f1b(a);
  arbiter_reset(a);
  return a;
}

void arbiter_destroy(arbiter_t* a) { delete a; }

int arbiter_reset(arbiter_t* a) {
  if (!a) return fail(nullptr, ARB_EINVAL, "arbiter handle is NULL");
  for (int d = 0; d < 3; ++d) {
    for (auto& b : a->ready[d]) b.clear();
    for (auto& b : a->done[d]) b.clear();
    a->count[d] = 0;
    a->n_ready[d] = 0;
  }
  a->phase = 0;
  a->in_flight = false;
  a->fixed_pos = 0;
  if (a->c.stage == 0) {   // stage 0 admits the first chunk's forwards itself
    for (int j = 0; j < a->c.n_microbatches; ++j) a->ready[ARB_F][0].set(j);
    a->n_ready[ARB_F] = a->c.n_microbatches;
  }
  return ARB_OK;
}

int arbiter_post_ready(arbiter_t* a, int32_t dir, int32_t j, int32_t ch) {
  if (!a) return fail(nullptr, ARB_EINVAL, "arbiter handle is NULL");
  if ((dir != ARB_F && dir != ARB_B) || j < 0 || j >= a->c.n_microbatches || ch < 0 || ch >= a->c.n_chunks)
    return fail(a, ARB_EINVAL, "post_ready: bad task (dir %d, microbatch %d, chunk %d)", dir, j, ch);
  const bool flying = a->in_flight && a->flight.dir == dir && a->flight.microbatch == j && a->flight.chunk == ch;
  if (a->ready[dir][ch].test(j) || a->done[dir][ch].test(j) || flying)
    return fail(a, ARB_ESTATE, "post_ready: %c(%d, chunk %d) already present or done", dir == ARB_F ? 'F' : 'B', j, ch);
  if (dir == ARB_B && !a->done[ARB_F][ch].test(j))
    return fail(a, ARB_ESTATE, "post_ready: backward input of (%d, chunk %d) before its local forward completed", j, ch);
  a->ready[dir][ch].set(j);
  ++a->n_ready[dir];
  return ARB_OK;
}

int arbiter_next(arbiter_t* a, arbiter_task* out) {
  if (!a || !out) return fail(a, ARB_EINVAL, "arbiter_next: NULL argument");
  if (a->in_flight) return fail(a, ARB_ESTATE, "arbiter_next: a task is still in flight");
  if (a->completed() >= a->target()) return ARB_DONE;
  if (!arbitrate(a, out)) return ARB_WAIT;
  a->in_flight = true;
  a->flight = *out;
  return ARB_TASK;
}

int arbiter_complete(arbiter_t* a, const arbiter_task* t) {
  if (!a || !t) return fail(a, ARB_EINVAL, "arbiter_complete: NULL argument");
  if (!a->in_flight || t->dir != a->flight.dir || t->microbatch != a->flight.microbatch || t->chunk != a->flight.chunk)
    return fail(a, ARB_ESTATE, "arbiter_complete: not the task in flight");
  a->in_flight = false;
  ++a->count[t->dir];
  a->done[t->dir][t->chunk].set(t->microbatch);
  if (t->dir == ARB_F && a->c.stage == a->c.n_stages - 1 && t->chunk == a->c.n_chunks - 1) {
    // last stage, last chunk: the forward output becomes the local backward input (App. C.1)
    a->ready[ARB_B][t->chunk].set(t->microbatch);
    ++a->n_ready[ARB_B];
  }
  if (t->dir == ARB_B && a->c.hint == ARB_HINT_BFW) {
    a->ready[ARB_W][t->chunk].set(t->microbatch);
    ++a->n_ready[ARB_W];
  }
  return ARB_OK;
}

int arbiter_counters(const arbiter_t* a, int64_t out[5]) {
  if (!a || !out) return ARB_EINVAL;
  out[0] = a->count[0]; out[1] = a->count[1]; out[2] = a->count[2];
  out[3] = a->backpressure() ? 1 : 0;
  out[4] = a->completed();
  return ARB_OK;
}

const char* arbiter_last_error(const arbiter_t* a) { return a ? a->error.c_str() : g_tls_error.c_str(); }

}  // extern "C"

// ---------------------------------------------------------------------------------------------
// Simulator
// ---------------------------------------------------------------------------------------------
namespace {

inline uint64_t splitmix64(uint64_t x) {
  uint64_t z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

struct Arrival {
  double time;
  int32_t stage, dir, microbatch, chunk;
  bool operator>(const Arrival& o) const { return time > o.time; }
};

}  // namespace

struct jitter {
  double p, base, alpha;
  uint64_t seed;
  int32_t stage, M, C;
  double e = 0.0;
  bool e_set = false;
};

extern "C" jitter_t* jitter_create(double p, double base_seconds, double alpha, uint64_t seed, int32_t stage,
                                   int32_t n_microbatches, int32_t n_chunks) {
  if (p < 0 || p > 1 || base_seconds < 0 || alpha < 0 || stage < 0 || n_microbatches < 1 || n_chunks < 1) {
    fail(nullptr, ARB_EINVAL, "jitter_create: invalid parameters");
    return nullptr;
  }
  jitter* j = new (std::nothrow) jitter();
  if (!j) return nullptr;
  j->p = p; j->base = base_seconds; j->alpha = alpha; j->seed = seed;
  j->stage = stage; j->M = n_microbatches; j->C = n_chunks;
  return j;
}

extern "C" void jitter_destroy(jitter_t* j) { delete j; }

extern "C" double jitter_next_delay(jitter_t* j, int32_t dir, int32_t microbatch, int32_t chunk, double c) {
  if (!j) return 0.0;
  j->e = j->e_set ? 0.9 * j->e + 0.1 * c : c;
  j->e_set = true;
  const uint64_t k = (((uint64_t)j->stage * 3 + dir) * j->C + chunk) * j->M + microbatch;
  const double u1 = (double)(splitmix64(j->seed ^ splitmix64(2 * k)) >> 11) * 0x1.0p-53;
  const double u2 = (double)(splitmix64(j->seed ^ splitmix64(2 * k + 1)) >> 11) * 0x1.0p-53;
  if (u1 < j->p) return j->alpha * std::max(j->base, j->e) * (0.5 + u2);
  return 0.0;
}

// The event loop of a whole pipeline as a resumable object: rrfp_pipe_next() advances the virtual clock to
// the next dispatch and returns it; the caller supplies that task's duration before asking again.  The
// simulator below and a runtime that enqueues real stage tasks both drive this one loop, so the routing
// rule (who sends which message to whom, Sec. 4.1; the local turn-around at the last stage, App. C.1) exists
// once.
struct rrfp_pipe {
  rrfp_sim_config cfg{};
  int N = 0, M = 0, C = 0;
  bool fwd_only = false, bwd_only = false, only = false;
  std::vector<arbiter*> st;
  struct Run { bool busy = false; arbiter_task t{}; double end = 0; };
  std::vector<Run> run;
  std::priority_queue<Arrival, std::vector<Arrival>, std::greater<Arrival>> arrivals;
  std::vector<double> busy;
  std::vector<jitter> inject;
  std::vector<int64_t> fwd_held, bwd_held, max_f, max_b, max_D, done;
  int64_t only_target = 0, n_events = 0;
  double makespan = 0.0, t = 0.0;
  int scan = -1;            // -1: completions and arrivals at time t not processed yet; else next stage to arbitrate
  int pending = -1;         // stage whose dispatched task still waits for its duration
  bool finished = false, deadlock = false;

  ~rrfp_pipe() { for (auto* a : st) arbiter_destroy(a); }

  void deliver(int s, int dir, int j, int c) {
    arbiter_post_ready(st[s], dir, j, c);
    if (dir == ARB_F) { if (++fwd_held[s] > max_f[s]) max_f[s] = fwd_held[s]; }
    else { if (++bwd_held[s] > max_b[s]) max_b[s] = bwd_held[s]; }
  }

  bool init(const rrfp_sim_config* c) {
    cfg = *c;
    N = c->n_stages; M = c->n_microbatches; C = c->n_chunks;
    fwd_only = c->mode == 1; bwd_only = c->mode == 2; only = c->mode != 0;
    st.assign(N, nullptr);
    for (int s = 0; s < N; ++s) {
      arbiter_config ac{M, C, c->hint, c->buffer_limit, s, N};
      if (only) {
        // reference executions: one direction only; no backpressure, the loop seeds the first buffer itself
        ac.hint = ARB_HINT_BF;
        ac.buffer_limit = 0;
      }
      st[s] = arbiter_create(&ac);
      if (!st[s]) return false;
    }
    run.assign(N, Run{});
    busy.assign(N, 0.0);
    inject.assign(N, jitter{});
    for (int s = 0; s < N; ++s) {
      inject[s].p = c->jitter_p; inject[s].base = c->jitter_base; inject[s].alpha = c->jitter_alpha;
      inject[s].seed = c->jitter_seed; inject[s].stage = s; inject[s].M = M; inject[s].C = C;
    }
    fwd_held.assign(N, 0); bwd_held.assign(N, 0); max_f.assign(N, 0); max_b.assign(N, 0); max_D.assign(N, 0); done.assign(N, 0);
    only_target = (int64_t)M * C;
    if (bwd_only) {
      // all backward work available at the last stage: mark the local forwards as done first
      for (int s = 0; s < N; ++s)
        for (int cc = 0; cc < C; ++cc)
          for (int j = 0; j < M; ++j) st[s]->done[ARB_F][cc].set(j);
      for (int j = 0; j < M; ++j) deliver(N - 1, ARB_B, j, C - 1);
      // stage 0's self-admitted forwards are not part of this reference run
      st[0]->ready[ARB_F][0].clear();
      st[0]->n_ready[ARB_F] = 0;
    }
    return true;
  }

  // A task of stage s has ended at time `at`: completion bookkeeping and the message it sends.
  void finish(int s, const arbiter_task& tk, double at) {
    if (!(fwd_only && s == N - 1 && tk.dir == ARB_F && tk.chunk == C - 1)) {
      arbiter_complete(st[s], &tk);
    } else {
      // forward-only reference: no turn-around at the last stage
      st[s]->in_flight = false;
      ++st[s]->count[ARB_F];
      st[s]->done[ARB_F][tk.chunk].set(tk.microbatch);
    }
    ++done[s];
    if (tk.dir == ARB_F) {
      if (s + 1 < N) arrivals.push(Arrival{at + cfg.latency, s + 1, ARB_F, tk.microbatch, tk.chunk});
      else if (tk.chunk + 1 < C) arrivals.push(Arrival{at + cfg.latency, 0, ARB_F, tk.microbatch, tk.chunk + 1});
      else if (!fwd_only) { if (++bwd_held[s] > max_b[s]) max_b[s] = bwd_held[s]; }   // local move (done inside the arbiter)
    } else if (tk.dir == ARB_B) {
      if (!bwd_only) --fwd_held[s];
      --bwd_held[s];
      if (s > 0) arrivals.push(Arrival{at + cfg.latency, s - 1, ARB_B, tk.microbatch, tk.chunk});
      else if (tk.chunk > 0) arrivals.push(Arrival{at + cfg.latency, N - 1, ARB_B, tk.microbatch, tk.chunk - 1});
    }
  }

  bool all_done() const {
    for (int s = 0; s < N; ++s) {
      if (only ? done[s] < only_target : st[s]->completed() < st[s]->target()) return false;
      if (run[s].busy) return false;
    }
    return true;
  }

  // Who produced the input of task (dir, chunk) at stage s: the neighbour in that direction, the other end of
  // the pipeline when the microbatch changes chunk, or nobody (-1: the caller's tensor; for the backward of
  // the last stage's last chunk, the caller's output gradient).
  void source(int s, int dir, int c, int32_t* src_stage, int32_t* src_chunk) const {
    *src_stage = -1; *src_chunk = -1;
    if (dir == ARB_F) {
      if (s > 0) { *src_stage = s - 1; *src_chunk = c; }
      else if (c > 0) { *src_stage = N - 1; *src_chunk = c - 1; }
    } else if (dir == ARB_B) {
      if (s + 1 < N) { *src_stage = s + 1; *src_chunk = c; }
      else if (c + 1 < C) { *src_stage = 0; *src_chunk = c + 1; }
    }
  }

  // Advances to the next dispatch.  ARB_TASK: *out filled, the stage is busy from out->start and the caller owes
  // set_duration(); ARB_DONE: everything has completed; ARB_ESTATE: stalled (unfinished work, nothing in flight).
  int next(rrfp_pipe_dispatch* out) {
    if (pending >= 0) return ARB_ESTATE;
    if (finished) return deadlock ? ARB_ESTATE : ARB_DONE;
    for (;;) {
      if (scan < 0) {
        for (int s = 0; s < N; ++s)
          if (run[s].busy && run[s].end <= t) { run[s].busy = false; finish(s, run[s].t, run[s].end); }
        while (!arrivals.empty() && arrivals.top().time <= t) {
          const Arrival a = arrivals.top();
          arrivals.pop();
          deliver(a.stage, a.dir, a.microbatch, a.chunk);
        }
        scan = 0;
      }
      for (; scan < N; ++scan) {
        const int s = scan;
        if (run[s].busy) continue;
        if (only && done[s] >= only_target) continue;
        const int64_t D = st[s]->count[ARB_F] - st[s]->count[ARB_B];
        if (D > max_D[s]) max_D[s] = D;
        arbiter_task task;
        if (arbiter_next(st[s], &task) != ARB_TASK) continue;
        if (s == 0 && task.dir == ARB_F && task.chunk == 0) { if (++fwd_held[0] > max_f[0]) max_f[0] = fwd_held[0]; }
        run[s].busy = true;
        run[s].t = task;
        run[s].end = t;
        out->stage = s; out->dir = task.dir; out->microbatch = task.microbatch; out->chunk = task.chunk;
        out->start = t;
        source(s, task.dir, task.chunk, &out->src_stage, &out->src_chunk);
        pending = s;
        ++scan;
        ++n_events;
        return ARB_TASK;
      }
      scan = -1;
      if (all_done()) { finished = true; return ARB_DONE; }
      bool have = false;
      double nxt = 0.0;
      for (int s = 0; s < N; ++s)
        if (run[s].busy && (!have || run[s].end < nxt)) { nxt = run[s].end; have = true; }
      if (!arrivals.empty() && (!have || arrivals.top().time < nxt)) { nxt = arrivals.top().time; have = true; }
      if (!have) { finished = true; deadlock = true; return ARB_ESTATE; }
      t = nxt;
    }
  }

  // Duration of the task next() returned last; adds the jitter delay of the configuration (F and B tasks
  // only) and returns it through *delay.
  int set_duration(double seconds, double* delay, double* end) {
    if (pending < 0 || !(seconds >= 0.0)) return ARB_ESTATE;
    const int s = pending;
    pending = -1;
    double p = seconds, d = 0.0;
    if (cfg.jitter_p > 0.0 && run[s].t.dir != ARB_W) {
      d = jitter_next_delay(&inject[s], run[s].t.dir, run[s].t.microbatch, run[s].t.chunk, p);
      p = p + d;
    }
    run[s].end = t + p;
    busy[s] += p;
    if (run[s].end > makespan) makespan = run[s].end;
    if (delay) *delay = d;
    if (end) *end = run[s].end;
    return ARB_OK;
  }
};

namespace {
bool valid_sim_cfg(const rrfp_sim_config* cfg) {
  return cfg && cfg->n_stages >= 1 && cfg->n_microbatches >= 1 && cfg->n_chunks >= 1 && cfg->mode >= 0 && cfg->mode <= 2 &&
         cfg->latency >= 0 && cfg->jitter_p >= 0 && cfg->jitter_p <= 1 && cfg->jitter_base >= 0 && cfg->jitter_alpha >= 0;
}
}  // namespace

extern "C" rrfp_pipe_t* rrfp_pipe_create(const rrfp_sim_config* cfg) {
  if (!valid_sim_cfg(cfg)) { fail(nullptr, ARB_EINVAL, "rrfp_pipe_create: invalid configuration"); return nullptr; }
  rrfp_pipe* p = new (std::nothrow) rrfp_pipe();
  if (!p) { fail(nullptr, ARB_EINVAL, "rrfp_pipe_create: out of memory"); return nullptr; }
  if (!p->init(cfg)) { delete p; return nullptr; }   // arbiter_create left the message
  return p;
}

extern "C" void rrfp_pipe_destroy(rrfp_pipe_t* p) { delete p; }

extern "C" int rrfp_pipe_next(rrfp_pipe_t* p, rrfp_pipe_dispatch* out) {
  if (!p || !out) return fail(nullptr, ARB_EINVAL, "rrfp_pipe_next: NULL argument");
  const int rc = p->next(out);
  if (rc == ARB_ESTATE)
    fail(nullptr, ARB_ESTATE, p->deadlock ? "rrfp_pipe_next: pipeline stalled (unfinished work, nothing in flight)"
                                          : "rrfp_pipe_next: the previous task still waits for rrfp_pipe_set_duration");
  return rc;
}

extern "C" int rrfp_pipe_set_duration(rrfp_pipe_t* p, double seconds, double* delay_seconds, double* end) {
  if (!p) return fail(nullptr, ARB_EINVAL, "rrfp_pipe_set_duration: NULL handle");
  const int rc = p->set_duration(seconds, delay_seconds, end);
  if (rc != ARB_OK) fail(nullptr, rc, "rrfp_pipe_set_duration: no task waits for a duration, or the duration is negative");
  return rc;
}

extern "C" int rrfp_sim_run(const rrfp_sim_config* cfg, const double* dur_f, const double* dur_b, const double* dur_w,
                            rrfp_sim_result* result, double* per_stage, rrfp_sim_event* trace, int64_t trace_cap) {
  if (!cfg || !result || !dur_f || !dur_b) return fail(nullptr, ARB_EINVAL, "rrfp_sim_run: NULL argument");
  if (!valid_sim_cfg(cfg) || (trace && trace_cap < 0)) return fail(nullptr, ARB_EINVAL, "rrfp_sim_run: invalid configuration");
  if (cfg->hint == ARB_HINT_BFW && !dur_w) return fail(nullptr, ARB_EINVAL, "rrfp_sim_run: BFW needs dur_w");
  rrfp_pipe pipe;
  if (!pipe.init(cfg)) return ARB_EINVAL;
  const int M = cfg->n_microbatches, C = cfg->n_chunks;
  rrfp_pipe_dispatch d;
  int rc;
  while ((rc = pipe.next(&d)) == ARB_TASK) {
    const size_t idx = ((size_t)d.stage * C + d.chunk) * M + d.microbatch;
    const double p = d.dir == ARB_F ? dur_f[idx] : d.dir == ARB_B ? dur_b[idx] : dur_w[idx];
    double end = 0.0;
    pipe.set_duration(p, nullptr, &end);
    const int64_t k = pipe.n_events - 1;
    if (trace && k < trace_cap) trace[k] = rrfp_sim_event{d.stage, d.dir, d.microbatch, d.chunk, d.start, end};
  }
  result->makespan = pipe.makespan;
  result->n_events = pipe.n_events;
  result->deadlock = pipe.deadlock ? 1 : 0;
  if (per_stage)
    for (int s = 0; s < cfg->n_stages; ++s) {
      per_stage[4 * s + 0] = pipe.busy[s];
      per_stage[4 * s + 1] = (double)pipe.max_f[s];
      per_stage[4 * s + 2] = (double)pipe.max_b[s];
      per_stage[4 * s + 3] = (double)pipe.max_D[s];
    }
  return ARB_OK;
}
