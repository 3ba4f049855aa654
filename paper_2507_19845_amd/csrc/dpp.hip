// Traversal of the (micro-batch, model chunk) task matrix: the depth-first, breadth-first
// and best-effort breadth-first orders of the paper's section 5.2 (MegaDPP, "parallel
// scheduler"), and a driver that issues the tasks of several chunks held by one GPU through
// the decoupled entry points.  Host code only: the arithmetic is in the stage kernels.
#include "../../include/gpt_stage.h"

#include <chrono>
#include <thread>
#include <vector>

#include "kernels.hpp"

using gpts::set_error;

namespace {

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// micro-batches per window
int window(int policy, int C, int M, int max_live_stash) {
  if (policy == GPT_DPP_DFC) return 1;
  if (policy == GPT_DPP_BFC) return M;
  int w = max_live_stash / C;
  if (w < 1) w = 1;
  if (w > M) w = M;
  return w;
}

// simple free list over equal slots of a caller-provided pool
struct Pool {
  char* base;
  size_t slot;
  std::vector<int> free_ids;
  int live = 0, peak = 0;
  Pool(void* b, size_t slot_bytes, size_t pool_bytes) : base(static_cast<char*>(b)), slot(slot_bytes) {
    const int n = slot_bytes ? (int)(pool_bytes / slot_bytes) : 0;
    for (int i = n - 1; i >= 0; --i) free_ids.push_back(i);
  }
  int take() {
    if (free_ids.empty()) return -1;
    const int id = free_ids.back();
    free_ids.pop_back();
    if (++live > peak) peak = live;
    return id;
  }
  void give(int id) {
    free_ids.push_back(id);
    --live;
  }
  void* at(int id) const { return base + (size_t)id * slot; }
};

// ---- run-time scheduling: the ready set -----------------------------------------------------
// Section 5.2: with asynchronous transfers "a compute thread can always pick the highest-priority
// ready input for execution".  A task is READY when the tasks it depends on have been issued and
// its external input (x of micro-batch i for F(i,0), dy of micro-batch i for B(i,C-1)) has
// arrived; the priority of a task is its position in the static plan of the chosen policy.
// Two more rules keep the results and the memory use those of the static plan:
//  * backward tasks of one chunk are issued in ascending micro-batch order (the order in which
//    the chunk's gradients accumulate, hence every result bit);
//  * a forward task needs a free stash slot, and a micro-batch is only STARTED (F(i,0)) while
//    the free slots, after setting aside what the micro-batches in flight still need to reach
//    the last chunk, cover all its chunks -- so a micro-batch that has started can always finish;
//    started ahead of a lower-numbered one, it leaves another n_chunks slots free, through which
//    the lower ones (whose backward tasks go first) can pass one after the other.
struct ReadySet {
  int C, M, free_slots, reserved = 0;
  std::vector<gpt_dpp_task> plan;
  std::vector<char> issued, x_ok, dy_ok;       // issued: by plan position
  std::vector<int> pos_of;                     // plan position of task (phase, i, j)
  std::vector<int> next_bwd;                   // per chunk: the micro-batch whose backward is due
  int n_issued = 0, first_open = 0;
  int id(int phase, int i, int j) const { return (phase * M + i) * C + j; }
  ReadySet(int policy, int C_, int M_, int allowance, int slots)
      : C(C_), M(M_), free_slots(slots), plan((size_t)2 * C_ * M_), issued((size_t)2 * C_ * M_, 0),
        x_ok(M_, 0), dy_ok(M_, 0), pos_of((size_t)2 * C_ * M_, -1), next_bwd(C_, 0) {
    const int n = gpt_dpp_plan(policy, C, M, allowance, plan.data(), (int)plan.size(), nullptr);
    for (int t = 0; t < n; ++t) pos_of[id(plan[t].phase, plan[t].microbatch, plan[t].chunk)] = t;
  }
  bool done(int phase, int i, int j) const { return issued[pos_of[id(phase, i, j)]] != 0; }
  bool ready(const gpt_dpp_task& k) const {
    const int i = k.microbatch, j = k.chunk;
    if (k.phase == GPT_DPP_FWD) {
      if (j == 0 ? !x_ok[i] : !done(GPT_DPP_FWD, i, j - 1)) return false;
      if (j > 0) return free_slots > 0;
      // starting ahead of a lower-numbered micro-batch: its backward tasks will have to wait for
      // that one's, so room for the lower ones to pass through (one at a time) stays set aside
      bool lower_started = true;
      for (int k = 0; k < i && lower_started; ++k) lower_started = done(GPT_DPP_FWD, k, 0);
      return free_slots - reserved >= (lower_started ? C : 2 * C);
    }
    if (!done(GPT_DPP_FWD, i, j) || next_bwd[j] != i) return false;
    return j == C - 1 ? dy_ok[i] != 0 : done(GPT_DPP_BWD, i, j + 1);
  }
  // plan position of the first ready task, or -1
  int pick() {
    while (first_open < (int)plan.size() && issued[first_open]) ++first_open;
    for (int t = first_open; t < (int)plan.size(); ++t)
      if (!issued[t] && ready(plan[t])) return t;
    return -1;
  }
  void issue(int t) {
    const gpt_dpp_task& k = plan[t];
    issued[t] = 1;
    ++n_issued;
    if (k.phase == GPT_DPP_FWD) {
      --free_slots;
      reserved += k.chunk == 0 ? C - 1 : -1;
    } else {
      ++free_slots;
      ++next_bwd[k.chunk];
    }
  }
  bool finished() const { return n_issued == (int)plan.size(); }
};

int check_counts(int policy, int C, int M, const char* who) {
  if (policy != GPT_DPP_DFC && policy != GPT_DPP_BFC && policy != GPT_DPP_BFC_BEST_EFFORT)
    return set_error(GPTS_EINVAL, who);
  if (C < 1 || M < 1 || C > (1 << 15) || M > (1 << 15) || (long long)2 * C * M > (1ll << 30))
    return set_error(GPTS_EINVAL, who);
  return GPTS_OK;
}

// Issues one task of a job through the decoupled stage entry points, taking and returning
// stash slots and boundary buffers (shared by the static and the run-time driver).
struct TaskIssuer {
  const gpt_dpp_job* job;
  void* stream;
  Pool stash, act;
  std::vector<int> slot_of, fwd_buf, bwd_buf, left;
  // weight phase per chunk and window (job->grad_pool): W micro-batches per window, stash slot of
  // task (i, j) fixed at j*W + i%W so that a chunk's stashes of one window are equally spaced
  int W = 0;
  size_t stash_slot_bytes, grad_slot_bytes = 0;
  int live_fixed = 0, peak_fixed = 0;
  TaskIssuer(const gpt_dpp_job* j, void* st, size_t stash_slot, size_t act_slot)
      : job(j), stream(st), stash(j->stash_pool, stash_slot, j->stash_pool ? j->stash_pool_bytes : 0),
        act(j->act_pool, act_slot, j->act_pool ? j->act_pool_bytes : 0),
        slot_of((size_t)j->n_chunks * j->n_microbatches, -1), fwd_buf(j->n_microbatches, -1),
        bwd_buf(j->n_microbatches, -1), left(j->n_chunks, j->n_microbatches), stash_slot_bytes(stash_slot) {}
  void* stash_at(int i, int j) { return static_cast<char*>(job->stash_pool) + (size_t)(j * W + i % W) * stash_slot_bytes; }
  void* grad_at(int i) { return static_cast<char*>(job->grad_pool) + (size_t)(i % W) * grad_slot_bytes; }
  int issue(const gpt_dpp_task& k) {
    const int C = job->n_chunks, i = k.microbatch, j = k.chunk;
    if (k.phase == GPT_DPP_FWD) {
      const void* in = (j == 0) ? job->x[i] : act.at(fwd_buf[i]);
      int out_id = -1;
      void* out = job->y[i];
      if (j != C - 1) {
        if (act.free_ids.empty()) return set_error(GPTS_ENOMEM, "dpp: boundary-activation pool exhausted");
        out_id = act.take();
        out = act.at(out_id);
      }
      void* slot;
      if (W > 0) {
        slot = stash_at(i, j);
        if (++live_fixed > peak_fixed) peak_fixed = live_fixed;
      } else {
        if (stash.free_ids.empty()) return set_error(GPTS_ENOMEM, "dpp: stash pool exhausted");
        const int s = stash.take();
        slot_of[(size_t)i * C + j] = s;
        slot = stash.at(s);
      }
      const int rc = gpt_stage_fwd_only(&job->chunks[j], in, slot, out, stream, nullptr);
      if (rc != GPTS_OK) return rc;
      if (j != 0) act.give(fwd_buf[i]);
      fwd_buf[i] = out_id;
    } else {
      const void* din = (j == C - 1) ? job->dy[i] : act.at(bwd_buf[i]);
      int out_id = -1;
      void* dout = job->dx[i];
      if (j != 0) {
        if (act.free_ids.empty()) return set_error(GPTS_ENOMEM, "dpp: boundary-activation pool exhausted");
        out_id = act.take();
        dout = act.at(out_id);
      }
      if (W > 0) {
        int rc = gpt_stage_bwd_data_only(&job->chunks[j], stash_at(i, j), din, dout, job->dparams[j], grad_at(i), stream, nullptr);
        if (rc != GPTS_OK) return rc;
        const int M = job->n_microbatches;
        if (i % W == W - 1 || i == M - 1) {
          // the chunk has seen every micro-batch of the window: one weight phase over them
          const int w0 = i / W * W, n = i - w0 + 1;
          std::vector<const void*> as(n), gs(n);
          for (int m = 0; m < n; ++m) {
            as[m] = stash_at(w0 + m, j);
            gs[m] = grad_at(w0 + m);
          }
          rc = gpt_stage_wgrad_flush(&job->chunks[j], n, as.data(), gs.data(), job->dparams[j], stream);
          if (rc != GPTS_OK) return rc;
          live_fixed -= n;
        }
      } else {
        const int s = slot_of[(size_t)i * C + j];
        const int rc = gpt_stage_bwd_only(&job->chunks[j], stash.at(s), din, dout, job->dparams[j], stream, nullptr);
        if (rc != GPTS_OK) return rc;
        stash.give(s);
      }
      if (j != C - 1) act.give(bwd_buf[i]);
      bwd_buf[i] = out_id;
      if (--left[j] == 0 && job->grad_ready && job->grad_ready[j]) {
        const hipError_t e = hipEventRecord(static_cast<hipEvent_t>(job->grad_ready[j]), static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return set_error(GPTS_EHIP, "dpp: recording a grad_ready event failed");
      }
    }
    return GPTS_OK;
  }
};

int check_job(const gpt_dpp_job* job, const char* who) {
  if (!job) return set_error(GPTS_EINVAL, who);
  const int C = job->n_chunks, M = job->n_microbatches;
  if (C < 1 || M < 1 || C > (1 << 15) || M > (1 << 15)) return set_error(GPTS_EINVAL, "dpp: n_chunks and n_microbatches must be in [1, 32768]");
  if (!job->chunks || !job->x || !job->dy || !job->y || !job->dx || !job->dparams)
    return set_error(GPTS_EINVAL, "dpp: chunks / x / dy / y / dx / dparams array is NULL");
  for (int j = 0; j < C; ++j) {
    const int rc = gpt_stage_validate(&job->chunks[j].cfg);
    if (rc != GPTS_OK) return rc;
    const gpt_stage_cfg &a = job->chunks[0].cfg, &b = job->chunks[j].cfg;
    if (a.batch != b.batch || a.seq != b.seq || a.hidden != b.hidden || a.dtype != b.dtype)
      return set_error(GPTS_ESHAPE, "dpp: chunks must share batch, seq, hidden and dtype");
    if (!job->dparams[j]) return set_error(GPTS_EINVAL, "dpp: a dparams pointer is NULL");
  }
  for (int i = 0; i < M; ++i)
    if (!job->x[i] || !job->dy[i] || !job->y[i] || !job->dx[i])
      return set_error(GPTS_EINVAL, "dpp: an x / dy / y / dx pointer is NULL");
  return GPTS_OK;
}

}  // namespace

extern "C" {

int gpt_dpp_simulate_ready(int policy, int n_chunks, int n_microbatches, int max_live_stash,
                           const int32_t* x_at, const int32_t* dy_at, int dynamic, gpt_dpp_task* order,
                           int capacity, int32_t* n_steps, int32_t* idle_steps) {
  int rc = check_counts(policy, n_chunks, n_microbatches, "dpp_simulate_ready: unknown policy or counts outside [1, 32768]");
  if (rc != GPTS_OK) return rc;
  const int C = n_chunks, M = n_microbatches, total = 2 * C * M;
  if (!order || capacity < total) return set_error(GPTS_ENOMEM, "dpp_simulate_ready: order array holds fewer than 2*chunks*microbatches entries");
  for (int i = 0; i < M; ++i)
    if ((x_at && x_at[i] < 0) || (dy_at && dy_at[i] < 0)) return set_error(GPTS_EINVAL, "dpp_simulate_ready: arrival steps must be >= 0");
  // slots: what the static plan of the policy needs at its peak (so the dynamic order never holds more)
  std::vector<gpt_dpp_task> plan((size_t)total);
  int slots = 0;
  gpt_dpp_plan(policy, C, M, max_live_stash, plan.data(), total, &slots);
  ReadySet rs(policy, C, M, max_live_stash, slots);
  int step = 0, idle = 0, n = 0;
  const long long limit = 4ll * total + 8;   // arrivals later than this would only add idle steps
  long long last_arrival = 0;
  for (int i = 0; i < M; ++i) {
    if (x_at && x_at[i] > last_arrival) last_arrival = x_at[i];
    if (dy_at && dy_at[i] > last_arrival) last_arrival = dy_at[i];
  }
  while (!rs.finished()) {
    if (step > last_arrival + limit) return set_error(GPTS_EINVAL, "dpp_simulate_ready: the schedule cannot make progress");
    for (int i = 0; i < M; ++i) {
      rs.x_ok[i] = !x_at || x_at[i] <= step;
      rs.dy_ok[i] = !dy_at || dy_at[i] <= step;
    }
    int t;
    if (dynamic) {
      t = rs.pick();
    } else {               // static: the plan's next task or nothing
      while (rs.first_open < total && rs.issued[rs.first_open]) ++rs.first_open;
      t = rs.ready(rs.plan[rs.first_open]) ? rs.first_open : -1;
    }
    if (t >= 0) {
      order[n++] = rs.plan[t];
      rs.issue(t);
    } else {
      ++idle;
    }
    ++step;
  }
  if (n_steps) *n_steps = step;
  if (idle_steps) *idle_steps = idle;
  return n;
}

int gpt_dpp_plan(int policy, int n_chunks, int n_microbatches, int max_live_stash,
                 gpt_dpp_task* tasks, int capacity, int* peak_live_stash) {
  if (policy != GPT_DPP_DFC && policy != GPT_DPP_BFC && policy != GPT_DPP_BFC_BEST_EFFORT)
    return set_error(GPTS_EINVAL, "dpp_plan: unknown policy");
  if (n_chunks < 1 || n_microbatches < 1 || n_chunks > (1 << 15) || n_microbatches > (1 << 15))
    return set_error(GPTS_EINVAL, "dpp_plan: n_chunks and n_microbatches must be in [1, 32768]");
  if (!tasks) return set_error(GPTS_EINVAL, "dpp_plan: tasks is NULL");
  const int C = n_chunks, M = n_microbatches;
  // the task count is also the return value, an int
  if ((long long)2 * C * M > (1ll << 30))
    return set_error(GPTS_EINVAL, "dpp_plan: 2*chunks*microbatches must not exceed 2^30");
  const int total = 2 * C * M;
  if (capacity < total) return set_error(GPTS_ENOMEM, "dpp_plan: tasks array holds fewer than 2*chunks*microbatches entries");
  const int W = window(policy, C, M, max_live_stash);
  int n = 0, live = 0, peak = 0;
  for (int w0 = 0; w0 < M; w0 += W) {
    const int w1 = w0 + W < M ? w0 + W : M;
    for (int j = 0; j < C; ++j)
      for (int i = w0; i < w1; ++i) {
        tasks[n++] = gpt_dpp_task{GPT_DPP_FWD, i, j};
        if (++live > peak) peak = live;
      }
    for (int j = C - 1; j >= 0; --j)
      for (int i = w0; i < w1; ++i) {
        tasks[n++] = gpt_dpp_task{GPT_DPP_BWD, i, j};
        --live;
      }
  }
  if (peak_live_stash) *peak_live_stash = peak;
  return n;
}

size_t gpt_dpp_stash_slot_bytes(const gpt_stage_params* chunks, int n_chunks) {
  if (!chunks || n_chunks < 1) return 0;
  size_t m = 0;
  for (int j = 0; j < n_chunks; ++j) {
    const size_t b = gpt_stage_stash_bytes(&chunks[j].cfg);
    if (b == 0) return 0;
    if (b > m) m = b;
  }
  return align256(m);
}

size_t gpt_dpp_grad_slot_bytes(const gpt_stage_params* chunks, int n_chunks) {
  if (!chunks || n_chunks < 1) return 0;
  size_t m = 0;
  for (int j = 0; j < n_chunks; ++j) {
    const size_t b = gpt_stage_grad_stash_bytes(&chunks[j].cfg);
    if (b == 0) return 0;
    if (b > m) m = b;
  }
  return align256(m);
}

size_t gpt_dpp_act_slot_bytes(const gpt_stage_cfg* cfg) {
  if (gpt_stage_validate(cfg) != GPTS_OK) return 0;
  return align256((size_t)cfg->batch * cfg->seq * cfg->hidden * (cfg->dtype == GPTS_BF16 ? 2 : 4));
}

int gpt_dpp_allowance_from_free_memory(const gpt_stage_params* chunks, int n_chunks, int n_microbatches,
                                       size_t reserve_bytes, size_t* stash_pool_bytes,
                                       size_t* act_pool_bytes) {
  if (!chunks || n_chunks < 1 || n_microbatches < 1 || n_chunks > (1 << 15) || n_microbatches > (1 << 15))
    return set_error(GPTS_EINVAL, "dpp_allowance: chunks NULL or counts outside [1, 32768]");
  const size_t slot = gpt_dpp_stash_slot_bytes(chunks, n_chunks);
  const size_t act_slot = gpt_dpp_act_slot_bytes(&chunks[0].cfg);
  if (!slot || !act_slot) return set_error(GPTS_ESHAPE, "dpp_allowance: a chunk's cfg is not valid");
  size_t free_b = 0, total_b = 0;
  if (hipMemGetInfo(&free_b, &total_b) != hipSuccess) return set_error(GPTS_EHIP, "dpp_allowance: hipMemGetInfo failed");
  // boundary buffers: a window of W micro-batches keeps at most W + 1 alive; budget for the widest
  const size_t act_bytes = ((size_t)n_microbatches + 1) * act_slot;
  const size_t need_first = reserve_bytes + act_bytes;
  size_t slots = free_b > need_first ? (free_b - need_first) / slot : 0;
  const size_t all = (size_t)n_chunks * n_microbatches;
  if (slots > all) slots = all;
  // whole windows only: the scheduler runs W = slots / chunks micro-batches per window
  slots = slots / n_chunks * n_chunks;
  if (stash_pool_bytes) *stash_pool_bytes = slots * slot;
  if (act_pool_bytes) *act_pool_bytes = act_bytes;
  return (int)slots;
}

int gpt_dpp_run(const gpt_dpp_job* job, void* stream, gpt_dpp_report* report) {
  int rc = check_job(job, "dpp_run: job is NULL");
  if (rc != GPTS_OK) return rc;
  const int C = job->n_chunks, M = job->n_microbatches;
  const size_t stash_slot = gpt_dpp_stash_slot_bytes(job->chunks, C);
  const size_t act_slot = gpt_dpp_act_slot_bytes(&job->chunks[0].cfg);
  // best effort without a caller-given allowance: as wide as the stash pool at hand allows
  // (section 5.2: breadth first "as long as it does not cause" out-of-memory)
  int allowance = job->max_live_stash;
  if (job->policy == GPT_DPP_BFC_BEST_EFFORT && allowance <= 0) {
    const size_t slots = (job->stash_pool && stash_slot) ? job->stash_pool_bytes / stash_slot : 0;
    allowance = slots > (size_t)C * M ? C * M : (int)slots;
  }
  std::vector<gpt_dpp_task> plan((size_t)2 * C * M);
  int peak_stash = 0;
  const int n = gpt_dpp_plan(job->policy, C, M, allowance, plan.data(), (int)plan.size(), &peak_stash);
  if (n < 0) return n;
  TaskIssuer issuer(job, stream, stash_slot, act_slot);
  if (job->grad_pool) {
    const int W = window(job->policy, C, M, allowance);
    const size_t gslot = gpt_dpp_grad_slot_bytes(job->chunks, C);
    if (!gslot) return set_error(GPTS_ESHAPE, "dpp_run: a chunk's cfg is not valid");
    if (job->grad_pool_bytes < (size_t)W * gslot)
      return set_error(GPTS_ENOMEM, "dpp_run: grad_pool too small (one gradient-stash slot per micro-batch of a window)");
    if (!job->stash_pool || job->stash_pool_bytes < (size_t)C * W * stash_slot)
      return set_error(GPTS_ENOMEM, "dpp_run: with grad_pool the stash pool must hold n_chunks * window slots");
    issuer.W = W;
    issuer.grad_slot_bytes = gslot;
  }

  // dry run of the pool usage, so that nothing is enqueued when a pool is too small
  {
    int live_act = 0, peak_act = 0;
    for (int t = 0; t < n; ++t) {
      const gpt_dpp_task& k = plan[t];
      const bool edge = (k.phase == GPT_DPP_FWD) ? (k.chunk == C - 1) : (k.chunk == 0);   // writes y / dx
      const bool first = (k.phase == GPT_DPP_FWD) ? (k.chunk == 0) : (k.chunk == C - 1);  // reads x / dy
      if (!edge && ++live_act > peak_act) peak_act = live_act;
      if (!first) --live_act;
    }
    if (!issuer.W && (size_t)peak_stash > issuer.stash.free_ids.size()) return set_error(GPTS_ENOMEM, "dpp_run: stash pool too small for this policy");
    if ((size_t)peak_act > issuer.act.free_ids.size()) return set_error(GPTS_ENOMEM, "dpp_run: boundary-activation pool too small for this policy");
  }
  for (int t = 0; t < n; ++t) {
    rc = issuer.issue(plan[t]);
    if (rc != GPTS_OK) return rc;
  }
  if (report) {
    report->n_tasks = n;
    report->peak_live_stash = issuer.W ? issuer.peak_fixed : issuer.stash.peak;
    report->peak_live_act = issuer.act.peak;
    report->stash_slot_bytes = stash_slot;
    report->act_slot_bytes = act_slot;
  }
  return GPTS_OK;
}

int gpt_dpp_run_ready(const gpt_dpp_job* job, const void* const* x_ready, const void* const* dy_ready,
                      double timeout_seconds, void* stream, gpt_dpp_task* order_out, int capacity,
                      gpt_dpp_report* report) {
  int rc = check_job(job, "dpp_run_ready: job is NULL");
  if (rc != GPTS_OK) return rc;
  rc = check_counts(job->policy, job->n_chunks, job->n_microbatches, "dpp_run_ready: unknown policy");
  if (rc != GPTS_OK) return rc;
  if (job->grad_pool) return set_error(GPTS_EINVAL, "dpp_run_ready: the per-chunk weight phase (grad_pool) is for gpt_dpp_run");
  const int C = job->n_chunks, M = job->n_microbatches, total = 2 * C * M;
  if (order_out && capacity < total) return set_error(GPTS_ENOMEM, "dpp_run_ready: order_out holds fewer than 2*chunks*microbatches entries");
  if (!(timeout_seconds > 0)) return set_error(GPTS_EINVAL, "dpp_run_ready: timeout_seconds must be > 0");
  const size_t stash_slot = gpt_dpp_stash_slot_bytes(job->chunks, C);
  const size_t act_slot = gpt_dpp_act_slot_bytes(&job->chunks[0].cfg);
  TaskIssuer issuer(job, stream, stash_slot, act_slot);
  // memory decides the width at run time: as many stashes as the pool holds (at most the policy's
  // own peak), and every micro-batch in flight may hold one boundary buffer per direction
  const size_t pool_slots = issuer.stash.free_ids.size();
  int allowance = job->max_live_stash;
  if (job->policy == GPT_DPP_BFC_BEST_EFFORT && allowance <= 0) allowance = pool_slots > (size_t)C * M ? C * M : (int)pool_slots;
  std::vector<gpt_dpp_task> plan((size_t)total);
  int peak_plan = 0;
  gpt_dpp_plan(job->policy, C, M, allowance, plan.data(), total, &peak_plan);
  const int slots = (size_t)peak_plan < pool_slots ? peak_plan : (int)pool_slots;
  if (slots < C) return set_error(GPTS_ENOMEM, "dpp_run_ready: the stash pool must hold at least one slot per chunk");
  // a micro-batch in flight holds at most one boundary buffer; one more is taken before one is returned
  if (C > 1 && issuer.act.free_ids.size() < (size_t)((M < slots ? M : slots) + 1))
    return set_error(GPTS_ENOMEM, "dpp_run_ready: boundary-activation pool too small (needs min(micro-batches, stash slots) + 1 buffers)");
  ReadySet rs(job->policy, C, M, allowance, slots);
  const auto t0 = std::chrono::steady_clock::now();
  int n = 0;
  while (!rs.finished()) {
    // what has arrived (an event that has not completed yet is queried again next time round)
    for (int i = 0; i < M; ++i) {
      if (!rs.x_ok[i]) rs.x_ok[i] = !x_ready || !x_ready[i] || hipEventQuery(static_cast<hipEvent_t>(const_cast<void*>(x_ready[i]))) == hipSuccess;
      if (!rs.dy_ok[i]) rs.dy_ok[i] = !dy_ready || !dy_ready[i] || hipEventQuery(static_cast<hipEvent_t>(const_cast<void*>(dy_ready[i]))) == hipSuccess;
    }
    (void)hipGetLastError();   // hipErrorNotReady from the queries is not an error
    const int t = rs.pick();
    if (t < 0) {
      // nothing can run until an input arrives: give up after the caller's limit, so that this
      // loop ends even if an event is never recorded
      const double waited = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
      if (waited > timeout_seconds) return set_error(GPTS_EHIP, "dpp_run_ready: inputs did not arrive within timeout_seconds");
      std::this_thread::yield();
      continue;
    }
    rc = issuer.issue(rs.plan[t]);
    if (rc != GPTS_OK) return rc;
    if (order_out) order_out[n] = rs.plan[t];
    ++n;
    rs.issue(t);
  }
  if (report) {
    report->n_tasks = n;
    report->peak_live_stash = issuer.stash.peak;
    report->peak_live_act = issuer.act.peak;
    report->stash_slot_bytes = stash_slot;
    report->act_slot_bytes = act_slot;
  }
  return GPTS_OK;
}

}  // extern "C"
