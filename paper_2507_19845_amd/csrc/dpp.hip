// Traversal of the (micro-batch, model chunk) task matrix: the depth-first, breadth-first
// and best-effort breadth-first orders of the paper's section 5.2 (MegaDPP, "parallel
// scheduler"), and a driver that issues the tasks of several chunks held by one GPU through
// the decoupled entry points.  Host code only: the arithmetic is in the stage kernels.
#include "../../include/gpt_stage.h"

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

}  // namespace

extern "C" {

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
  if (!job) return set_error(GPTS_EINVAL, "dpp_run: job is NULL");
  const int C = job->n_chunks, M = job->n_microbatches;
  if (C < 1 || M < 1 || C > (1 << 15) || M > (1 << 15)) return set_error(GPTS_EINVAL, "dpp_run: n_chunks and n_microbatches must be in [1, 32768]");
  if (!job->chunks || !job->x || !job->dy || !job->y || !job->dx || !job->dparams)
    return set_error(GPTS_EINVAL, "dpp_run: chunks / x / dy / y / dx / dparams array is NULL");
  for (int j = 0; j < C; ++j) {
    const int rc = gpt_stage_validate(&job->chunks[j].cfg);
    if (rc != GPTS_OK) return rc;
    const gpt_stage_cfg &a = job->chunks[0].cfg, &b = job->chunks[j].cfg;
    if (a.batch != b.batch || a.seq != b.seq || a.hidden != b.hidden || a.dtype != b.dtype)
      return set_error(GPTS_ESHAPE, "dpp_run: chunks must share batch, seq, hidden and dtype");
    if (!job->dparams[j]) return set_error(GPTS_EINVAL, "dpp_run: a dparams pointer is NULL");
  }
  for (int i = 0; i < M; ++i)
    if (!job->x[i] || !job->dy[i] || !job->y[i] || !job->dx[i])
      return set_error(GPTS_EINVAL, "dpp_run: an x / dy / y / dx pointer is NULL");

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

  Pool stash(job->stash_pool, stash_slot, job->stash_pool ? job->stash_pool_bytes : 0);
  Pool act(job->act_pool, act_slot, job->act_pool ? job->act_pool_bytes : 0);

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
    if ((size_t)peak_stash > stash.free_ids.size()) return set_error(GPTS_ENOMEM, "dpp_run: stash pool too small for this policy");
    if ((size_t)peak_act > act.free_ids.size()) return set_error(GPTS_ENOMEM, "dpp_run: boundary-activation pool too small for this policy");
  }

  std::vector<int> slot_of((size_t)C * M, -1);   // stash slot of task (i, j)
  std::vector<int> fwd_buf(M, -1), bwd_buf(M, -1);  // boundary buffer holding the latest output of micro-batch i
  std::vector<int> left(C, M);                   // backward tasks still to run per chunk
  for (int t = 0; t < n; ++t) {
    const gpt_dpp_task& k = plan[t];
    const int i = k.microbatch, j = k.chunk;
    if (k.phase == GPT_DPP_FWD) {
      const void* in = (j == 0) ? job->x[i] : act.at(fwd_buf[i]);
      int out_id = -1;
      void* out = job->y[i];
      if (j != C - 1) {
        out_id = act.take();
        out = act.at(out_id);
      }
      const int s = stash.take();
      slot_of[(size_t)i * C + j] = s;
      const int rc = gpt_stage_fwd_only(&job->chunks[j], in, stash.at(s), out, stream, nullptr);
      if (rc != GPTS_OK) return rc;
      if (j != 0) act.give(fwd_buf[i]);
      fwd_buf[i] = out_id;
    } else {
      const void* din = (j == C - 1) ? job->dy[i] : act.at(bwd_buf[i]);
      int out_id = -1;
      void* dout = job->dx[i];
      if (j != 0) {
        out_id = act.take();
        dout = act.at(out_id);
      }
      const int s = slot_of[(size_t)i * C + j];
      const int rc = gpt_stage_bwd_only(&job->chunks[j], stash.at(s), din, dout, job->dparams[j], stream, nullptr);
      if (rc != GPTS_OK) return rc;
      stash.give(s);
      if (j != C - 1) act.give(bwd_buf[i]);
      bwd_buf[i] = out_id;
      if (--left[j] == 0 && job->grad_ready && job->grad_ready[j]) {
        const hipError_t e = hipEventRecord(static_cast<hipEvent_t>(job->grad_ready[j]), static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return set_error(GPTS_EHIP, "dpp_run: recording a grad_ready event failed");
      }
    }
  }
  if (report) {
    report->n_tasks = n;
    report->peak_live_stash = stash.peak;
    report->peak_live_act = act.peak;
    report->stash_slot_bytes = stash_slot;
    report->act_slot_bytes = act_slot;
  }
  return GPTS_OK;
}

}  // extern "C"
