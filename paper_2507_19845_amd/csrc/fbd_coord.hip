// Host-side simulation of the communication coordinator of the paper's section 4.2
// (MegaFBD, "communication coordinator"): several training threads (virtual ranks) share a
// control thread per GPU; a collective is started only once every rank of its group has
// posted the same request.  Each control thread keeps a table of one bit vector per
// communication group, one bit per virtual rank, flattened to one array; the tables are
// aligned by a bitwise-OR all-reduce; a group is ready when its vector equals the expected
// mask; ready collectives run in ascending group order.  No GPU code in this file.
#include "../../include/gpt_stage.h"

#include <stdint.h>

#include <deque>
#include <new>
#include <vector>

#include "kernels.hpp"

using gpts::set_error;

namespace {

struct Coord {
  int n_ranks, n_groups, n_control, words;   // words: 64-bit words per bit vector
  std::vector<std::vector<int>> members;     // per group, ascending
  std::vector<int> control_of;               // per rank
  std::vector<uint64_t> expected;            // [group][word]
  std::vector<std::vector<uint64_t>> table;  // per control thread: flattened [group][word]

  uint64_t* vec(int control, int g) { return table[control].data() + (size_t)g * words; }
  bool ready_on(int control, int g) {
    const uint64_t* v = vec(control, g);
    for (int w = 0; w < words; ++w)
      if (v[w] != expected[(size_t)g * words + w]) return false;
    return true;
  }
  void align() {   // bitwise-OR all-reduce of the flattened tables
    const size_t n = (size_t)n_groups * words;
    std::vector<uint64_t> acc(n, 0);
    for (int c = 0; c < n_control; ++c)
      for (size_t i = 0; i < n; ++i) acc[i] |= table[c][i];
    for (int c = 0; c < n_control; ++c) table[c] = acc;
  }
  void clear_group(int g) {
    for (int c = 0; c < n_control; ++c)
      for (int w = 0; w < words; ++w) vec(c, g)[w] = 0;
  }
  bool member(int g, int r) const {
    return (expected[(size_t)g * words + r / 64] >> (r % 64)) & 1u;
  }
};

Coord* as_coord(void* h) { return static_cast<Coord*>(h); }

}  // namespace

extern "C" {

int gpt_fbd_coord_create(int n_ranks, int n_groups, const int32_t* group_start, const int32_t* group_members,
                         int n_control, const int32_t* control_of_rank, void** coord) {
  if (!coord || !group_start || !group_members || !control_of_rank)
    return set_error(GPTS_EINVAL, "fbd_coord_create: NULL argument");
  if (n_ranks < 1 || n_groups < 1 || n_control < 1 || n_ranks > (1 << 16) || n_groups > (1 << 16))
    return set_error(GPTS_EINVAL, "fbd_coord_create: counts out of range");
  Coord* c = new (std::nothrow) Coord;
  if (!c) return set_error(GPTS_ENOMEM, "fbd_coord_create: out of host memory");
  c->n_ranks = n_ranks;
  c->n_groups = n_groups;
  c->n_control = n_control;
  c->words = (n_ranks + 63) / 64;
  c->members.resize(n_groups);
  c->expected.assign((size_t)n_groups * c->words, 0);
  for (int g = 0; g < n_groups; ++g) {
    if (group_start[g + 1] <= group_start[g]) { delete c; return set_error(GPTS_EINVAL, "fbd_coord_create: empty group"); }
    for (int k = group_start[g]; k < group_start[g + 1]; ++k) {
      const int r = group_members[k];
      if (r < 0 || r >= n_ranks || c->member(g, r)) { delete c; return set_error(GPTS_EINVAL, "fbd_coord_create: bad or repeated group member"); }
      c->members[g].push_back(r);
      c->expected[(size_t)g * c->words + r / 64] |= (uint64_t)1 << (r % 64);
    }
  }
  c->control_of.assign(control_of_rank, control_of_rank + n_ranks);
  for (int r = 0; r < n_ranks; ++r)
    if (c->control_of[r] < 0 || c->control_of[r] >= n_control) { delete c; return set_error(GPTS_EINVAL, "fbd_coord_create: control thread index out of range"); }
  c->table.assign(n_control, std::vector<uint64_t>((size_t)n_groups * c->words, 0));
  *coord = c;
  return GPTS_OK;
}

int gpt_fbd_coord_destroy(void* coord) {
  delete as_coord(coord);
  return GPTS_OK;
}

int gpt_fbd_coord_expected(void* coord, int group, char* bits) {
  Coord* c = as_coord(coord);
  if (!c || !bits || group < 0 || group >= c->n_groups) return set_error(GPTS_EINVAL, "fbd_coord_expected: bad argument");
  for (int r = 0; r < c->n_ranks; ++r) bits[r] = c->member(group, r) ? '1' : '0';
  bits[c->n_ranks] = 0;
  return GPTS_OK;
}

int gpt_fbd_coord_register(void* coord, int rank, int group) {
  Coord* c = as_coord(coord);
  if (!c || rank < 0 || rank >= c->n_ranks || group < 0 || group >= c->n_groups)
    return set_error(GPTS_EINVAL, "fbd_coord_register: bad argument");
  if (!c->member(group, rank)) return set_error(GPTS_EINVAL, "fbd_coord_register: rank is not a member of the group");
  c->vec(c->control_of[rank], group)[rank / 64] |= (uint64_t)1 << (rank % 64);
  return GPTS_OK;
}

int gpt_fbd_coord_align(void* coord) {
  Coord* c = as_coord(coord);
  if (!c) return set_error(GPTS_EINVAL, "fbd_coord_align: NULL");
  c->align();
  return GPTS_OK;
}

int gpt_fbd_coord_ready(void* coord, int control, int32_t* groups, int capacity) {
  Coord* c = as_coord(coord);
  if (!c || control < 0 || control >= c->n_control || (!groups && capacity > 0))
    return set_error(GPTS_EINVAL, "fbd_coord_ready: bad argument");
  int n = 0;
  for (int g = 0; g < c->n_groups; ++g)
    if (c->ready_on(control, g)) {
      if (n >= capacity) return set_error(GPTS_ENOMEM, "fbd_coord_ready: groups array too small");
      groups[n++] = g;
    }
  return n;
}

int gpt_fbd_coord_execute(void* coord, int32_t* groups, int capacity) {
  Coord* c = as_coord(coord);
  if (!c || (!groups && capacity > 0)) return set_error(GPTS_EINVAL, "fbd_coord_execute: bad argument");
  // after alignment every control thread holds the same table, so every one of them
  // finds the same ready set and walks it in the same (ascending) order
  int n = 0;
  for (int g = 0; g < c->n_groups; ++g)
    if (c->ready_on(0, g)) {
      for (int k = 1; k < c->n_control; ++k)
        if (!c->ready_on(k, g)) return set_error(GPTS_EINVAL, "fbd_coord_execute: tables differ, call align first");
      if (n >= capacity) return set_error(GPTS_ENOMEM, "fbd_coord_execute: groups array too small");
      groups[n++] = g;
    }
  for (int i = 0; i < n; ++i) c->clear_group(groups[i]);
  return n;
}

int gpt_fbd_coord_simulate(void* coord, const int32_t* prog_start, const int32_t* prog, int verify,
                           int32_t* log, int log_capacity, int32_t* n_executed, int32_t* deadlocked) {
  Coord* c = as_coord(coord);
  if (!c || !prog_start || !prog || !n_executed || !deadlocked || (!log && log_capacity > 0))
    return set_error(GPTS_EINVAL, "fbd_coord_simulate: NULL argument");
  const int R = c->n_ranks;
  for (int r = 0; r < R; ++r)
    for (int k = prog_start[r]; k < prog_start[r + 1]; ++k)
      if (prog[k] < 0 || prog[k] >= c->n_groups || !c->member(prog[k], r))
        return set_error(GPTS_EINVAL, "fbd_coord_simulate: a program names a group its rank is not in");
  for (auto& t : c->table) t.assign(t.size(), 0);
  std::vector<int> pc(R);
  for (int r = 0; r < R; ++r) pc[r] = prog_start[r];
  int n = 0;
  *deadlocked = 0;
  auto put = [&](int g) -> bool {
    if (n >= log_capacity) return false;
    log[n++] = g;
    return true;
  };
  if (verify) {
    std::vector<char> waiting(R, 0);
    std::vector<int32_t> ready(c->n_groups);
    for (;;) {
      bool pending = false;
      for (int r = 0; r < R; ++r) {
        if (!waiting[r] && pc[r] < prog_start[r + 1]) {
          gpt_fbd_coord_register(c, r, prog[pc[r]]);   // step 1
          waiting[r] = 1;
        }
        pending |= waiting[r] != 0;
      }
      if (!pending) break;
      c->align();                                       // step 2
      const int nr = gpt_fbd_coord_execute(c, ready.data(), c->n_groups);   // steps 3 and 4
      if (nr < 0) return nr;
      if (nr == 0) { *deadlocked = 1; break; }
      for (int i = 0; i < nr; ++i) {
        if (!put(ready[i])) return set_error(GPTS_ENOMEM, "fbd_coord_simulate: log too small");
        for (int r : c->members[ready[i]]) { ++pc[r]; waiting[r] = 0; }
      }
    }
  } else {
    // No verification: a control thread starts the oldest request it holds and stays busy
    // with it until the collective completes, i.e. until every member's request for that
    // group is the one its own control thread has started.
    std::vector<std::deque<int>> queue(c->n_control);   // ranks with a posted, unstarted request
    std::vector<int> busy(c->n_control, -1);            // rank whose request the thread has started
    std::vector<char> posted(R, 0);
    for (;;) {
      bool progress = false;
      for (int r = 0; r < R; ++r)
        if (!posted[r] && pc[r] < prog_start[r + 1]) { queue[c->control_of[r]].push_back(r); posted[r] = 1; progress = true; }
      for (int k = 0; k < c->n_control; ++k)
        if (busy[k] < 0 && !queue[k].empty()) { busy[k] = queue[k].front(); queue[k].pop_front(); progress = true; }
      for (int g = 0; g < c->n_groups; ++g) {
        bool all = true;
        for (int r : c->members[g])
          if (busy[c->control_of[r]] != r || prog[pc[r]] != g) { all = false; break; }
        if (!all) continue;
        if (!put(g)) return set_error(GPTS_ENOMEM, "fbd_coord_simulate: log too small");
        for (int r : c->members[g]) { busy[c->control_of[r]] = -1; ++pc[r]; posted[r] = 0; }
        progress = true;
      }
      bool pending = false;
      for (int r = 0; r < R; ++r) pending |= pc[r] < prog_start[r + 1];
      if (!pending) break;
      if (!progress) { *deadlocked = 1; break; }
    }
  }
  *n_executed = n;
  return GPTS_OK;
}

}  // extern "C"
