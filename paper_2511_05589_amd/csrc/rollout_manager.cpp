// Host-side rollout manager (Section 4): concurrency-controlled generation with a fixed
// pool of N' requests, early termination once B inputs have all of their N trajectories,
// buffering of partial trajectories with their per-stage log-prob pieces (Eq. 6), and
// prioritized resumption in the next stage.  No GPU code: this is the scheduling that
// decides which sequences the decode, re-prefill and log-prob kernels see at every step.
// The model is replaced by given response lengths, so a whole training run's schedule can
// be laid out (and its off-policy / re-prefill / utilisation figures read off) in
// microseconds.
//
// The schedule advances from one finish event to the next instead of token by token: with
// the active set fixed, every running trajectory grows by the same number of tokens, and
// nothing the schedule depends on changes in between.
#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <deque>
#include <vector>

#include "copris.h"

namespace {

struct Traj {
  int32_t target = 0;        // response length
  int32_t gen = 0;           // tokens generated so far
  int32_t gen_before = 0;    // ... of which before the current stage (off-policy once consumed)
  int32_t first_stage = -1;  // stage of the first generated token
  int32_t last_stage = -1;   // stage of the last generated token
  bool started = false;
};

}  // namespace

extern "C" int copris_rollout_schedule(const int32_t* prompt_len, const int32_t* resp_len,
                                       int n_inputs, int samples, int pool, int batch_inputs,
                                       int page_size, int max_stages, copris_stage_stats* stats,
                                       int32_t* batch_out, int* n_stages) {
  if (!n_stages) return COPRIS_EINVAL;
  *n_stages = 0;
  if (n_inputs < 0 || samples <= 0 || pool <= 0 || batch_inputs <= 0 || page_size <= 0 || max_stages < 0)
    return COPRIS_EINVAL;
  if (n_inputs > 0 && (!prompt_len || !resp_len)) return COPRIS_EINVAL;
  if (max_stages > 0 && (!stats || !batch_out)) return COPRIS_EINVAL;
  const int64_t n_traj = static_cast<int64_t>(n_inputs) * samples;
  if (n_traj >= (1ll << 31)) return COPRIS_EINVAL;
  for (int64_t t = 0; t < n_traj; ++t)
    if (resp_len[t] < 1) return COPRIS_EINVAL;
  for (int i = 0; i < n_inputs; ++i)
    if (prompt_len[i] < 0) return COPRIS_EINVAL;

  std::vector<Traj> tr(static_cast<size_t>(n_traj));
  for (int64_t t = 0; t < n_traj; ++t) tr[t].target = resp_len[t];
  std::vector<int32_t> finished_of(static_cast<size_t>(n_inputs), 0);   // finished trajectories per input
  std::vector<char> consumed(static_cast<size_t>(n_inputs), 0);
  int64_t fresh = 0;          // trajectories [fresh, n_traj) have not started (dispatch is input-major)
  int complete = 0;           // inputs with all trajectories finished, not yet consumed
  std::vector<int32_t> paused;   // unfinished started trajectories, ascending (the resume queue)
  std::vector<int32_t> active, next_active;

  auto pages_of = [&](int32_t t) {
    return (static_cast<int64_t>(prompt_len[t / samples]) + tr[t].gen + page_size - 1) / page_size;
  };

  for (int k = 0; k < max_stages; ++k) {
    copris_stage_stats st{};
    for (int32_t t : paused) tr[t].gen_before = tr[t].gen;
    size_t rpos = 0;
    active.clear();
    bool done = complete >= batch_inputs;
    while (!done) {
      while (static_cast<int>(active.size()) < pool) {
        int32_t t;
        if (rpos < paused.size()) {
          t = paused[rpos++];
          st.resumed += 1;
          st.reprefill_tokens += prompt_len[t / samples] + tr[t].gen;
        } else if (fresh < n_traj) {
          t = static_cast<int32_t>(fresh++);
          tr[t].started = true;
          tr[t].gen_before = 0;
        } else {
          break;
        }
        active.push_back(t);
      }
      if (active.empty()) break;
      // advance to the next finish event
      int32_t d = INT32_MAX;
      for (int32_t t : active) d = std::min(d, tr[t].target - tr[t].gen);
      st.steps += d;
      st.generated += static_cast<int64_t>(d) * static_cast<int64_t>(active.size());
      st.slot_steps_idle += static_cast<int64_t>(d) * (pool - static_cast<int64_t>(active.size()));
      int64_t pg = 0;
      next_active.clear();
      for (int32_t t : active) {
        if (tr[t].first_stage < 0) tr[t].first_stage = k;
        tr[t].last_stage = k;
        tr[t].gen += d;
        pg += pages_of(t);      // pages only grow inside the interval: its last step is the peak
        if (tr[t].gen >= tr[t].target) {
          const int i = t / samples;
          if (++finished_of[i] == samples) ++complete;
        } else {
          next_active.push_back(t);
        }
      }
      st.peak_pages = std::max<int64_t>(st.peak_pages, pg);
      active.swap(next_active);
      done = complete >= batch_inputs;
    }
    if (!done) break;    // inputs exhausted: this stage cannot complete a batch

    // the B complete inputs with the lowest indices form the training batch
    int taken = 0;
    for (int i = 0; i < n_inputs && taken < batch_inputs; ++i) {
      if (consumed[i] || finished_of[i] != samples) continue;
      consumed[i] = 1;
      batch_out[static_cast<size_t>(k) * batch_inputs + taken++] = i;
      for (int s = 0; s < samples; ++s) {
        const Traj& x = tr[static_cast<size_t>(i) * samples + s];
        // tokens of an earlier stage: everything, if the trajectory did not run in this
        // stage; else what it had when the stage began
        const int32_t stale = x.last_stage < k ? x.gen : x.gen_before;
        st.batch_tokens += x.gen;
        st.batch_offpolicy += stale;
        if (stale > 0) st.batch_traj_offpolicy += 1;
        if (x.gen > 0) st.max_staleness = std::max<int64_t>(st.max_staleness, k - x.first_stage);
      }
    }
    complete -= batch_inputs;
    // what stays in the buffer: unfinished trajectories (resumed first next stage, in
    // (input, sample) order) and finished ones of inputs that are not complete
    std::vector<int32_t> still;
    for (size_t r = rpos; r < paused.size(); ++r) still.push_back(paused[r]);   // never resumed this stage
    for (int32_t t : active) still.push_back(t);
    std::sort(still.begin(), still.end());
    paused.swap(still);
    st.paused = static_cast<int64_t>(paused.size());
    for (int i = 0; i < n_inputs; ++i)
      if (!consumed[i]) st.buffered_complete += finished_of[i];
    stats[k] = st;
    *n_stages = k + 1;
  }
  return COPRIS_OK;
}

// --------------------------------------------------------------------------
// The same rules, one decode step at a time, for a caller that runs the kernels
// between the calls.  The manager owns every decision of Section 4 - which trajectory
// sits in which pool slot, what is (re-)prefilled, when the stage stops, which inputs
// leave as the batch - and the KV page allocator; the caller owns the device.
// --------------------------------------------------------------------------
struct copris_rollout {
  int n_inputs = 0, samples = 0, pool = 0, batch_inputs = 0, page_size = 0, max_pages = 0;
  std::vector<int32_t> prompt;
  std::vector<Traj> tr;
  std::vector<int32_t> finished_of;
  std::vector<char> consumed;
  int64_t fresh = 0;                 // trajectories [fresh, n_traj) have not started
  int complete = 0;                  // inputs with every trajectory finished, not yet consumed
  std::vector<int32_t> paused;       // resume queue of the stage, ascending
  size_t rpos = 0;                   // ... next one to resume
  int stage = 0;
  bool in_stage = false;
  copris_stage_stats st{};
  // pool slots and their KV pages
  std::vector<int32_t> slot_traj;    // occupant of every slot (-1: idle)
  std::vector<int32_t> slot_npages;
  std::vector<int32_t> table;        // [pool][max_pages] physical page of every held page
  std::deque<int32_t> free_pages;
  int64_t pages_held = 0;
  std::vector<int32_t> vacated;      // slots emptied since the last plan
  // the plan handed out by next_step (valid until the next call)
  std::vector<int32_t> plan_slot_traj, entered, finishing, cmds_slot, cmds_page, cmds;

  int64_t n_traj() const { return static_cast<int64_t>(n_inputs) * samples; }
  int32_t prompt_of(int32_t t) const { return prompt[t / samples]; }

  void release_slot(int slot) {
    int32_t* row = table.data() + static_cast<size_t>(slot) * max_pages;
    for (int p = 0; p < slot_npages[slot]; ++p) free_pages.push_back(row[p]);
    pages_held -= slot_npages[slot];
    slot_npages[slot] = 0;
    slot_traj[slot] = -1;
    vacated.push_back(slot);
  }
  void finish(int slot) {
    const int32_t t = slot_traj[slot];
    release_slot(slot);
    if (++finished_of[t / samples] == samples) ++complete;
  }
};

extern "C" {

int copris_rollout_create(const int32_t* prompt_len, const int32_t* resp_len, int n_inputs,
                          int samples, int pool, int batch_inputs, int page_size, int64_t num_pages,
                          const int32_t* page_order, copris_rollout** out) {
  if (!out) return COPRIS_EINVAL;
  *out = nullptr;
  if (n_inputs <= 0 || samples <= 0 || pool <= 0 || batch_inputs <= 0 || page_size <= 0 ||
      !prompt_len || !resp_len)
    return COPRIS_EINVAL;
  const int64_t n_traj = static_cast<int64_t>(n_inputs) * samples;
  if (n_traj >= (1ll << 31)) return COPRIS_EINVAL;
  int64_t longest = 1;
  for (int i = 0; i < n_inputs; ++i) {
    if (prompt_len[i] < 0) return COPRIS_EINVAL;
    for (int s = 0; s < samples; ++s) {
      const int32_t r = resp_len[static_cast<size_t>(i) * samples + s];
      if (r < 1) return COPRIS_EINVAL;
      longest = std::max<int64_t>(longest, static_cast<int64_t>(prompt_len[i]) + r);
    }
  }
  const int64_t max_pages = (longest + page_size - 1) / page_size;
  // a request can always grow to its full length: no preemption, no KV recomputation
  if (max_pages >= (1ll << 31) || num_pages < static_cast<int64_t>(pool) * max_pages ||
      num_pages >= (1ll << 31))
    return COPRIS_EINVAL;
  if (page_order) {   // must be a permutation of 0 .. num_pages-1
    std::vector<char> seen(static_cast<size_t>(num_pages), 0);
    for (int64_t p = 0; p < num_pages; ++p) {
      const int32_t x = page_order[p];
      if (x < 0 || x >= num_pages || seen[x]) return COPRIS_EINVAL;
      seen[x] = 1;
    }
  }
  copris_rollout* h = new copris_rollout();
  h->n_inputs = n_inputs;
  h->samples = samples;
  h->pool = pool;
  h->batch_inputs = batch_inputs;
  h->page_size = page_size;
  h->max_pages = static_cast<int>(max_pages);
  h->prompt.assign(prompt_len, prompt_len + n_inputs);
  h->tr.resize(static_cast<size_t>(n_traj));
  for (int64_t t = 0; t < n_traj; ++t) h->tr[t].target = resp_len[t];
  h->finished_of.assign(static_cast<size_t>(n_inputs), 0);
  h->consumed.assign(static_cast<size_t>(n_inputs), 0);
  h->slot_traj.assign(static_cast<size_t>(pool), -1);
  h->slot_npages.assign(static_cast<size_t>(pool), 0);
  h->table.assign(static_cast<size_t>(pool) * h->max_pages, 0);
  for (int64_t p = 0; p < num_pages; ++p)
    h->free_pages.push_back(page_order ? page_order[p] : static_cast<int32_t>(p));
  h->plan_slot_traj.assign(static_cast<size_t>(pool), -1);
  *out = h;
  return COPRIS_OK;
}

void copris_rollout_destroy(copris_rollout* h) { delete h; }

int copris_rollout_max_pages(const copris_rollout* h) { return h ? h->max_pages : 0; }

int64_t copris_rollout_free_pages(const copris_rollout* h) {
  return h ? static_cast<int64_t>(h->free_pages.size()) : 0;
}

int copris_rollout_begin_stage(copris_rollout* h) {
  if (!h || h->in_stage) return COPRIS_EINVAL;
  h->in_stage = true;
  h->st = copris_stage_stats{};
  h->rpos = 0;
  for (int32_t t : h->paused) h->tr[t].gen_before = h->tr[t].gen;
  return h->stage;
}

int copris_rollout_next_step(copris_rollout* h, copris_rollout_plan* plan) {
  if (!h || !plan || !h->in_stage) return COPRIS_EINVAL;
  *plan = copris_rollout_plan{};
  plan->stage = h->stage;
  plan->block_table = h->table.data();
  if (h->complete >= h->batch_inputs) return COPRIS_ROLLOUT_STAGE_END;
  const int k = h->stage, P = h->page_size;
  h->entered.clear();
  h->finishing.clear();
  h->cmds_slot.clear();
  h->cmds_page.clear();
  std::vector<char> refilled(static_cast<size_t>(h->pool), 0);
  // every idle slot takes the next request: paused trajectories first, then new ones
  for (int slot = 0; slot < h->pool; ++slot) {
    if (h->slot_traj[slot] >= 0) continue;
    int32_t t, resumed = 0;
    if (h->rpos < h->paused.size()) {
      t = h->paused[h->rpos++];
      resumed = 1;
      h->st.resumed += 1;
      h->st.reprefill_tokens += h->prompt_of(t) + h->tr[t].gen;
    } else if (h->fresh < h->n_traj()) {
      t = static_cast<int32_t>(h->fresh++);
      h->tr[t].started = true;
      h->tr[t].gen_before = 0;
    } else {
      break;
    }
    h->slot_traj[slot] = t;
    refilled[slot] = 1;
    const int32_t have = h->prompt_of(t) + h->tr[t].gen;   // tokens to (re-)prefill
    const int32_t e[4] = {slot, t, have, resumed};
    h->entered.insert(h->entered.end(), e, e + 4);
    const int32_t c[4] = {slot, t, have + 1, h->tr[t].gen};
    h->cmds_slot.insert(h->cmds_slot.end(), c, c + 4);
  }
  for (int32_t slot : h->vacated) {
    if (refilled[slot]) continue;
    const int32_t c[4] = {slot, -1, 0, 0};
    h->cmds_slot.insert(h->cmds_slot.end(), c, c + 4);
  }
  h->vacated.clear();
  int n_active = 0;
  for (int slot = 0; slot < h->pool; ++slot) {
    const int32_t t = h->slot_traj[slot];
    h->plan_slot_traj[slot] = t;
    if (t < 0) continue;
    ++n_active;
    // pages for the context of this step: what is cached plus the new position
    const int need = (h->prompt_of(t) + h->tr[t].gen + 1 + P - 1) / P;
    int32_t* row = h->table.data() + static_cast<size_t>(slot) * h->max_pages;
    while (h->slot_npages[slot] < need) {
      const int32_t page = h->free_pages.front();   // create() made sure there always is one
      h->free_pages.pop_front();
      const int32_t c[3] = {slot, h->slot_npages[slot], page};
      h->cmds_page.insert(h->cmds_page.end(), c, c + 3);
      row[h->slot_npages[slot]++] = page;
      ++h->pages_held;
    }
  }
  h->cmds = h->cmds_slot;
  h->cmds.insert(h->cmds.end(), h->cmds_page.begin(), h->cmds_page.end());
  plan->n_active = n_active;
  plan->n_entered = static_cast<int32_t>(h->entered.size() / 4);
  plan->n_slot_cmds = static_cast<int32_t>(h->cmds_slot.size() / 4);
  plan->n_page_cmds = static_cast<int32_t>(h->cmds_page.size() / 3);
  plan->slot_traj = h->plan_slot_traj.data();
  plan->entered = h->entered.data();
  plan->cmds = h->cmds.data();
  if (n_active == 0) return COPRIS_ROLLOUT_EXHAUSTED;
  // the step: every running request generates one token
  h->st.steps += 1;
  h->st.generated += n_active;
  h->st.slot_steps_idle += h->pool - n_active;
  h->st.peak_pages = std::max<int64_t>(h->st.peak_pages, h->pages_held);
  for (int slot = 0; slot < h->pool; ++slot) {
    const int32_t t = h->slot_traj[slot];
    if (t < 0) continue;
    Traj& x = h->tr[t];
    if (x.first_stage < 0) x.first_stage = k;
    x.last_stage = k;
    if (++x.gen >= x.target) {
      h->finishing.push_back(slot);
      h->finish(slot);
    }
  }
  plan->n_finishing = static_cast<int32_t>(h->finishing.size());
  plan->finishing = h->finishing.data();
  return COPRIS_ROLLOUT_STEP;
}

int copris_rollout_stop(copris_rollout* h, const int32_t* slots, int n) {
  if (!h || !h->in_stage || n < 0 || (n > 0 && !slots)) return COPRIS_EINVAL;
  for (int j = 0; j < n; ++j)
    if (slots[j] < 0 || slots[j] >= h->pool) return COPRIS_EINVAL;
  for (int j = 0; j < n; ++j) {
    const int slot = slots[j];
    const int32_t t = h->slot_traj[slot];
    if (t < 0) continue;             // finished by its length in the same step
    h->tr[t].target = h->tr[t].gen;
    h->finish(slot);
  }
  return COPRIS_OK;
}

int copris_rollout_end_stage(copris_rollout* h, copris_stage_stats* stats, int32_t* batch_inputs_out,
                             int32_t* batch_traj_out) {
  if (!h || !h->in_stage || !stats || !batch_inputs_out || !batch_traj_out) return COPRIS_EINVAL;
  if (h->complete < h->batch_inputs) return COPRIS_EINVAL;
  const int k = h->stage;
  copris_stage_stats& st = h->st;
  // running requests are paused: their pages are dropped (the next policy invalidates them)
  std::vector<int32_t> still(h->paused.begin() + static_cast<ptrdiff_t>(h->rpos), h->paused.end());
  for (int slot = 0; slot < h->pool; ++slot) {
    if (h->slot_traj[slot] < 0) continue;
    still.push_back(h->slot_traj[slot]);
    h->release_slot(slot);
  }
  std::sort(still.begin(), still.end());
  h->paused.swap(still);
  // the complete inputs with the lowest indices leave as the training batch
  int taken = 0;
  for (int i = 0; i < h->n_inputs && taken < h->batch_inputs; ++i) {
    if (h->consumed[i] || h->finished_of[i] != h->samples) continue;
    h->consumed[i] = 1;
    batch_inputs_out[taken] = i;
    for (int s = 0; s < h->samples; ++s) {
      const int32_t t = i * h->samples + s;
      const Traj& x = h->tr[t];
      const int32_t stale = x.last_stage < k ? x.gen : x.gen_before;
      int32_t* row = batch_traj_out + (static_cast<size_t>(taken) * h->samples + s) * 3;
      row[0] = t;
      row[1] = x.gen;
      row[2] = stale;
      st.batch_tokens += x.gen;
      st.batch_offpolicy += stale;
      if (stale > 0) st.batch_traj_offpolicy += 1;
      if (x.gen > 0) st.max_staleness = std::max<int64_t>(st.max_staleness, k - x.first_stage);
    }
    ++taken;
  }
  h->complete -= h->batch_inputs;
  st.paused = static_cast<int64_t>(h->paused.size());
  for (int i = 0; i < h->n_inputs; ++i)
    if (!h->consumed[i]) st.buffered_complete += h->finished_of[i];
  *stats = st;
  h->in_stage = false;
  h->stage = k + 1;
  return COPRIS_OK;
}

}  // extern "C"
