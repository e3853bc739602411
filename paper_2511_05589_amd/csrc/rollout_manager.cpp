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
#include <cstdint>
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
