// Host-side cycle scheduler for DMTD decoding (paper Sec. 2.2, Fig. 3, Eq. 7).
// Pure host code: no HIP.  It decides, for each decode call, which steps run (one full
// step at a cycle boundary, then late-only steps), how many rows the full step's front
// layers carry (the pending in-cycle tokens plus the newest token), and keeps the
// counters and the schedule trace that the tests compare with the paper.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace dmtd {

struct Step {
  bool full;   // true: front layers (refill rows + newest) then late layers; false: late layers only
  int rows;    // rows per sequence in the front layers (full step), 1 otherwise
  int pos;     // absolute position of the token-emitting row
};

struct Sched {
  int n_layers = 0;
  int max_seq_len = 0;
  int n_tok = 0;      // tokens that have entered the late layers' caches
  int n_front = 0;    // tokens that have entered the front layers' caches
  int phase = 0;      // tokens of the current cycle already emitted (prefill's token counts for cycle 1)
  int n_late_in_use = 0;
  int n_early = 0;    // ExDy variant: encoding layers the in-cycle tokens pass in their own step (0 = plain method)
  int pass_no = 0;
  int64_t gen_layer_visits = 0, refill_layer_visits = 0, n_emitted = 0, n_full_steps = 0;
  std::vector<int32_t> trace;   // records of 4: pass, group (0 front or thinking / 1 late / 2 encoding), first position, count

  void reset() {
    n_tok = n_front = phase = n_late_in_use = pass_no = 0;   // n_early is a setting: it survives a reset
    gen_layer_visits = refill_layer_visits = n_emitted = n_full_steps = 0;
    trace.clear();
  }

  void record(int group, int first, int count) {
    trace.push_back(pass_no); trace.push_back(group); trace.push_back(first); trace.push_back(count);
  }

  void note_prefill(int prompt_len, int n_late) {
    pass_no = 1;
    record(0, 0, prompt_len);
    record(1, 0, prompt_len);
    n_tok = n_front = prompt_len;
    phase = 1;
    n_late_in_use = n_late;   // 0 = not fixed yet
  }

  // Plan the steps of one decode call without changing state.  Returns false with a
  // reason and an error class (1 = invalid argument, 2 = state, 3 = capacity).
  bool plan(int tau, int n_late, int max_new, int max_rows, std::vector<Step>& steps, int& err, std::string& why) const {
    steps.clear();
    if (n_tok == 0) { err = 2; why = "decode before prefill"; return false; }
    if (tau < 1) { err = 1; why = "tau must be >= 1"; return false; }
    if (n_late < 1 || n_late > n_layers) { err = 1; why = "n_late must be in [1, n_layers]"; return false; }
    if (n_early + n_late > n_layers) { err = 1; why = "n_early + n_late exceeds the number of layers"; return false; }
    if (n_late_in_use != 0 && n_late_in_use != n_late && n_front != n_tok) {
      err = 2; why = "n_late changed while tokens await refill"; return false;
    }
    const long cap = max_new > 0 ? max_new : (1L << 30);
    int t = n_tok, f = n_front, ph = phase;
    if (ph >= tau || ph == 0) {
      steps.push_back({true, t - f + 1, t});
      t += 1; f = t; ph = 1;
    }
    while (ph < tau && (long)steps.size() < cap) {
      steps.push_back({false, 1, t});
      t += 1; ph += 1;
    }
    if (t > max_seq_len) { err = 3; why = "sequence would exceed max_seq_len"; return false; }
    for (const Step& s : steps)
      if (s.rows > max_rows) { err = 3; why = "more pending refill rows than the workspace holds"; return false; }
    return true;
  }

  void commit(const std::vector<Step>& steps, int n_late) {
    const int F = n_layers - n_late;
    for (const Step& s : steps) {
      pass_no += 1;
      if (n_early > 0) record(2, s.pos, 1);          // the step's own token through the encoding layers
      if (s.full) {
        if (F - n_early > 0) record(0, n_front, s.rows);
        record(1, s.pos, 1);
        gen_layer_visits += n_layers;
        refill_layer_visits += (int64_t)(s.rows - 1) * (F - n_early);
        n_tok += 1; n_front = n_tok; phase = 1;
        n_full_steps += 1;
      } else {
        record(1, s.pos, 1);
        gen_layer_visits += n_early + n_late;
        n_tok += 1; phase += 1;
      }
      n_emitted += 1;
    }
    n_late_in_use = n_late;
  }
};

}  // namespace dmtd
