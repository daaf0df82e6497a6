// Host-side integer schedules (Section 3.2 and Algorithms 1-2 of the DistFlashAttn paper),
// in closed 0-indexed form.  At step t >= 1 worker w either has an earlier chunk at
// distance t (w >= t: OWN pair (w, w-t)), or it has run out of own work and lends its
// keys/values to the worker P-t positions later (HELP pair (w-t+P, w)), except when
// 2t == P, where that pair is the late worker's own pair of the same step.
#include "dfa.h"

static void fill(dfa_step* s, int t, int kind, int qc, int kc, int to, int from) {
  s->t = t; s->kind = kind; s->q_chunk = qc; s->kv_chunk = kc; s->send_to = to; s->recv_from = from;
}

extern "C" int dfa_schedule_mode(int32_t mode, int32_t P, int32_t w, dfa_step* out, int32_t cap) {
  if (P < 1 || w < 0 || w >= P || cap < 0) return DFA_ERR_ARG;
  if (mode != DFA_SCHED_BALANCED && mode != DFA_SCHED_RING) return DFA_ERR_ARG;
  if (cap > 0 && out == nullptr) return DFA_ERR_NULL;
  const int n = (mode == DFA_SCHED_BALANCED) ? 1 + P / 2 : P;
  for (int t = 0; t < n && t < cap; ++t) {
    dfa_step* s = &out[t];
    if (t == 0) { fill(s, 0, DFA_STEP_DIAG, w, w, -1, -1); continue; }
    if (mode == DFA_SCHED_RING) {
      if (t <= w) fill(s, t, DFA_STEP_OWN, w, w - t, -1, -1);
      else fill(s, t, DFA_STEP_IDLE, -1, -1, -1, -1);
      continue;
    }
    const bool coincide = (2 * t == P);
    if (w >= t) {
      // a helper exists for me iff the chunk P-t positions earlier exists: w - (P - t) >= 0
      const int helper = w + t - P;
      fill(s, t, DFA_STEP_OWN, w, w - t, -1, (!coincide && helper >= 0) ? helper : -1);
    } else if (!coincide) {
      const int owner = w - t + P;
      fill(s, t, DFA_STEP_HELP, owner, w, owner, -1);
    } else {
      fill(s, t, DFA_STEP_IDLE, -1, -1, -1, -1);
    }
  }
  return n;
}

// Appendix on sparse patterns, local sliding windows: only the end of the vanilla loop changes.
extern "C" int dfa_schedule_window(int32_t P, int32_t w, int32_t window_chunks, dfa_step* out, int32_t cap) {
  if (P < 1 || w < 0 || w >= P || cap < 0 || window_chunks < 0) return DFA_ERR_ARG;
  if (cap > 0 && out == nullptr) return DFA_ERR_NULL;
  const int n = 1 + (window_chunks < P - 1 ? window_chunks : P - 1);
  for (int t = 0; t < n && t < cap; ++t) {
    if (t == 0) fill(&out[t], 0, DFA_STEP_DIAG, w, w, -1, -1);
    else if (t <= w) fill(&out[t], t, DFA_STEP_OWN, w, w - t, -1, -1);
    else fill(&out[t], t, DFA_STEP_IDLE, -1, -1, -1, -1);
  }
  return n;
}

extern "C" int dfa_schedule(int32_t P, int32_t w, dfa_step* out, int32_t cap) {
  return dfa_schedule_mode(DFA_SCHED_BALANCED, P, w, out, cap);
}
