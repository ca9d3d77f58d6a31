// Measurement hook for benchmarks (off by default): HIP-event timing of the library's launches,
// by kind.  Between prof_begin and prof_end every launch site that calls prof_mark_begin /
// prof_mark_end is bracketed by a pair of events recorded on the launch stream; prof_end waits for
// the events and adds up, per kind, the elapsed time, the number of launches and the work the
// launch sites declared (floating-point operations for the GEMM kind, algorithmic bytes for the
// bandwidth-bound kinds).  These are the only functions of the library that create HIP objects
// or synchronise.  Not thread-safe.
#include "common.h"

namespace mixlora {

namespace {
struct Prof {
  bool on = false;
  int cap = 0, used = 0;
  hipEvent_t *beg = nullptr, *end = nullptr;
  int *kind = nullptr;
  double *work = nullptr;
  double ms[PROF_KINDS] = {}, work_total[PROF_KINDS] = {};
  int launches[PROF_KINDS] = {};
} g_prof;
}  // namespace

bool prof_on() { return g_prof.on; }

int prof_begin(int max_launches) {
  if (g_prof.on || max_launches < 1) return -1;
  if (g_prof.cap < max_launches) {
    hipEvent_t *b = new hipEvent_t[max_launches], *e = new hipEvent_t[max_launches];
    for (int i = 0; i < max_launches; i++)
      if (hipEventCreate(&b[i]) != hipSuccess || hipEventCreate(&e[i]) != hipSuccess) return -1;
    // an earlier, smaller pool is kept alive until process exit
    g_prof.beg = b;
    g_prof.end = e;
    g_prof.kind = new int[max_launches];
    g_prof.work = new double[max_launches];
    g_prof.cap = max_launches;
  }
  g_prof.used = 0;
  g_prof.on = true;
  return 0;
}

int prof_mark_begin(int kind, hipStream_t st) {
  if (!g_prof.on || g_prof.used >= g_prof.cap || kind < 0 || kind >= PROF_KINDS) return -1;
  const int slot = g_prof.used++;
  g_prof.kind[slot] = kind;
  g_prof.work[slot] = 0.0;
  (void)hipEventRecord(g_prof.beg[slot], st);
  return slot;
}

void prof_mark_end(int slot, hipStream_t st, double work) {
  if (slot < 0) return;
  g_prof.work[slot] = work;
  (void)hipEventRecord(g_prof.end[slot], st);
}

int prof_end() {
  if (!g_prof.on) return -1;
  g_prof.on = false;
  for (int k = 0; k < PROF_KINDS; k++) {
    g_prof.ms[k] = g_prof.work_total[k] = 0.0;
    g_prof.launches[k] = 0;
  }
  for (int i = 0; i < g_prof.used; i++) {
    if (hipEventSynchronize(g_prof.end[i]) != hipSuccess) return -1;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_prof.beg[i], g_prof.end[i]) != hipSuccess) return -1;
    const int k = g_prof.kind[i];
    g_prof.ms[k] += t;
    g_prof.work_total[k] += g_prof.work[i];
    g_prof.launches[k]++;
  }
  return 0;
}

int prof_kind(int kind, double *ms_total, int *launches, double *work_total) {
  if (kind < 0 || kind >= PROF_KINDS) return -1;
  *ms_total = g_prof.ms[kind];
  *launches = g_prof.launches[kind];
  *work_total = g_prof.work_total[kind];
  return 0;
}

}  // namespace mixlora
