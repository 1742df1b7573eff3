#include "prof.h"

#include <stdint.h>

#include <vector>

namespace mg {
namespace {
struct Rec { int cls; double flops, bytes; };
bool g_on = false;
std::vector<hipEvent_t> g_ev;      // 2 per record
std::vector<Rec> g_rec;
size_t g_used = 0;
bool g_overflow = false;
}  // namespace

bool prof_enabled() { return g_on; }

void prof_begin(int cls, double flops, double bytes, hipStream_t st) {
  if (g_used >= g_rec.size()) { g_overflow = true; return; }
  g_rec[g_used] = Rec{cls, flops, bytes};
  (void)hipEventRecord(g_ev[2 * g_used], st);
}

void prof_end(hipStream_t st) {
  if (g_used >= g_rec.size()) return;
  (void)hipEventRecord(g_ev[2 * g_used + 1], st);
  ++g_used;
}

}  // namespace mg

extern "C" {

// max_records > 0: create the event pool and start recording; 0: stop and destroy it.
int mgrit_profile_enable(int max_records) {
  using namespace mg;
  for (hipEvent_t e : g_ev) (void)hipEventDestroy(e);
  g_ev.clear(); g_rec.clear(); g_used = 0; g_overflow = false; g_on = false;
  if (max_records <= 0) return 0;
  g_ev.resize(2 * (size_t)max_records);
  for (auto& e : g_ev)
    if (hipEventCreate(&e) != hipSuccess) return -4;
  g_rec.resize(max_records);
  g_on = true;
  return 0;
}

void mgrit_profile_reset(void) { mg::g_used = 0; mg::g_overflow = false; }

// Totals of one class since the last reset.  The caller must have synchronised the stream.
// Returns 0, or -1 for a bad class, -3 if the pool overflowed (totals are then partial).
int mgrit_profile_read(int cls, double* total_ms, double* flops, double* bytes, int64_t* launches) {
  using namespace mg;
  if (cls < 0 || cls >= PC_COUNT) return -1;
  double ms = 0, fl = 0, by = 0;
  int64_t n = 0;
  for (size_t i = 0; i < g_used; ++i) {
    if (g_rec[i].cls != cls) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_ev[2 * i], g_ev[2 * i + 1]) != hipSuccess) continue;
    ms += t; fl += g_rec[i].flops; by += g_rec[i].bytes; ++n;
  }
  if (total_ms) *total_ms = ms;
  if (flops) *flops = fl;
  if (bytes) *bytes = by;
  if (launches) *launches = n;
  return g_overflow ? -3 : 0;
}

}  // extern "C"
