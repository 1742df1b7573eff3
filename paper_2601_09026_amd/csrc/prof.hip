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

// ---------------------------------------------------------------------------
// Measured ceilings of the box, for the "fraction of achievable" beside the datasheet fractions:
// a register-resident 32x32x16 bf16 MFMA loop (8 independent accumulators per wavefront, operands
// pseudo-random so that the clock sees a realistic power draw) and a streaming copy.
// ---------------------------------------------------------------------------
namespace mg {
namespace {
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 pk_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float pk_f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float pk_f32x4;

__global__ void __launch_bounds__(256) mfma_ceiling_kernel(float* out, int iters) {
  constexpr int NACC = 8;
  pk_f32x16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  pk_bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    unsigned x = (threadIdx.x * 8 + e) * 2654435761u;
    a[e] = (__bf16)(((x >> 8) & 0xffff) / 65536.0f - 0.5f);
    x = x * 1664525u + 1013904223u;
    b[e] = (__bf16)(((x >> 8) & 0xffff) / 65536.0f - 0.5f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = sum;
}

__global__ void empty_kernel() {}

__global__ void __launch_bounds__(256) copy_ceiling_kernel(const pk_f32x4* in, pk_f32x4* out, long n) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) out[i] = in[i];
}

// time `launch()` (already warmed up by one call) between two events on `st`; host-synchronous
template <typename F>
int timed_ms(F launch, hipStream_t st, float* ms) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return -4;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -4; }
  launch();
  int rc = 0;
  if (hipEventRecord(e0, st) != hipSuccess) rc = -4;
  launch();
  if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
      hipEventElapsedTime(ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess)
    rc = -4;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}
}  // namespace
}  // namespace mg

extern "C" {

// scratch: device, at least 512 KiB.  Returns 0 and the rate of the MFMA loop, -1 on bad arguments,
// -4 on a HIP error.  Synchronises the stream.
int mgrit_measure_mfma_ceiling(void* scratch, size_t scratch_bytes, int iters, double* tflops, void* stream) {
  using namespace mg;
  const int blocks = 512;                                // two 4-wavefront blocks per compute unit
  if (!scratch || !tflops || iters <= 0 || iters > (1 << 20) || scratch_bytes < (size_t)blocks * 256 * sizeof(float))
    return -1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float ms = 0.f;
  const int rc = timed_ms([&] {
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(blocks), dim3(256), 0, st, static_cast<float*>(scratch), iters);
  }, st, &ms);
  if (rc != 0) return rc;
  *tflops = (double)blocks * 4 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12;
  return 0;
}

// src, dst: device, `bytes` each (a multiple of 16, at least 1 MiB), not overlapping.  Returns 0 and
// the read + write rate of a grid-stride copy in GB/s (the best of three grid sizes).  Synchronises the stream.
int mgrit_measure_copy_ceiling(const void* src, void* dst, size_t bytes, double* gbs, void* stream) {
  using namespace mg;
  if (!src || !dst || !gbs || bytes < (1u << 20) || bytes % 16 != 0) return -1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long n = (long)(bytes / 16);
  // The rate of a streaming copy depends on how many wavefronts share the memory system: with few
  // resident blocks the accesses of the whole chip stay inside a window of a few MB and the DRAM
  // pages they open are used up before they are closed; with many the window grows and the rate
  // falls (measured at 1 GiB: 5.6 TB/s with 4 blocks per compute unit, 4.6 TB/s with 32).  The
  // ceiling reported is the best of three grid sizes.
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  double best = 0.0;
  for (int per_cu : {4, 8, 32}) {
    float ms = 0.f;
    const int rc = timed_ms([&] {
      hipLaunchKernelGGL(copy_ceiling_kernel, dim3(cus * per_cu), dim3(256), 0, st, static_cast<const pk_f32x4*>(src),
                         static_cast<pk_f32x4*>(dst), n);
    }, st, &ms);
    if (rc != 0) return rc;
    const double rate = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;
    if (rate > best) best = rate;
  }
  *gbs = best;
  return 0;
}


// What an event pair adds to the launch it brackets: the median time between two events recorded on
// `stream` around a kernel that does nothing, over 64 launches.  Synchronises the stream.
int mgrit_measure_event_bracket(double* us, void* stream) {
  using namespace mg;
  if (!us) return -1;
  hipStream_t st = static_cast<hipStream_t>(stream);
  constexpr int N = 64;
  hipEvent_t ev[2 * N];
  int made = 0, rc = 0;
  for (; made < 2 * N; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) { rc = -4; break; }
  float t[N];
  if (rc == 0) {
    for (int i = 0; i < N && rc == 0; ++i) {
      if (hipEventRecord(ev[2 * i], st) != hipSuccess) rc = -4;
      hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, st);
      if (hipEventRecord(ev[2 * i + 1], st) != hipSuccess) rc = -4;
    }
    if (rc == 0 && hipStreamSynchronize(st) != hipSuccess) rc = -4;
    for (int i = 0; i < N && rc == 0; ++i)
      if (hipEventElapsedTime(&t[i], ev[2 * i], ev[2 * i + 1]) != hipSuccess) rc = -4;
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  if (rc != 0) return rc;
  for (int i = 1; i < N; ++i)                            // insertion sort: median of 64
    for (int j = i; j > 0 && t[j] < t[j - 1]; --j) { const float x = t[j]; t[j] = t[j - 1]; t[j - 1] = x; }
  *us = 0.5 * (t[N / 2 - 1] + t[N / 2]) * 1e3;
  return 0;
}

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
