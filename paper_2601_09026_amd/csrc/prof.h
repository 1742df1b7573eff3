// Optional per-launch timing with HIP events on the launch stream (off by default).
// Used by the benchmark to report achieved FLOP/s and bytes/s of each kernel class.
#pragma once
#include <hip/hip_runtime.h>

namespace mg {

enum ProfClass : int {
  PC_GEMM_SIMPLE = 0, PC_ATTN_FWD = 1, PC_ATTN_BWD = 2, PC_LN_FWD = 3, PC_LN_BWD = 4, PC_ELEMENTWISE = 5,
  PC_LN_FWD_SINGLE = 6, PC_LN_BWD_SINGLE = 7,   // LayerNorm launches over a single group (coarse chain)
  PC_GEMM_MFMA = 8,          // + epilogue id (0..6): launches over several groups (relaxation sweeps)
  PC_GEMM_MFMA_SINGLE = 16,  // + epilogue id: one group per launch (the serial coarse chain)
  PC_COUNT = 24
};

bool prof_enabled();
void prof_begin(int cls, double flops, double bytes, hipStream_t st);
void prof_end(hipStream_t st);

struct ProfScope {
  hipStream_t st; bool on;
  ProfScope(int cls, double flops, double bytes, hipStream_t s) : st(s), on(prof_enabled()) {
    if (on) prof_begin(cls, flops, bytes, st);
  }
  ~ProfScope() { if (on) prof_end(st); }
};

}  // namespace mg
