// Shared device-side declarations of the MGRIT hot-path kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mg {

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int WAVE = 64;

// ---------------------------------------------------------------------------
// Per-group addressing.  A batched launch works on `n` independent groups
// (coarse intervals).  Everything a group touches is found through device
// pointer tables indexed affinely by the group number, so that one launch can
// serve any sweep of the MGRIT driver without re-uploading pointers:
//   table entry of group g = tab[i0 + g*is]
// Packed intermediate buffers are indexed by "slot" = slot0 + g*slot_s.
// ---------------------------------------------------------------------------
struct Rows {                       // fp32 [T,d] states reached through a table
  const void* const* tab;           // device array of device pointers (may be null)
  int i0, is;
  long off;                         // element offset inside every state (a row range of a stacked state)
  __device__ __forceinline__ float* at(int g) const {
    return (float*)const_cast<void*>(tab[i0 + (long)g * is]) + off;
  }
  __host__ __device__ bool present() const { return tab != nullptr; }
};

struct Params {                     // packed parameter blocks reached through a table
  const void* const* tab;
  int i0, is;
  __device__ __forceinline__ const char* at(int g) const {
    return (const char*)tab[i0 + (long)g * is];
  }
};

struct Slots {
  int s0, ss;
  __host__ __device__ __forceinline__ long of(int g) const { return s0 + (long)g * ss; }
};

// ---------------------------------------------------------------------------
// scalar helpers
// ---------------------------------------------------------------------------
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16>(bf16 v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float v) { return (bf16)v; }   // RNE

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

__device__ __forceinline__ float gelu_f(float z) {
  return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_prime_f(float z) {
  const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
  return cdf + z * pdf;
}

// Fast erf for the bf16 path: odd polynomial x*P(x^2) fitted by least squares on Chebyshev
// nodes of |x| <= 2.8, evaluated at the argument clamped to that range (erf(2.8) = 0.99992);
// absolute error at most 1.1e-4 everywhere (bf16 keeps 8 bits), no transcendental instruction.
__device__ __forceinline__ float erf_fast(float x) {
  x = fminf(fmaxf(x, -2.8f), 2.8f);
  const float t = x * x;
  float p = -5.83171111e-07f;
  p = fmaf(p, t, 2.22840511e-05f);
  p = fmaf(p, t, -3.73322994e-04f);
  p = fmaf(p, t, 3.65856420e-03f);
  p = fmaf(p, t, -2.37276428e-02f);
  p = fmaf(p, t, 1.09334266e-01f);
  p = fmaf(p, t, -3.74316462e-01f);
  p = fmaf(p, t, 1.12810103e+00f);
  return x * p;
}
__device__ __forceinline__ float gelu_fast(float z) {
  return 0.5f * z * (1.0f + erf_fast(z * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_prime_fast(float z) {
  const float cdf = 0.5f * (1.0f + erf_fast(z * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
  return cdf + z * pdf;
}
template <typename T> __device__ __forceinline__ float gelu_t(float z);
template <> __device__ __forceinline__ float gelu_t<float>(float z) { return gelu_f(z); }
template <> __device__ __forceinline__ float gelu_t<bf16>(float z) { return gelu_fast(z); }
template <typename T> __device__ __forceinline__ float gelu_prime_t(float z);
template <> __device__ __forceinline__ float gelu_prime_t<float>(float z) { return gelu_prime_f(z); }
template <> __device__ __forceinline__ float gelu_prime_t<bf16>(float z) { return gelu_prime_fast(z); }

// Accesses with the non-temporal hint, for data a kernel touches once.  Only for pointers into
// device global memory (never LDS or scratch): they are issued as global, not flat, instructions,
// which do not count against the counter that LDS reads are waited for on.
template <typename V> __device__ __forceinline__ void st_stream(V* p, V v) {
  typedef __attribute__((address_space(1))) V* gptr;
  __builtin_nontemporal_store(v, (gptr)p);
}
template <typename V> __device__ __forceinline__ V ld_stream(const V* p) {
  typedef const __attribute__((address_space(1))) V* gptr;
  return __builtin_nontemporal_load((gptr)p);
}

// load / store 4 consecutive elements as floats
template <typename T> __device__ __forceinline__ f32x4 load4(const T* p);
template <> __device__ __forceinline__ f32x4 load4<float>(const float* p) {
  return *reinterpret_cast<const f32x4*>(p);
}
template <> __device__ __forceinline__ f32x4 load4<bf16>(const bf16* p) {
  bf16x4 v = *reinterpret_cast<const bf16x4*>(p);
  f32x4 r = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
  return r;
}
template <typename T> __device__ __forceinline__ void store4(T* p, f32x4 v);
template <> __device__ __forceinline__ void store4<float>(float* p, f32x4 v) {
  *reinterpret_cast<f32x4*>(p) = v;
}
template <> __device__ __forceinline__ void store4<bf16>(bf16* p, f32x4 v) {
  bf16x4 r = {(bf16)v[0], (bf16)v[1], (bf16)v[2], (bf16)v[3]};
  *reinterpret_cast<bf16x4*>(p) = r;
}

// ---------------------------------------------------------------------------
// GEMM epilogues:  C[m,n] = sum_k A[m,k] B[n,k]  (+ bias[n]), then
// ---------------------------------------------------------------------------
enum Epi : int {
  EPI_STORE = 0,        // out = acc + bias                               (packed, operand type)
  EPI_GELU = 1,         // out = gelu(acc + bias); optionally z = acc + bias kept for the adjoint
  EPI_RESID_INNER = 2,  // ybar[m,n] (fp32, packed) = [base +] acc + bias      (sum of attention sublayers)
  EPI_RESID_OUTER = 3,  // OUT[m,n] = X + h*(ybar + acc + bias) + rhs          (the Euler update)
  EPI_DGELU = 4,        // out = acc * g[m,n], g = the cached gelu'(z)          (adjoint of the activation)
  EPI_STORE_F32 = 5,    // out (fp32, packed or inside the group's output block) = hstep * (acc + bias)
  EPI_GELU_PRIME = 6,   // out = gelu'(acc + bias) (operand type); optionally z = acc + bias kept as well:
                        // the linearisation cache holds the derivative, evaluated once per layer
  EPI_GELU_BOTH = 7     // out = gelu(acc + bias) and aux2 = gelu'(acc + bias); optionally z kept as well:
                        // a forward step that also leaves its layer's entry of the linearisation cache
};

struct GemmArgs {
  int n_groups;
  int M, N, K;                 // per group: C is [M,N], reduction length K
  // A operand: packed [slot, M, K] of operand type; a_group_stride = 0 shares A between groups
  const void* A; long a_slot_stride; Slots a_slots;
  // B operand: inside the parameter block (or its transposed copy) at byte offset b_off, [N,K]
  Params B; long b_off;
  long bias_off;               // byte offset of fp32 bias[N] inside the parameter block, -1 = none
  Params bias;
  // outputs / epilogue operands
  void* out; long out_slot_stride; Slots out_slots;      // packed output (operand type or fp32)
  void* aux; long aux_slot_stride; Slots aux_slots;      // EPI_GELU, EPI_GELU_PRIME: z out (may be null); EPI_DGELU: g in;
                                                         // EPI_RESID_OUTER: ybar (fp32 packed)
  void* aux2; long aux2_slot_stride; Slots aux2_slots;   // EPI_GELU_BOTH: gelu'(z) out (operand type)
  Rows X;                      // EPI_RESID_OUTER: the step's input state
  const float* base; long base_slot_stride; Slots base_slots;   // EPI_RESID_INNER: optional packed fp32 addend
  Rows OUT;                    // EPI_RESID_OUTER: the step's output state
  Rows RHS;                    // EPI_RESID_OUTER: optional right-hand side
  float hstep;
  float rhs_sign;              // EPI_RESID_OUTER with RHS: OUT = RHS + rhs_sign * (X + h*(..)); +1 the step, -1 the
                               // coarse right-hand side g' = R - Phi'(w) formed in the step that evaluates Phi'
  Params out_tab; long out_tab_off;    // EPI_STORE_F32: if set, group g writes at out_tab[g] + out_tab_off
};

}  // namespace mg
