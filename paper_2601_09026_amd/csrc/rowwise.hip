// Bandwidth-bound kernels of the layer step and of the MGRIT driver: LayerNorm forward
// and its VJP (one 64-lane wavefront per token row, 16-byte accesses, row kept in
// registers, two-pass statistics), casts, residual differences and norms, pointer
// tables, weight transposition for the adjoint.
#include "common.h"
#include "kernels.h"
#include "prof.h"

namespace mg {
// streamed inputs (read once per launch): non-temporal loads; outputs are stored normally, the
// next kernel of the chain reads them
template <typename T> __device__ __forceinline__ f32x4 rload4(const T* p);
template <> __device__ __forceinline__ f32x4 rload4<float>(const float* p) { return ld_stream(reinterpret_cast<const f32x4*>(p)); }
template <> __device__ __forceinline__ f32x4 rload4<bf16>(const bf16* p) {
  bf16x4 v = ld_stream(reinterpret_cast<const bf16x4*>(p));
  f32x4 r = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
  return r;
}

// One 64-lane wavefront walks token rows with a grid stride.  NV = float4 per lane (row kept in
// registers), d <= 256*NV.  Rows of up to 256 elements keep the next row's loads in flight while the
// current one is reduced and written; for longer rows the second register set costs more in resident
// wavefronts than the overlap gains (d = 768: 74 -> 48 registers, +5 % bandwidth, and a block then
// fits beside a resident GEMM block of the other lane).
constexpr int LN_MAXV = 8;          // d <= 64*4*8 = 2048
constexpr int LN_FWD_BLOCKS_PER_CU = 16;   // grid caps (measured: the forward kernel gains from the larger one,
constexpr int LN_BWD_BLOCKS_PER_CU = 16;   // the VJP likewise once it no longer prefetches rows of more than 512 elements)

// LN input = state row (optional) + packed fp32 addend (optional); at least one is present
__device__ __forceinline__ f32x4 load_sum(const float* x, const float* xa, int c) {
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (x) v = ld_stream(reinterpret_cast<const f32x4*>(x + c));
  if (xa) v += ld_stream(reinterpret_cast<const f32x4*>(xa + c));
  return v;
}

__device__ __forceinline__ float sum4(f32x4 v) { return (v[0] + v[1]) + (v[2] + v[3]); }
__device__ __forceinline__ float dot4(f32x4 a, f32x4 b) { return (a[0] * b[0] + a[1] * b[1]) + (a[2] * b[2] + a[3] * b[3]); }

// sum over the LPR consecutive lanes that share a row
template <int LPR> __device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// LPR lanes per row: 64 (one row per wavefront, NV vectors of 4 per lane), or 32 / 16 for rows of at
// most 128 / 64 elements (NV = 1), where a wavefront works on 2 / 4 rows at once.
template <typename TO, int NV, int LPR>
__global__ void __launch_bounds__(256) ln_fwd_kernel(const LnFwdArgs a) {
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & (LPR - 1);
  const int total = a.n_groups * a.T;
  const int nwaves = gridDim.x * 4 * RPW;
  const int d = a.d;
  int row = (blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + ((threadIdx.x & 63) / LPR);
  if (row >= total) return;

  auto src = [&](int r, const float*& x, const float*& xa, int& g, int& t) {
    g = r / a.T; t = r - g * a.T;
    x = a.X.present() ? a.X.at(g) + (long)t * d : nullptr;
    xa = a.xp ? a.xp + a.xp_slots.of(g) * a.xp_slot_stride + (long)t * d : nullptr;
  };
  auto load = [&](int r, f32x4* v) {
    const float *x, *xa; int g, t;
    src(r, x, xa, g, t);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (i * LPR + lane) * 4;
      if (c < d) v[i] = load_sum(x, xa, c);
    }
  };
  constexpr bool PREFETCH = NV == 1;
  f32x4 cur[NV], nxt[PREFETCH ? NV : 1];
  load(row, cur);
  while (true) {
    const int next = row + nwaves;
    if (PREFETCH && next < total) load(next, nxt);
    const int g = row / a.T, t = row - g * a.T;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if ((i * LPR + lane) * 4 < d) s += sum4(cur[i]);
    const float mu = group_sum<LPR>(s) / d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if ((i * LPR + lane) * 4 < d) { cur[i] = cur[i] - mu; q += dot4(cur[i], cur[i]); }
    const float rstd = 1.0f / sqrtf(group_sum<LPR>(q) / d + a.eps);
    const char* pb = a.P.at(g);
    const float* gamma = reinterpret_cast<const float*>(pb + a.gamma_off);
    const float* beta = reinterpret_cast<const float*>(pb + a.beta_off);
    TO* out = reinterpret_cast<TO*>(a.out) + a.out_slots.of(g) * a.out_slot_stride + (long)t * d;
    TO* xh = a.xhat ? reinterpret_cast<TO*>(a.xhat) + a.xhat_slots.of(g) * a.xhat_slot_stride + (long)t * d : nullptr;
    if (xh && lane == 0) a.rstd[a.xhat_slots.of(g) * a.T + t] = rstd;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (i * LPR + lane) * 4;
      if (c < d) {
        const f32x4 xn = cur[i] * rstd;
        if (xh) store4<TO>(xh + c, xn);
        store4<TO>(out + c, xn * *reinterpret_cast<const f32x4*>(gamma + c) + *reinterpret_cast<const f32x4*>(beta + c));
      }
    }
    if (next >= total) break;
    if constexpr (PREFETCH) {
#pragma unroll
      for (int i = 0; i < NV; ++i) cur[i] = nxt[i];
    } else {
      load(next, cur);
    }
    row = next;
  }
}

static int ln_lanes_per_row(int d) { return d <= 64 ? 16 : d <= 128 ? 32 : 64; }

static unsigned ln_grid(long rows, int d, int blocks_per_cu) {
  const long per_block = 4 * (64 / ln_lanes_per_row(d));
  long want = (rows + per_block - 1) / per_block;
  const long cap = 256L * blocks_per_cu;
  return (unsigned)(want < cap ? want : cap);
}

template <typename TO>
static void ln_fwd_dispatch(const LnFwdArgs& a, unsigned blocks, hipStream_t st) {
  const int nv = (a.d + 255) / 256, lpr = ln_lanes_per_row(a.d);
  if (lpr == 16) hipLaunchKernelGGL((ln_fwd_kernel<TO, 1, 16>), dim3(blocks), dim3(256), 0, st, a);
  else if (lpr == 32) hipLaunchKernelGGL((ln_fwd_kernel<TO, 1, 32>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv <= 1) hipLaunchKernelGGL((ln_fwd_kernel<TO, 1, 64>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv == 2) hipLaunchKernelGGL((ln_fwd_kernel<TO, 2, 64>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv == 3) hipLaunchKernelGGL((ln_fwd_kernel<TO, 3, 64>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv == 4) hipLaunchKernelGGL((ln_fwd_kernel<TO, 4, 64>), dim3(blocks), dim3(256), 0, st, a);
  else hipLaunchKernelGGL((ln_fwd_kernel<TO, 8, 64>), dim3(blocks), dim3(256), 0, st, a);
}

hipError_t launch_ln_fwd(const LnFwdArgs& a, bool is_bf16, hipStream_t st) {
  const long rows = (long)a.n_groups * a.T;
  if (rows <= 0) return hipSuccess;
  if (rows > 0x7fffffffL || a.d > 256 * LN_MAXV) return hipErrorInvalidValue;
  const unsigned blocks = ln_grid(rows, a.d, LN_FWD_BLOCKS_PER_CU);
  const double esz = is_bf16 ? 2 : 4;
  ProfScope ps(a.n_groups > 1 ? PC_LN_FWD : PC_LN_FWD_SINGLE, 8.0 * rows * a.d,
               (double)rows * a.d * ((a.X.present() ? 4 : 0) + (a.xp ? 4 : 0) + esz), st);
  if (is_bf16) ln_fwd_dispatch<bf16>(a, blocks, st);
  else ln_fwd_dispatch<float>(a, blocks, st);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// LayerNorm VJP with fused residual bookkeeping
//   xhat = (x-mu)*rstd, dxhat = dy*gamma,
//   vjp  = rstd*(dxhat - mean(dxhat) - xhat*mean(dxhat*xhat))
//   v = add + vjp;  out_f32 = v;  out_op = c + v;  OUT = c + hstep*v + RHS
// ---------------------------------------------------------------------------
template <typename TO, int NV, bool XH, int LPR>
__global__ void __launch_bounds__(256) ln_bwd_kernel(const LnBwdArgs a) {
  constexpr int RPW = 64 / LPR;                      // rows per wavefront, as in ln_fwd_kernel
  const int lane = threadIdx.x & (LPR - 1);
  const int total = a.n_groups * a.T;
  const int nwaves = gridDim.x * 4 * RPW;
  const int d = a.d;
  int row = (blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + ((threadIdx.x & 63) / LPR);
  if (row >= total) return;

  // XH: the row arrives normalised (cached xhat, rs = its rstd); otherwise as X (+ addend)
  auto load = [&](int r, f32x4* v, f32x4* w, float& rs) {
    const int g = r / a.T, t = r - g * a.T;
    const long ro = (long)t * d;
    const TO* dy = reinterpret_cast<const TO*>(a.dy) + a.dy_slots.of(g) * a.dy_slot_stride + ro;
    if constexpr (XH) {
      const TO* xh = reinterpret_cast<const TO*>(a.xhat) + a.xhat_slots.of(g) * a.xhat_slot_stride + ro;
      rs = a.rstd[a.xhat_slots.of(g) * a.T + t];
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * LPR + lane) * 4;
        if (c < d) { v[i] = rload4<TO>(xh + c); w[i] = rload4<TO>(dy + c); }
      }
    } else {
      const float* x = a.X.present() ? a.X.at(g) + ro : nullptr;
      const float* xa = a.xp ? a.xp + a.xp_slots.of(g) * a.xp_slot_stride + ro : nullptr;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = (i * LPR + lane) * 4;
        if (c < d) { v[i] = load_sum(x, xa, c); w[i] = rload4<TO>(dy + c); }
      }
    }
  };
  constexpr bool PREFETCH = NV <= 2;                 // wider rows would spill: load in place instead
  f32x4 v[NV], w[NV], nv_[PREFETCH ? NV : 1], nw_[PREFETCH ? NV : 1];
  float rs_cur = 0.f, rs_next = 0.f;
  load(row, v, w, rs_cur);
  while (true) {
    const int next = row + nwaves;
    if (PREFETCH && next < total) load(next, nv_, nw_, rs_next);
    const int g = row / a.T, t = row - g * a.T;
    const long ro = (long)t * d;
    const float* gamma = reinterpret_cast<const float*>(a.P.at(g) + a.gamma_off);
    float rstd = rs_cur;
    if constexpr (!XH) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i)
        if ((i * LPR + lane) * 4 < d) s += sum4(v[i]);
      const float mu = group_sum<LPR>(s) / d;
      float q = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i)
        if ((i * LPR + lane) * 4 < d) { v[i] = v[i] - mu; q += dot4(v[i], v[i]); }
      rstd = 1.0f / sqrtf(group_sum<LPR>(q) / d + a.eps);
    }
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (i * LPR + lane) * 4;
      if (c < d) {
        if constexpr (!XH) v[i] = v[i] * rstd;                           // xhat
        w[i] = w[i] * *reinterpret_cast<const f32x4*>(gamma + c);        // dxhat
        s1 += sum4(w[i]);
        s2 += dot4(w[i], v[i]);
      }
    }
    const float m1 = group_sum<LPR>(s1) / d, m2 = group_sum<LPR>(s2) / d;
    const float* add = a.add ? a.add + a.add_slots.of(g) * a.add_slot_stride + ro : nullptr;
    float* of = a.out_f32 ? a.out_f32 + a.of_slots.of(g) * a.of_slot_stride + ro : nullptr;
    TO* oo = a.out_op ? reinterpret_cast<TO*>(a.out_op) + a.oo_slots.of(g) * a.oo_slot_stride + ro : nullptr;
    const TO* cop = a.cop ? reinterpret_cast<const TO*>(a.cop) + a.cop_slots.of(g) * a.cop_slot_stride + ro : nullptr;
    const bool need_c = (oo != nullptr && !cop) || a.OUT.present();
    const float* cvec = need_c ? a.C.at(g) + ro : nullptr;
    float* OUT = a.OUT.present() ? a.OUT.at(g) + ro : nullptr;
    TO* ocast = a.out_cast ? reinterpret_cast<TO*>(a.out_cast) + a.oc_slots.of(g) * a.oc_slot_stride + ro : nullptr;
    const float* RHS = a.RHS.present() ? a.RHS.at(g) + ro : nullptr;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (i * LPR + lane) * 4;
      if (c < d) {
        f32x4 r = rstd * (w[i] - m1 - v[i] * m2);
        if (add) r += ld_stream(reinterpret_cast<const f32x4*>(add + c));
        if (of) *reinterpret_cast<f32x4*>(of + c) = r;
        if (oo && cop) store4<TO>(oo + c, rload4<TO>(cop + c) + r);
        if (need_c) {
          f32x4 cc = *reinterpret_cast<const f32x4*>(cvec + c);
          if (oo && !cop) store4<TO>(oo + c, cc + r);
          if (OUT) {
            f32x4 res = cc + a.hstep * r;
            if (RHS) {
              // rhs_sign = 1: res + rhs; -1: rhs - res (the coarse right-hand side), each rounded once
              const f32x4 rhs = ld_stream(reinterpret_cast<const f32x4*>(RHS + c));
#pragma unroll
              for (int e = 0; e < 4; ++e) res[e] = __builtin_fmaf(a.rhs_sign, res[e], rhs[e]);
            }
            *reinterpret_cast<f32x4*>(OUT + c) = res;
            if (ocast) store4<TO>(ocast + c, res);
          }
        }
      }
    }
    if (next >= total) break;
    if constexpr (PREFETCH) {
#pragma unroll
      for (int i = 0; i < NV; ++i) { v[i] = nv_[i]; w[i] = nw_[i]; }
      rs_cur = rs_next;
    } else {
      load(next, v, w, rs_cur);
    }
    row = next;
  }
}

template <typename TO, bool XH>
static void ln_bwd_dispatch(const LnBwdArgs& a, unsigned blocks, hipStream_t st) {
  const int nv = (a.d + 255) / 256, lpr = ln_lanes_per_row(a.d);
  if (lpr == 16) hipLaunchKernelGGL((ln_bwd_kernel<TO, 1, XH, 16>), dim3(blocks), dim3(256), 0, st, a);
  else if (lpr == 32) hipLaunchKernelGGL((ln_bwd_kernel<TO, 1, XH, 32>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv <= 1) hipLaunchKernelGGL((ln_bwd_kernel<TO, 1, XH, 64>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv == 2) hipLaunchKernelGGL((ln_bwd_kernel<TO, 2, XH, 64>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv == 3) hipLaunchKernelGGL((ln_bwd_kernel<TO, 3, XH, 64>), dim3(blocks), dim3(256), 0, st, a);
  else if (nv == 4) hipLaunchKernelGGL((ln_bwd_kernel<TO, 4, XH, 64>), dim3(blocks), dim3(256), 0, st, a);
  else hipLaunchKernelGGL((ln_bwd_kernel<TO, 8, XH, 64>), dim3(blocks), dim3(256), 0, st, a);
}

hipError_t launch_ln_bwd(const LnBwdArgs& a, bool is_bf16, hipStream_t st) {
  const long rows = (long)a.n_groups * a.T;
  if (rows <= 0) return hipSuccess;
  if (rows > 0x7fffffffL || a.d > 256 * LN_MAXV) return hipErrorInvalidValue;
  const unsigned blocks = ln_grid(rows, a.d, LN_BWD_BLOCKS_PER_CU);
  const double esz = is_bf16 ? 2 : 4;
  const bool xh = a.xhat != nullptr;
  if (xh && !a.rstd) return hipErrorInvalidValue;
  const bool c_rows = (a.out_op && !a.cop) || a.OUT.present();
  const double per_elem = esz + (xh ? esz : (a.X.present() ? 4 : 0) + (a.xp ? 4 : 0)) + (a.add ? 4 : 0) +
                          (a.out_f32 ? 4 : 0) + (c_rows ? 4 : 0) + (a.out_op && a.cop ? esz : 0) +
                          (a.out_op ? esz : 0) + (a.OUT.present() ? 4 : 0) + (a.RHS.present() ? 4 : 0) +
                          (a.out_cast && a.OUT.present() ? esz : 0);
  ProfScope ps(a.n_groups > 1 ? PC_LN_BWD : PC_LN_BWD_SINGLE, 16.0 * rows * a.d, (double)rows * a.d * per_elem, st);
  if (is_bf16) { if (xh) ln_bwd_dispatch<bf16, true>(a, blocks, st); else ln_bwd_dispatch<bf16, false>(a, blocks, st); }
  else { if (xh) ln_bwd_dispatch<float, true>(a, blocks, st); else ln_bwd_dispatch<float, false>(a, blocks, st); }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// casts
// ---------------------------------------------------------------------------
template <typename TO>
__global__ void __launch_bounds__(256) cast_rows_kernel(long elems, Rows X, TO* out, long out_slot_stride,
                                                        Slots out_slots) {
  const int g = blockIdx.y;
  const float* x = X.at(g);
  TO* o = out + out_slots.of(g) * out_slot_stride;
  for (long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4; i < elems; i += (long)gridDim.x * 256 * 4)
    store4<TO>(o + i, ld_stream(reinterpret_cast<const f32x4*>(x + i)));
}

hipError_t launch_cast_rows(int n_groups, long elems, Rows X, void* out, long out_slot_stride,
                            Slots out_slots, bool is_bf16, hipStream_t st) {
  if (n_groups <= 0 || elems <= 0) return hipSuccess;
  long want = (elems / 4 + 255) / 256;
  const unsigned bx = (unsigned)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
  ProfScope ps(PC_ELEMENTWISE, 0.0, (double)n_groups * elems * (4 + (is_bf16 ? 2 : 4)), st);
  if (is_bf16)
    hipLaunchKernelGGL(cast_rows_kernel<bf16>, dim3(bx, n_groups), dim3(256), 0, st, elems, X, (bf16*)out,
                       out_slot_stride, out_slots);
  else
    hipLaunchKernelGGL(cast_rows_kernel<float>, dim3(bx, n_groups), dim3(256), 0, st, elems, X, (float*)out,
                       out_slot_stride, out_slots);
  return hipGetLastError();
}

template <typename TO>
__global__ void __launch_bounds__(256) cast_flat_kernel(const float* in, TO* out, long elems) {
  for (long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4; i < elems; i += (long)gridDim.x * 256 * 4)
    store4<TO>(out + i, ld_stream(reinterpret_cast<const f32x4*>(in + i)));
}

hipError_t launch_cast_flat(const float* in, void* out, long elems, bool is_bf16, hipStream_t st) {
  if (elems <= 0) return hipSuccess;
  long want = (elems / 4 + 255) / 256;
  const unsigned bx = (unsigned)(want < 1 ? 1 : (want > 4096 ? 4096 : want));
  if (is_bf16) hipLaunchKernelGGL(cast_flat_kernel<bf16>, dim3(bx), dim3(256), 0, st, in, (bf16*)out, elems);
  else hipLaunchKernelGGL(cast_flat_kernel<float>, dim3(bx), dim3(256), 0, st, in, (float*)out, elems);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// driver elementwise: differences and the residual norm
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) sub_rows_kernel(long elems, Rows A, Rows B, Rows D) {
  const int g = blockIdx.y;
  const float* pa = A.at(g);
  const float* pb = B.at(g);
  float* pd = D.at(g);
  for (long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4; i < elems; i += (long)gridDim.x * 256 * 4)
    *reinterpret_cast<f32x4*>(pd + i) =
        ld_stream(reinterpret_cast<const f32x4*>(pa + i)) - ld_stream(reinterpret_cast<const f32x4*>(pb + i));
}

hipError_t launch_sub_rows(int n_groups, long elems, Rows A, Rows B, Rows D, hipStream_t st) {
  if (n_groups <= 0 || elems <= 0) return hipSuccess;
  long want = (elems / 4 + 255) / 256;
  const unsigned bx = (unsigned)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
  ProfScope ps(PC_ELEMENTWISE, (double)n_groups * elems, (double)n_groups * elems * 12, st);
  hipLaunchKernelGGL(sub_rows_kernel, dim3(bx, n_groups), dim3(256), 0, st, elems, A, B, D);
  return hipGetLastError();
}

// D = A (+ B): the part of a stacked state that a step leaves alone, plus the right-hand side
__global__ void __launch_bounds__(256) add_rows_kernel(long elems, Rows A, Rows B, Rows D) {
  const int g = blockIdx.y;
  const float* pa = A.at(g);
  const float* pb = B.present() ? B.at(g) : nullptr;
  float* pd = D.at(g);
  for (long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4; i < elems; i += (long)gridDim.x * 256 * 4) {
    f32x4 v = ld_stream(reinterpret_cast<const f32x4*>(pa + i));
    if (pb) v += ld_stream(reinterpret_cast<const f32x4*>(pb + i));
    *reinterpret_cast<f32x4*>(pd + i) = v;
  }
}

hipError_t launch_add_rows(int n_groups, long elems, Rows A, Rows B, Rows D, hipStream_t st) {
  if (n_groups <= 0 || elems <= 0) return hipSuccess;
  long want = (elems / 4 + 255) / 256;
  const unsigned bx = (unsigned)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
  ProfScope ps(PC_ELEMENTWISE, B.present() ? (double)n_groups * elems : 0.0,
               (double)n_groups * elems * (B.present() ? 12 : 8), st);
  hipLaunchKernelGGL(add_rows_kernel, dim3(bx, n_groups), dim3(256), 0, st, elems, A, B, D);
  return hipGetLastError();
}

constexpr int RN_BLOCKS = 32;       // partial sums per group

__global__ void __launch_bounds__(256) resnorm_partial_kernel(long elems, Rows A, Rows B, double* partial) {
  __shared__ double red[256];
  const int g = blockIdx.y;
  const float* pa = A.at(g);
  const float* pb = B.at(g);
  float s = 0.f;
  double acc = 0.0;
  int cnt = 0;
  for (long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4; i < elems; i += (long)gridDim.x * 256 * 4) {
    f32x4 e = ld_stream(reinterpret_cast<const f32x4*>(pa + i)) - ld_stream(reinterpret_cast<const f32x4*>(pb + i));
    s += (e[0] * e[0] + e[1] * e[1]) + (e[2] * e[2] + e[3] * e[3]);
    if (++cnt == 64) { acc += (double)s; s = 0.f; cnt = 0; }
  }
  acc += (double)s;
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[(long)g * gridDim.x + blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(256) resnorm_final_kernel(const double* partial, int n, float* out) {
  __shared__ double red[256];
  double acc = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) acc += partial[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = (float)sqrt(red[0]);
}

hipError_t launch_resnorm(int n_groups, long elems, Rows A, Rows B, double* partial, int max_partial,
                          float* out, hipStream_t st) {
  if (n_groups <= 0 || elems <= 0) return hipSuccess;
  if (n_groups * RN_BLOCKS > max_partial) return hipErrorInvalidValue;
  ProfScope ps(PC_ELEMENTWISE, 3.0 * n_groups * elems, (double)n_groups * elems * 8, st);
  hipLaunchKernelGGL(resnorm_partial_kernel, dim3(RN_BLOCKS, n_groups), dim3(256), 0, st, elems, A, B, partial);
  hipLaunchKernelGGL(resnorm_final_kernel, dim3(1), dim3(256), 0, st, partial, n_groups * RN_BLOCKS, out);
  return hipGetLastError();
}
int resnorm_partials_per_group() { return RN_BLOCKS; }

// ---------------------------------------------------------------------------
// pointer tables
// ---------------------------------------------------------------------------
__global__ void fill_table_kernel(void** tab, char* base, long stride_bytes, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) tab[i] = base + (long)i * stride_bytes;
}

hipError_t launch_fill_table(void** tab, char* base, long stride_bytes, int n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, tab, base, stride_bytes, n);
  return hipGetLastError();
}

struct PtrPack { const void* p[32]; };
__global__ void upload_ptrs_kernel(void** tab, PtrPack pack, int n) {
  const int i = threadIdx.x;
  if (i < n) tab[i] = const_cast<void*>(pack.p[i]);
}

hipError_t upload_pointers(void** tab, const void* const* host_ptrs, int n, hipStream_t st) {
  for (int i0 = 0; i0 < n; i0 += 32) {
    PtrPack pack;
    const int m = n - i0 < 32 ? n - i0 : 32;
    for (int i = 0; i < 32; ++i) pack.p[i] = i < m ? host_ptrs[i0 + i] : nullptr;
    hipLaunchKernelGGL(upload_ptrs_kernel, dim3(1), dim3(32), 0, st, tab + i0, pack, m);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// weight transposition (adjoint): out_g[c,r] = in_g[r,c]
// ---------------------------------------------------------------------------
template <typename U>
__global__ void __launch_bounds__(256) transpose_kernel(Params in, Params out, long off, int rows, int cols) {
  __shared__ U tile[32][33];
  const int g = blockIdx.z;
  const U* src = reinterpret_cast<const U*>(in.at(g) + off);
  U* dst = reinterpret_cast<U*>(const_cast<char*>(out.at(g)) + off);
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8) {
    const int r = r0 + i, c = c0 + tx;
    if (r < rows && c < cols) tile[i][tx] = src[(long)r * cols + c];
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) dst[(long)c * rows + r] = tile[tx][i];
  }
}

hipError_t launch_transpose(int n_groups, Params in, Params out, long off, int rows, int cols, int elem_bytes,
                            hipStream_t st) {
  if (n_groups <= 0) return hipSuccess;
  dim3 grid((cols + 31) / 32, (rows + 31) / 32, n_groups);
  ProfScope ps(PC_ELEMENTWISE, 0.0, 2.0 * n_groups * rows * cols * elem_bytes, st);
  if (elem_bytes == 2)
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, st, in, out, off, rows, cols);
  else
    hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, st, in, out, off, rows, cols);
  return hipGetLastError();
}

}  // namespace mg
