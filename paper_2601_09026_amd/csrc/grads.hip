// Kernels of the parameter-gradient pass
//     dtheta_n = h * (dF/dtheta_n (Z_n))^T lambda_{n+1}            (paper section 3.1)
// that are not matrix products: operand transposition (the weight gradient dW = dY^T U is run
// as the same "both operands reduction-contiguous" GEMM on transposed copies) with the sums over
// tokens for the bias gradients taken on the way, and the LayerNorm gain / shift gradients.
// Sums over tokens are taken in two stages with a fixed order (no atomics): results are
// run-to-run identical.
#include "common.h"
#include "kernels.h"
#include "prof.h"

namespace mg {

// ---------------------------------------------------------------------------
// dst_g[c, r] = f(src_g[r, c]),  f = identity or GELU; packed operand-type buffers.
// Optionally also the column sums of the untransposed tile (fp32): partial[g][row block][c],
// which reduce_partials_kernel turns into the sum over all rows (the bias gradient).
// ---------------------------------------------------------------------------
constexpr int TR = 64;              // tile edge

// generic element type: one element per thread and step
template <typename T, bool GELU>
__global__ void __launch_bounds__(256) transpose_slots_kernel(const T* src, long src_slot_stride, Slots src_slots,
                                                              int rows, int cols, T* dst, long dst_slot_stride,
                                                              Slots dst_slots, float* partial) {
  __shared__ T tile[TR][TR + 2];
  const int g = blockIdx.z;
  const T* s = src + src_slots.of(g) * src_slot_stride;
  T* o = dst + dst_slots.of(g) * dst_slot_stride;
  const int c0 = blockIdx.x * TR, r0 = blockIdx.y * TR;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < TR; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    T v = from_f<T>(0.f);
    if (r < rows && c < cols) {
      v = s[(long)r * cols + c];
      if (GELU) v = from_f<T>(gelu_t<T>(to_f<T>(v)));
    }
    tile[i][tx] = v;
  }
  __syncthreads();
  for (int i = ty; i < TR; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) o[(long)c * rows + r] = tile[tx][i];
  }
  if (partial && ty == 0 && c0 + tx < cols) {
    float acc = 0.f;
    for (int i = 0; i < TR; ++i) acc += to_f<T>(tile[i][tx]);
    partial[((long)g * gridDim.y + blockIdx.y) * cols + c0 + tx] = acc;
  }
}

// bf16, rows and cols multiples of 64: a wavefront moves a 64x64 tile, each lane an 8x8 block
// that it transposes in registers; 8 lanes cover 128 contiguous bytes of a row on the way in
// (lane bits 0-2 walk the columns) and of a transposed row on the way out (lane bits 3-5 walk
// the rows), so both sides move whole 128-byte segments with 16-byte accesses and no LDS.
template <bool GELU>
__global__ void __launch_bounds__(256) transpose_slots_bf16_kernel(const bf16* src, long src_slot_stride,
                                                                   Slots src_slots, int rows, int cols, bf16* dst,
                                                                   long dst_slot_stride, Slots dst_slots,
                                                                   float* partial) {
  const int g = blockIdx.z;
  const int lane = threadIdx.x & 63, cb = lane & 7, rb = lane >> 3;
  const int row_block = blockIdx.y * 4 + (threadIdx.x >> 6);
  const int r0 = row_block * TR, c0 = blockIdx.x * TR;
  if (r0 >= rows) return;                                      // whole wavefront
  const bf16* s = src + src_slots.of(g) * src_slot_stride + (long)(r0 + 8 * rb) * cols + c0 + 8 * cb;
  bf16* o = dst + dst_slots.of(g) * dst_slot_stride + (long)(c0 + 8 * cb) * rows + r0 + 8 * rb;
  bf16x8 in[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    in[i] = *reinterpret_cast<const bf16x8*>(s + (long)i * cols);
    if (GELU) {
#pragma unroll
      for (int j = 0; j < 8; ++j) in[i][j] = (bf16)gelu_fast((float)in[i][j]);
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    bf16x8 v;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = in[i][j];
    *reinterpret_cast<bf16x8*>(o + (long)j * rows) = v;
  }
  if (partial) {
    const int n_row_blocks = (rows + TR - 1) / TR;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc += (float)in[i][j];
      acc += __shfl_xor(acc, 8, 64);
      acc += __shfl_xor(acc, 16, 64);
      acc += __shfl_xor(acc, 32, 64);
      if (rb == 0) partial[((long)g * n_row_blocks + row_block) * cols + c0 + 8 * cb + j] = acc;
    }
  }
}

// out_g[c] = scale * sum over slices of partial[g][slice][c0 + c] (row length ld), c < cols, written at
// byte offset `off` of the group's output block.  64 columns per block; the slices are dealt to four
// wavefronts and their four sums added in a fixed order.
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float* partial, int n_slices, int ld, int c0,
                                                              int cols, Params out, long off, float scale) {
  __shared__ float red[4][64];
  const int g = blockIdx.y;
  const int l = threadIdx.x & 63, ph = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + l;
  float acc = 0.f;
  if (c < cols) {
    const float* p = partial + (long)g * n_slices * ld + c0 + c;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int s = ph;
    for (; s + 12 < n_slices; s += 16) {
      a0 += p[(long)s * ld]; a1 += p[(long)(s + 4) * ld]; a2 += p[(long)(s + 8) * ld]; a3 += p[(long)(s + 12) * ld];
    }
    for (; s < n_slices; s += 4) a0 += p[(long)s * ld];
    acc = (a0 + a1) + (a2 + a3);
  }
  red[ph][l] = acc;
  __syncthreads();
  if (ph == 0 && c < cols) {
    float* o = reinterpret_cast<float*>(const_cast<char*>(out.at(g)) + off);
    o[c] = scale * ((red[0][l] + red[1][l]) + (red[2][l] + red[3][l]));
  }
}

__global__ void __launch_bounds__(256) sum_slots_kernel(const float* in, int n, long elems, float* out, float scale) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= elems) return;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < n; ++s) acc += *reinterpret_cast<const f32x4*>(in + (long)s * elems + i);
  *reinterpret_cast<f32x4*>(out + i) = scale * acc;
}

hipError_t launch_sum_slots(const float* in, int n, long elems, float* out, float scale, hipStream_t st) {
  if (n <= 0 || elems <= 0) return hipSuccess;
  if (elems % 4 != 0) return hipErrorInvalidValue;
  ProfScope ps(PC_ELEMENTWISE, 0.0, (double)(n + 1) * elems * 4, st);
  hipLaunchKernelGGL(sum_slots_kernel, dim3((unsigned)((elems / 4 + 255) / 256)), dim3(256), 0, st, in, n, elems, out,
                     scale);
  return hipGetLastError();
}

int transpose_row_blocks(int rows) { return (rows + TR - 1) / TR; }

hipError_t launch_transpose_slots(int n_groups, const void* src, long src_slot_stride, Slots src_slots, int rows,
                                  int cols, void* dst, long dst_slot_stride, Slots dst_slots, bool gelu,
                                  bool is_bf16, float* partial, Params sum_out, long sum_off, float sum_scale,
                                  hipStream_t st) {
  if (n_groups <= 0 || rows <= 0 || cols <= 0) return hipSuccess;
  const int n_row_blocks = (rows + TR - 1) / TR;
  const bool fast = is_bf16 && rows % TR == 0 && cols % TR == 0;
  dim3 grid((cols + TR - 1) / TR, fast ? (n_row_blocks + 3) / 4 : n_row_blocks, n_groups);
  {
    ProfScope ps(PC_ELEMENTWISE, 0.0, 2.0 * n_groups * rows * cols * (is_bf16 ? 2 : 4), st);
#define MG_TR(K, T)                                                                                          \
  hipLaunchKernelGGL(K, grid, dim3(256), 0, st, static_cast<const T*>(src), src_slot_stride, src_slots, rows, \
                     cols, static_cast<T*>(dst), dst_slot_stride, dst_slots, partial)
    if (fast) {
      if (gelu) MG_TR((transpose_slots_bf16_kernel<true>), bf16); else MG_TR((transpose_slots_bf16_kernel<false>), bf16);
    } else if (is_bf16) {
      if (gelu) MG_TR((transpose_slots_kernel<bf16, true>), bf16); else MG_TR((transpose_slots_kernel<bf16, false>), bf16);
    } else {
      if (gelu) MG_TR((transpose_slots_kernel<float, true>), float); else MG_TR((transpose_slots_kernel<float, false>), float);
    }
#undef MG_TR
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !partial) return e;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((cols + 63) / 64, n_groups), dim3(256), 0, st, partial,
                     n_row_blocks, cols, 0, cols, sum_out, sum_off, sum_scale);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// LayerNorm parameter gradients: dgamma[c] = sum_rows dy[r,c] * xhat[r,c], dbeta[c] = sum_rows
// dy[r,c], xhat recomputed from the LayerNorm input (state row + optional packed addend).
// One wavefront per row, LNP_WAVES wavefronts per group, a lane keeps the partial sums of its
// own columns in registers; partial[g][w] = [dgamma | dbeta] (2d floats); stage 2 as above.
// ---------------------------------------------------------------------------
constexpr int LNP_WAVES = 512;
constexpr int LNP_MAXV = 8;         // d <= 2048
int ln_param_partial_rows() { return LNP_WAVES; }

template <typename TO>
__global__ void __launch_bounds__(256) ln_param_partial_kernel(const LnParamArgs a, float* partial) {
  const int lane = threadIdx.x & 63;
  const int g = blockIdx.y;
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);          // 0 .. LNP_WAVES-1
  const int d = a.d;
  f32x4 ag[LNP_MAXV], ab[LNP_MAXV];
#pragma unroll
  for (int i = 0; i < LNP_MAXV; ++i) { ag[i] = f32x4{0.f, 0.f, 0.f, 0.f}; ab[i] = ag[i]; }
  const TO* dyb = reinterpret_cast<const TO*>(a.dy) + a.dy_slots.of(g) * a.dy_slot_stride;
  const float* xb = a.X.present() ? a.X.at(g) : nullptr;
  const float* xab = a.xp ? a.xp + a.xp_slots.of(g) * a.xp_slot_stride : nullptr;
  for (int t = w; t < a.T; t += LNP_WAVES) {
    const long ro = (long)t * d;
    f32x4 v[LNP_MAXV];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < LNP_MAXV; ++i) {
      const int c = (i * 64 + lane) * 4;
      if (c < d) {
        f32x4 x = {0.f, 0.f, 0.f, 0.f};
        if (xb) x = *reinterpret_cast<const f32x4*>(xb + ro + c);
        if (xab) x += *reinterpret_cast<const f32x4*>(xab + ro + c);
        v[i] = x;
        s += (x[0] + x[1]) + (x[2] + x[3]);
      }
    }
    const float mu = wave_sum(s) / d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < LNP_MAXV; ++i)
      if ((i * 64 + lane) * 4 < d) {
        v[i] = v[i] - mu;
        q += (v[i][0] * v[i][0] + v[i][1] * v[i][1]) + (v[i][2] * v[i][2] + v[i][3] * v[i][3]);
      }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / d + a.eps);
#pragma unroll
    for (int i = 0; i < LNP_MAXV; ++i) {
      const int c = (i * 64 + lane) * 4;
      if (c < d) {
        const f32x4 dy = load4<TO>(dyb + ro + c);
        ag[i] += dy * (v[i] * rstd);
        ab[i] += dy;
      }
    }
  }
  float* p = partial + ((long)g * LNP_WAVES + w) * 2 * d;
#pragma unroll
  for (int i = 0; i < LNP_MAXV; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < d) {
      *reinterpret_cast<f32x4*>(p + c) = ag[i];
      *reinterpret_cast<f32x4*>(p + d + c) = ab[i];
    }
  }
}

hipError_t launch_ln_param_grad(const LnParamArgs& a, float* partial, bool is_bf16, hipStream_t st) {
  if (a.n_groups <= 0 || a.T <= 0) return hipSuccess;
  if (a.d > 256 * LNP_MAXV || a.d % 4 != 0) return hipErrorInvalidValue;
  ProfScope ps(PC_ELEMENTWISE, 0.0, (double)a.n_groups * a.T * a.d * ((is_bf16 ? 2 : 4) + 4 + (a.xp ? 4 : 0)), st);
  dim3 grid(LNP_WAVES / 4, a.n_groups);
  if (is_bf16) hipLaunchKernelGGL(ln_param_partial_kernel<bf16>, grid, dim3(256), 0, st, a, partial);
  else hipLaunchKernelGGL(ln_param_partial_kernel<float>, grid, dim3(256), 0, st, a, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 g2((a.d + 63) / 64, a.n_groups);
  hipLaunchKernelGGL(reduce_partials_kernel, g2, dim3(256), 0, st, partial, LNP_WAVES, 2 * a.d, 0, a.d, a.out,
                     a.gamma_off, a.scale);
  hipLaunchKernelGGL(reduce_partials_kernel, g2, dim3(256), 0, st, partial, LNP_WAVES, 2 * a.d, a.d, a.d, a.out,
                     a.beta_off, a.scale);
  return hipGetLastError();
}

}  // namespace mg
