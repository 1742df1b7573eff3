// Fused softmax attention over all (group, sequence, head) triples of a batched layer
// step, forward and backward, without materialising the score matrix in HBM.
//
// Generic kernels (any operand type, d_head <= 128, any sequence length):
// one 64-lane wavefront owns a query (or key) row; keys (queries) are staged in LDS in
// chunks of 64; scores are one per lane, softmax statistics are wavefront reductions,
// and the value accumulation puts one feature per lane.  Online softmax keeps the
// running maximum m and denominator l per row; lse = m + log l is kept for the backward.
//
// Backward (no atomics, deterministic):
//   pass 1, per query row i : D_i = <dO_i, O_i>,  p_ij = exp(s_ij - lse_i),
//                             dA_ij = p_ij (dO_i.V_j - D_i),  dQ_i = scale * sum_j dA_ij K_j
//   pass 2, per key row j   : dV_j = sum_i p_ij dO_i,  dK_j = scale * sum_i dA_ij Q_i
#include "common.h"
#include "kernels.h"
#include "prof.h"

namespace mg {

constexpr int AT_CH = 64;      // rows staged per chunk
constexpr int AT_RB = 16;      // rows owned by a block (4 waves x 4 rows)

template <typename T>
__device__ __forceinline__ void stage_rows(float* dst, int ld, const T* src, long row_stride, int row0,
                                           int nrows_valid, int dh, float scale) {
  // dst[r][c] = scale * src[(row0+r)*row_stride + c] for r < AT_CH (zero beyond nrows_valid)
  const int per_row = dh >> 2;
  for (int i = threadIdx.x; i < AT_CH * per_row; i += blockDim.x) {
    const int r = i / per_row, c = (i - r * per_row) * 4;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (r < nrows_valid) v = load4<T>(src + (long)(row0 + r) * row_stride + c);
    float* p = dst + r * ld + c;
    p[0] = v[0] * scale; p[1] = v[1] * scale; p[2] = v[2] * scale; p[3] = v[3] * scale;
  }
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) attn_fwd_simple_kernel(const AttnArgs a) {
  extern __shared__ float sm[];
  const int dh = a.dh, ld = dh + 1;
  float* Ks = sm;                         // [64][ld]
  float* Vs = Ks + AT_CH * ld;            // [64][ld]
  float* Qs = Vs + AT_CH * ld;            // [16][dh]   (pre-scaled)
  float* Ps = Qs + AT_RB * dh;            // [4 waves][64]
  const int g = blockIdx.z;
  const int b = blockIdx.y / a.H, h = blockIdx.y - b * a.H;
  const int q0 = blockIdx.x * AT_RB;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float scale = rsqrtf((float)dh);

  const T* Q = reinterpret_cast<const T*>(a.q) + a.q_slots.of(g) * a.q_slot_stride +
               (long)b * a.Sq * a.q_row_stride + h * dh;
  const T* K = reinterpret_cast<const T*>(a.k) + a.k_slots.of(g) * a.k_slot_stride +
               (long)b * a.Sk * a.k_row_stride + h * dh;
  const T* V = reinterpret_cast<const T*>(a.v) + a.k_slots.of(g) * a.v_slot_stride +
               (long)b * a.Sk * a.v_row_stride + h * dh;

  // stage this block's query rows (scaled by 1/sqrt(dh))
  for (int i = threadIdx.x; i < AT_RB * dh; i += 256) {
    const int r = i / dh, c = i - r * dh;
    const int qi = q0 + r;
    Qs[i] = qi < a.Sq ? to_f<T>(Q[(long)qi * a.q_row_stride + c]) * scale : 0.f;
  }

  float m[4], l[4], acc[4][2];
#pragma unroll
  for (int r = 0; r < 4; ++r) { m[r] = -INFINITY; l[r] = 0.f; acc[r][0] = acc[r][1] = 0.f; }

  const int q_last = min(q0 + AT_RB, a.Sq) - 1;
  const int k_end = a.causal ? min(a.Sk, q_last + 1) : a.Sk;
  for (int k0 = 0; k0 < k_end; k0 += AT_CH) {
    __syncthreads();
    const int nv = min(AT_CH, a.Sk - k0);
    stage_rows<T>(Ks, ld, K, a.k_row_stride, k0, nv, dh, 1.f);
    stage_rows<T>(Vs, ld, V, a.v_row_stride, k0, nv, dh, 1.f);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int qr = wave * 4 + r, qi = q0 + qr;
      if (qi >= a.Sq) continue;                       // wave-uniform
      if (a.causal && k0 > qi) continue;
      const int kj = k0 + lane;
      float s = 0.f;
      const float* qrow = Qs + qr * dh;
      const float* krow = Ks + lane * ld;
      for (int c = 0; c < dh; ++c) s = fmaf(qrow[c], krow[c], s);
      const bool valid = kj < a.Sk && (!a.causal || kj <= qi);
      s = valid ? s : -INFINITY;
      const float mn = fmaxf(m[r], wave_max(s));
      const float p = valid ? __expf(s - mn) : 0.f;
      const float corr = __expf(m[r] - mn);          // exp(-inf) = 0 on the first chunk
      l[r] = l[r] * corr + wave_sum(p);
      m[r] = mn;
      Ps[wave * 64 + lane] = p;                       // same-wave exchange through LDS
      float a0 = acc[r][0] * corr, a1 = acc[r][1] * corr;
      const float* pw = Ps + wave * 64;
      if (lane < dh) {
        for (int j = 0; j < AT_CH; ++j) a0 = fmaf(pw[j], Vs[j * ld + lane], a0);
      }
      if (lane + 64 < dh) {
        for (int j = 0; j < AT_CH; ++j) a1 = fmaf(pw[j], Vs[j * ld + lane + 64], a1);
      }
      acc[r][0] = a0; acc[r][1] = a1;
    }
  }
  T* O = reinterpret_cast<T*>(a.o) + a.o_slots.of(g) * a.o_slot_stride + (long)b * a.Sq * a.o_row_stride + h * dh;
  float* lse = a.lse ? a.lse + a.lse_slots.of(g) * a.lse_slot_stride + ((long)b * a.H + h) * a.Sq : nullptr;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int qi = q0 + wave * 4 + r;
    if (qi >= a.Sq) continue;
    const float inv = 1.0f / l[r];
    if (lane < dh) O[(long)qi * a.o_row_stride + lane] = from_f<T>(acc[r][0] * inv);
    if (lane + 64 < dh) O[(long)qi * a.o_row_stride + lane + 64] = from_f<T>(acc[r][1] * inv);
    if (lse && lane == 0) lse[qi] = m[r] + __logf(l[r]);
  }
}

// ---------------------------------------------------------------------------
// backward pass 1: per query row  ->  D, dQ
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_dq_simple_kernel(const AttnArgs a) {
  extern __shared__ float sm[];
  const int dh = a.dh, ld = dh + 1;
  float* Ks = sm;                         // [64][ld]
  float* Vs = Ks + AT_CH * ld;            // [64][ld]
  float* Qs = Vs + AT_CH * ld;            // [16][dh]  pre-scaled q
  float* dOs = Qs + AT_RB * dh;           // [16][dh]
  float* Ps = dOs + AT_RB * dh;           // [4][64]
  const int g = blockIdx.z;
  const int b = blockIdx.y / a.H, h = blockIdx.y - b * a.H;
  const int q0 = blockIdx.x * AT_RB;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float scale = rsqrtf((float)dh);

  const T* Q = reinterpret_cast<const T*>(a.q) + a.q_slots.of(g) * a.q_slot_stride +
               (long)b * a.Sq * a.q_row_stride + h * dh;
  const T* K = reinterpret_cast<const T*>(a.k) + a.k_slots.of(g) * a.k_slot_stride +
               (long)b * a.Sk * a.k_row_stride + h * dh;
  const T* V = reinterpret_cast<const T*>(a.v) + a.k_slots.of(g) * a.v_slot_stride +
               (long)b * a.Sk * a.v_row_stride + h * dh;
  const T* O = reinterpret_cast<const T*>(a.o) + a.o_slots.of(g) * a.o_slot_stride +
               (long)b * a.Sq * a.o_row_stride + h * dh;
  const T* dO = reinterpret_cast<const T*>(a.dO) + a.do_slots.of(g) * a.do_slot_stride +
                (long)b * a.Sq * a.do_row_stride + h * dh;
  const float* lse = a.lse + a.lse_slots.of(g) * a.lse_slot_stride + ((long)b * a.H + h) * a.Sq;
  float* Dv = a.D + a.D_slots.of(g) * a.D_slot_stride + ((long)b * a.H + h) * a.Sq;

  for (int i = threadIdx.x; i < AT_RB * dh; i += 256) {
    const int r = i / dh, c = i - r * dh;
    const int qi = q0 + r;
    const bool ok = qi < a.Sq;
    Qs[i] = ok ? to_f<T>(Q[(long)qi * a.q_row_stride + c]) * scale : 0.f;
    dOs[i] = ok ? to_f<T>(dO[(long)qi * a.do_row_stride + c]) : 0.f;
  }
  __syncthreads();
  // D_i = <dO_i, O_i>
  float Drow[4], lrow[4], acc[4][2];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int qr = wave * 4 + r, qi = q0 + qr;
    float s = 0.f;
    if (qi < a.Sq) {
      if (lane < dh) s += dOs[qr * dh + lane] * to_f<T>(O[(long)qi * a.o_row_stride + lane]);
      if (lane + 64 < dh) s += dOs[qr * dh + lane + 64] * to_f<T>(O[(long)qi * a.o_row_stride + lane + 64]);
    }
    Drow[r] = wave_sum(s);
    lrow[r] = qi < a.Sq ? lse[qi] : 0.f;
    if (qi < a.Sq && lane == 0) Dv[qi] = Drow[r];
    acc[r][0] = acc[r][1] = 0.f;
  }

  const int q_last = min(q0 + AT_RB, a.Sq) - 1;
  const int k_end = a.causal ? min(a.Sk, q_last + 1) : a.Sk;
  for (int k0 = 0; k0 < k_end; k0 += AT_CH) {
    __syncthreads();
    const int nv = min(AT_CH, a.Sk - k0);
    stage_rows<T>(Ks, ld, K, a.k_row_stride, k0, nv, dh, 1.f);
    stage_rows<T>(Vs, ld, V, a.v_row_stride, k0, nv, dh, 1.f);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int qr = wave * 4 + r, qi = q0 + qr;
      if (qi >= a.Sq) continue;
      if (a.causal && k0 > qi) continue;
      const int kj = k0 + lane;
      float s = 0.f, dp = 0.f;
      const float* qrow = Qs + qr * dh;
      const float* drow = dOs + qr * dh;
      const float* krow = Ks + lane * ld;
      const float* vrow = Vs + lane * ld;
      for (int c = 0; c < dh; ++c) { s = fmaf(qrow[c], krow[c], s); dp = fmaf(drow[c], vrow[c], dp); }
      const bool valid = kj < a.Sk && (!a.causal || kj <= qi);
      const float p = valid ? __expf(s - lrow[r]) : 0.f;
      Ps[wave * 64 + lane] = p * (dp - Drow[r]);      // dA_ij
      const float* pw = Ps + wave * 64;
      float a0 = acc[r][0], a1 = acc[r][1];
      if (lane < dh) for (int j = 0; j < AT_CH; ++j) a0 = fmaf(pw[j], Ks[j * ld + lane], a0);
      if (lane + 64 < dh) for (int j = 0; j < AT_CH; ++j) a1 = fmaf(pw[j], Ks[j * ld + lane + 64], a1);
      acc[r][0] = a0; acc[r][1] = a1;
    }
  }
  T* dQ = reinterpret_cast<T*>(a.dq) + a.dqkv_slots.of(g) * a.dqkv_slot_stride +
          (long)b * a.Sq * a.dqkv_row_stride + h * dh;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int qi = q0 + wave * 4 + r;
    if (qi >= a.Sq) continue;
    if (lane < dh) dQ[(long)qi * a.dqkv_row_stride + lane] = from_f<T>(acc[r][0] * scale);
    if (lane + 64 < dh) dQ[(long)qi * a.dqkv_row_stride + lane + 64] = from_f<T>(acc[r][1] * scale);
  }
}

// ---------------------------------------------------------------------------
// backward pass 2: per key row  ->  dK, dV
// ---------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_dkv_simple_kernel(const AttnArgs a) {
  extern __shared__ float sm[];
  const int dh = a.dh, ld = dh + 1;
  float* Qc = sm;                         // [64][ld]  pre-scaled q chunk
  float* dOc = Qc + AT_CH * ld;           // [64][ld]
  float* Kr = dOc + AT_CH * ld;           // [16][dh]  this block's key rows
  float* Vr = Kr + AT_RB * dh;            // [16][dh]
  float* Ps = Vr + AT_RB * dh;            // [4][64]  p
  float* As = Ps + 4 * 64;                // [4][64]  dA
  float* Lc = As + 4 * 64;                // [64] lse chunk
  float* Dc = Lc + AT_CH;                 // [64] D chunk
  const int g = blockIdx.z;
  const int b = blockIdx.y / a.H, h = blockIdx.y - b * a.H;
  const int j0 = blockIdx.x * AT_RB;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float scale = rsqrtf((float)dh);

  const T* Q = reinterpret_cast<const T*>(a.q) + a.q_slots.of(g) * a.q_slot_stride +
               (long)b * a.Sq * a.q_row_stride + h * dh;
  const T* K = reinterpret_cast<const T*>(a.k) + a.k_slots.of(g) * a.k_slot_stride +
               (long)b * a.Sk * a.k_row_stride + h * dh;
  const T* V = reinterpret_cast<const T*>(a.v) + a.k_slots.of(g) * a.v_slot_stride +
               (long)b * a.Sk * a.v_row_stride + h * dh;
  const T* dO = reinterpret_cast<const T*>(a.dO) + a.do_slots.of(g) * a.do_slot_stride +
                (long)b * a.Sq * a.do_row_stride + h * dh;
  const float* lse = a.lse + a.lse_slots.of(g) * a.lse_slot_stride + ((long)b * a.H + h) * a.Sq;
  const float* Dv = a.D + a.D_slots.of(g) * a.D_slot_stride + ((long)b * a.H + h) * a.Sq;

  for (int i = threadIdx.x; i < AT_RB * dh; i += 256) {
    const int r = i / dh, c = i - r * dh;
    const int kj = j0 + r;
    const bool ok = kj < a.Sk;
    Kr[i] = ok ? to_f<T>(K[(long)kj * a.k_row_stride + c]) : 0.f;
    Vr[i] = ok ? to_f<T>(V[(long)kj * a.v_row_stride + c]) : 0.f;
  }
  float dk[4][2], dv[4][2];
#pragma unroll
  for (int r = 0; r < 4; ++r) { dk[r][0] = dk[r][1] = dv[r][0] = dv[r][1] = 0.f; }

  // causal: key j only sees queries i >= j
  const int i_begin = a.causal ? (j0 / AT_CH) * AT_CH : 0;
  for (int i0 = i_begin; i0 < a.Sq; i0 += AT_CH) {
    __syncthreads();
    const int nv = min(AT_CH, a.Sq - i0);
    stage_rows<T>(Qc, ld, Q, a.q_row_stride, i0, nv, dh, scale);
    stage_rows<T>(dOc, ld, dO, a.do_row_stride, i0, nv, dh, 1.f);
    if (threadIdx.x < AT_CH) {
      const int qi = i0 + threadIdx.x;
      Lc[threadIdx.x] = qi < a.Sq ? lse[qi] : 0.f;
      Dc[threadIdx.x] = qi < a.Sq ? Dv[qi] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int kr = wave * 4 + r, kj = j0 + kr;
      if (kj >= a.Sk) continue;
      const int qi = i0 + lane;
      float s = 0.f, dp = 0.f;
      const float* krow = Kr + kr * dh;
      const float* vrow = Vr + kr * dh;
      const float* qrow = Qc + lane * ld;
      const float* drow = dOc + lane * ld;
      for (int c = 0; c < dh; ++c) { s = fmaf(qrow[c], krow[c], s); dp = fmaf(drow[c], vrow[c], dp); }
      const bool valid = qi < a.Sq && (!a.causal || kj <= qi);
      const float p = valid ? __expf(s - Lc[lane]) : 0.f;
      Ps[wave * 64 + lane] = p;
      As[wave * 64 + lane] = p * (dp - Dc[lane]);
      const float* pw = Ps + wave * 64;
      const float* aw = As + wave * 64;
      if (lane < dh) {
        float v0 = dv[r][0], k0v = dk[r][0];
        for (int i = 0; i < AT_CH; ++i) {
          v0 = fmaf(pw[i], dOc[i * ld + lane], v0);
          k0v = fmaf(aw[i], Qc[i * ld + lane], k0v);      // Qc is pre-scaled: includes 1/sqrt(dh)
        }
        dv[r][0] = v0; dk[r][0] = k0v;
      }
      if (lane + 64 < dh) {
        float v1 = dv[r][1], k1v = dk[r][1];
        for (int i = 0; i < AT_CH; ++i) {
          v1 = fmaf(pw[i], dOc[i * ld + lane + 64], v1);
          k1v = fmaf(aw[i], Qc[i * ld + lane + 64], k1v);
        }
        dv[r][1] = v1; dk[r][1] = k1v;
      }
    }
  }
  const long kv_rs = a.dkv_row_stride ? a.dkv_row_stride : a.dqkv_row_stride;
  const long kv_ss = a.dkv_slot_stride ? a.dkv_slot_stride : a.dqkv_slot_stride;
  T* dK = reinterpret_cast<T*>(a.dk) + a.dqkv_slots.of(g) * kv_ss + (long)b * a.Sk * kv_rs + h * dh;
  T* dV = reinterpret_cast<T*>(a.dv) + a.dqkv_slots.of(g) * kv_ss + (long)b * a.Sk * kv_rs + h * dh;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int kj = j0 + wave * 4 + r;
    if (kj >= a.Sk) continue;
    if (lane < dh) {
      dK[(long)kj * kv_rs + lane] = from_f<T>(dk[r][0]);
      dV[(long)kj * kv_rs + lane] = from_f<T>(dv[r][0]);
    }
    if (lane + 64 < dh) {
      dK[(long)kj * kv_rs + lane + 64] = from_f<T>(dk[r][1]);
      dV[(long)kj * kv_rs + lane + 64] = from_f<T>(dv[r][1]);
    }
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
bool attn_mfma_supported(const AttnArgs& a);
hipError_t attn_fwd_mfma(const AttnArgs& a, hipStream_t st);
hipError_t attn_bwd_mfma(const AttnArgs& a, hipStream_t st);

static int g_attn_force_simple = 0;
void attn_force_simple(int on) { g_attn_force_simple = on; }

template <typename K>
static hipError_t set_smem(K kern, size_t smem) {
  if (smem <= 48 * 1024) return hipSuccess;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)smem);
}

template <typename T>
static hipError_t attn_fwd_simple(const AttnArgs& a, hipStream_t st) {
  const int ld = a.dh + 1;
  const size_t smem = sizeof(float) * (2 * AT_CH * ld + AT_RB * a.dh + 4 * 64);
  hipError_t e = set_smem(attn_fwd_simple_kernel<T>, smem);
  if (e != hipSuccess) return e;
  dim3 grid((a.Sq + AT_RB - 1) / AT_RB, a.B * a.H, a.n_groups);
  hipLaunchKernelGGL(attn_fwd_simple_kernel<T>, grid, dim3(256), smem, st, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t attn_bwd_simple(const AttnArgs& a, hipStream_t st) {
  const int ld = a.dh + 1;
  {
    const size_t smem = sizeof(float) * (2 * AT_CH * ld + 2 * AT_RB * a.dh + 4 * 64);
    hipError_t e = set_smem(attn_bwd_dq_simple_kernel<T>, smem);
    if (e != hipSuccess) return e;
    dim3 grid((a.Sq + AT_RB - 1) / AT_RB, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL(attn_bwd_dq_simple_kernel<T>, grid, dim3(256), smem, st, a);
  }
  if (a.dk) {                         // dK, dV pass (skipped when only dQ is wanted)
    const size_t smem = sizeof(float) * (2 * AT_CH * ld + 2 * AT_RB * a.dh + 8 * 64 + 2 * AT_CH);
    hipError_t e = set_smem(attn_bwd_dkv_simple_kernel<T>, smem);
    if (e != hipSuccess) return e;
    dim3 grid((a.Sk + AT_RB - 1) / AT_RB, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL(attn_bwd_dkv_simple_kernel<T>, grid, dim3(256), smem, st, a);
  }
  return hipGetLastError();
}

hipError_t launch_attn_fwd(const AttnArgs& a, bool is_bf16, hipStream_t st) {
  if (a.n_groups <= 0) return hipSuccess;
  if (a.dh > 128 || (a.dh & 3)) return hipErrorInvalidValue;
  const double heads = (double)a.n_groups * a.B * a.H, esz = is_bf16 ? 2 : 4;
  const double pairs = a.causal ? 0.5 * a.Sq * (a.Sk + 1.0) : (double)a.Sq * a.Sk;   // unmasked scores
  ProfScope ps(PC_ATTN_FWD, heads * pairs * a.dh * 4.0, heads * (2.0 * a.Sq + 2.0 * a.Sk) * a.dh * esz, st);
  if (is_bf16 && !g_attn_force_simple && attn_mfma_supported(a)) return attn_fwd_mfma(a, st);
  return is_bf16 ? attn_fwd_simple<bf16>(a, st) : attn_fwd_simple<float>(a, st);
}

hipError_t launch_attn_bwd(const AttnArgs& a, bool is_bf16, hipStream_t st) {
  if (a.n_groups <= 0) return hipSuccess;
  if (a.dh > 128 || (a.dh & 3)) return hipErrorInvalidValue;
  const double heads = (double)a.n_groups * a.B * a.H, esz = is_bf16 ? 2 : 4;
  const double pairs = a.causal ? 0.5 * a.Sq * (a.Sk + 1.0) : (double)a.Sq * a.Sk;
  // recompute scores + dP, dV, dQ, dK: five contractions over the unmasked pairs
  ProfScope ps(PC_ATTN_BWD, heads * pairs * a.dh * 10.0, heads * (4.0 * a.Sq + 4.0 * a.Sk) * a.dh * esz, st);
  if (is_bf16 && !g_attn_force_simple && attn_mfma_supported(a)) return attn_bwd_mfma(a, st);
  return is_bf16 ? attn_bwd_simple<bf16>(a, st) : attn_bwd_simple<float>(a, st);
}

}  // namespace mg
