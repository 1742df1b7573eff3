// Interval-batched grouped GEMM  C_g[m,n] = sum_k A_g[m,k] * W_g[n,k]  with fused
// epilogues, one launch for all groups of an F-/C-relaxation sweep; every group has
// its own weight matrix (the layer of its coarse interval), found through the
// parameter pointer table.
//
// Two kernels:
//  * gemm_mfma  : bf16 operands, fp32 accumulate on the 32x32x16 MFMA of gfx950.
//                 Block tile BM x BN x 64 staged through double-buffered, padded LDS;
//                 (BM/WM) x (BN/WN) per 64-lane wavefront.  The weight fragment is
//                 fed as the first MFMA operand so that each lane ends up with 4
//                 consecutive output columns per register quad (vector stores).
//  * gemm_simple: any operand type (fp32 path and odd shapes), LDS-tiled FMA.
#include "common.h"
#include "kernels.h"
#include "prof.h"

namespace mg {

// ---------------------------------------------------------------------------
// epilogue on 4 consecutive columns n..n+3 of row m of group g
// ---------------------------------------------------------------------------
template <int EPI, typename TO>
__device__ __forceinline__ void epilogue4(const GemmArgs& a, int g, const char* pblock, int m, int n,
                                          f32x4 acc) {
  if (a.bias_off >= 0) {
    const float* bias = reinterpret_cast<const float*>(a.bias.at(g) + a.bias_off);
    acc += *reinterpret_cast<const f32x4*>(bias + n);
  }
  (void)pblock;
  const long idx = (long)m * a.N + n;
  if constexpr (EPI == EPI_STORE) {
    TO* out = reinterpret_cast<TO*>(a.out) + a.out_slots.of(g) * a.out_slot_stride;
    store4<TO>(out + idx, acc);
  } else if constexpr (EPI == EPI_STORE_F32) {
    float* out = reinterpret_cast<float*>(a.out) + a.out_slots.of(g) * a.out_slot_stride;
    store4<float>(out + idx, acc);
  } else if constexpr (EPI == EPI_GELU) {
    TO* out = reinterpret_cast<TO*>(a.out) + a.out_slots.of(g) * a.out_slot_stride;
    if (a.aux) {
      TO* z = reinterpret_cast<TO*>(a.aux) + a.aux_slots.of(g) * a.aux_slot_stride;
      store4<TO>(z + idx, acc);
    }
    f32x4 y = {gelu_f(acc[0]), gelu_f(acc[1]), gelu_f(acc[2]), gelu_f(acc[3])};
    store4<TO>(out + idx, y);
  } else if constexpr (EPI == EPI_DGELU) {
    TO* out = reinterpret_cast<TO*>(a.out) + a.out_slots.of(g) * a.out_slot_stride;
    const TO* z = reinterpret_cast<const TO*>(a.aux) + a.aux_slots.of(g) * a.aux_slot_stride;
    f32x4 zz = load4<TO>(z + idx);
    f32x4 y = {acc[0] * gelu_prime_f(zz[0]), acc[1] * gelu_prime_f(zz[1]),
               acc[2] * gelu_prime_f(zz[2]), acc[3] * gelu_prime_f(zz[3])};
    store4<TO>(out + idx, y);
  } else if constexpr (EPI == EPI_RESID_INNER) {
    float* out = reinterpret_cast<float*>(a.out) + a.out_slots.of(g) * a.out_slot_stride;
    if (a.base) acc += *reinterpret_cast<const f32x4*>(a.base + a.base_slots.of(g) * a.base_slot_stride + idx);
    store4<float>(out + idx, acc);
  } else if constexpr (EPI == EPI_RESID_OUTER) {
    const float* ybar = reinterpret_cast<const float*>(a.aux) + a.aux_slots.of(g) * a.aux_slot_stride;
    f32x4 x = *reinterpret_cast<const f32x4*>(a.X.at(g) + idx);
    f32x4 yb = *reinterpret_cast<const f32x4*>(ybar + idx);
    f32x4 r = x + a.hstep * (yb + acc);
    if (a.RHS.present()) r += *reinterpret_cast<const f32x4*>(a.RHS.at(g) + idx);
    store4<float>(a.OUT.at(g) + idx, r);
  }
}

// ---------------------------------------------------------------------------
// MFMA kernel
// ---------------------------------------------------------------------------
constexpr int GEMM_BK = 64;
constexpr int GEMM_LDK = GEMM_BK + 8;   // padded LDS row (144 B): conflict-free 16-byte fragment reads

template <int BM, int BN, int WM, int WN, int EPI, typename TO>
__global__ void __launch_bounds__(WM * WN * 64)
gemm_mfma_kernel(const GemmArgs a, int tiles_m, int tiles_n, int total_tiles, int per_xcd) {
  constexpr int NT = WM * WN * 64;
  constexpr int WTM = BM / WM, WTN = BN / WN;      // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;      // 32x32 MFMA tiles per wave
  constexpr int A_CH = BM * (GEMM_BK / 8) / NT;    // 16-byte chunks per thread
  constexpr int B_CH = BN * (GEMM_BK / 8) / NT;
  static_assert(BM * (GEMM_BK / 8) % NT == 0 && BN * (GEMM_BK / 8) % NT == 0, "tile/threads");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16* As = reinterpret_cast<bf16*>(smem_raw);                   // [2][BM][LDK]
  bf16* Bs = As + 2 * BM * GEMM_LDK;                              // [2][BN][LDK]

  // XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, so give each
  // XCD one contiguous range of tiles (neighbouring tiles share an activation row panel and
  // the group's weight matrix in that XCD's L2).
  const int pid = blockIdx.x;
  const int tile = (pid & 7) * per_xcd + (pid >> 3);
  if (tile >= total_tiles) return;
  const int tiles_per_group = tiles_m * tiles_n;
  const int g = tile / tiles_per_group;
  const int tg = tile - g * tiles_per_group;
  const int tm = tg / tiles_n, tn = tg - tm * tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;

  const bf16* A = reinterpret_cast<const bf16*>(a.A) + a.a_slots.of(g) * a.a_slot_stride;
  const char* pblock = a.B.at(g);
  const bf16* B = reinterpret_cast<const bf16*>(pblock + a.b_off);
  const int K = a.K, M = a.M;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  bf16x8 ra[A_CH], rb[B_CH];
  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = tid + i * NT;
      const int row = c >> 3, kc = c & 7;
      int gm = m0 + row;
      gm = gm < M ? gm : M - 1;                     // ragged tail: clamp (never stored)
      ra[i] = *reinterpret_cast<const bf16x8*>(A + (long)gm * K + k0 + kc * 8);
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int c = tid + i * NT;
      const int row = c >> 3, kc = c & 7;
      rb[i] = *reinterpret_cast<const bf16x8*>(B + (long)(n0 + row) * K + k0 + kc * 8);
    }
  };
  auto sstore = [&](int buf) {
    bf16* as = As + buf * BM * GEMM_LDK;
    bf16* bs = Bs + buf * BN * GEMM_LDK;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = tid + i * NT;
      *reinterpret_cast<bf16x8*>(as + (c >> 3) * GEMM_LDK + (c & 7) * 8) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int c = tid + i * NT;
      *reinterpret_cast<bf16x8*>(bs + (c >> 3) * GEMM_LDK + (c & 7) * 8) = rb[i];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = K / GEMM_BK;
  gload(0);
  sstore(0);
  __syncthreads();
  const int lr = lane & 31, lk = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) gload((kt + 1) * GEMM_BK);
    const bf16* as = As + buf * BM * GEMM_LDK + (wm0 + lr) * GEMM_LDK + lk * 8;
    const bf16* bs = Bs + buf * BN * GEMM_LDK + (wn0 + lr) * GEMM_LDK + lk * 8;
#pragma unroll
    for (int ks = 0; ks < GEMM_BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * GEMM_LDK + ks * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * GEMM_LDK + ks * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) sstore(buf ^ 1);
    __syncthreads();
  }

  // acc[i][j] register 4q+r of lane l  =  C[m = wm0+32i + l%32][n = wn0+32j + 8q + 4*(l/32) + r]
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm0 + i * 32 + lr;
    if (m < M) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + wn0 + j * 32 + q * 8 + lk * 4;
          f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          epilogue4<EPI, TO>(a, g, pblock, m, n, v);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// generic kernel: 64x64x16 tile, 256 threads, 4x4 outputs per thread
// ---------------------------------------------------------------------------
template <typename TA, int EPI, typename TO>
__global__ void __launch_bounds__(256)
gemm_simple_kernel(const GemmArgs a, int tiles_m, int tiles_n) {
  constexpr int BT = 64, BKS = 16, LD = BT + 4;
  __shared__ float As[BKS][LD];
  __shared__ float Bs[BKS][LD];
  const int g = blockIdx.z;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x - tm * tiles_n;
  const int m0 = tm * BT, n0 = tn * BT;
  const TA* A = reinterpret_cast<const TA*>(a.A) + a.a_slots.of(g) * a.a_slot_stride;
  const char* pblock = a.B.at(g);
  const TA* B = reinterpret_cast<const TA*>(pblock + a.b_off);
  const int M = a.M, N = a.N, K = a.K;
  const int tid = threadIdx.x;
  const int lrow = tid >> 2, lk = (tid & 3) * 4;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BKS) {
    f32x4 va = {0, 0, 0, 0}, vb = {0, 0, 0, 0};
    if (m0 + lrow < M && k0 + lk < K) va = load4<TA>(A + (long)(m0 + lrow) * K + k0 + lk);
    if (n0 + lrow < N && k0 + lk < K) vb = load4<TA>(B + (long)(n0 + lrow) * K + k0 + lk);
#pragma unroll
    for (int i = 0; i < 4; ++i) { As[lk + i][lrow] = va[i]; Bs[lk + i][lrow] = vb[i]; }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BKS; ++k) {
      f32x4 x = *reinterpret_cast<const f32x4*>(&As[k][ty * 4]);
      f32x4 y = *reinterpret_cast<const f32x4*>(&Bs[k][tx * 4]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(x[i], y[j], acc[i][j]);
    }
    __syncthreads();
  }
  const int n = n0 + tx * 4;
  if (n < N) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + ty * 4 + i;
      if (m < M) {
        f32x4 v = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
        epilogue4<EPI, TO>(a, g, pblock, m, n, v);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------
static int g_force_simple = 0;
void gemm_force_simple(int on) { g_force_simple = on; }

template <int BM, int BN, int WM, int WN, int EPI>
static hipError_t launch_mfma(const GemmArgs& a, hipStream_t st) {
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = a.N / BN;
  const int total = tiles_m * tiles_n * a.n_groups;
  const int per_xcd = (total + 7) / 8;
  const size_t smem = (size_t)2 * (BM + BN) * GEMM_LDK * sizeof(bf16);
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, EPI, bf16>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(WM * WN * 64), smem, st, a, tiles_m, tiles_n, total,
                     per_xcd);
  return hipGetLastError();
}

template <typename TA, int EPI>
static hipError_t launch_simple(const GemmArgs& a, hipStream_t st) {
  const int tiles_m = (a.M + 63) / 64, tiles_n = (a.N + 63) / 64;
  hipLaunchKernelGGL((gemm_simple_kernel<TA, EPI, TA>), dim3(tiles_m * tiles_n, 1, a.n_groups), dim3(256), 0,
                     st, a, tiles_m, tiles_n);
  return hipGetLastError();
}

// algorithmic HBM bytes of one grouped GEMM launch: operands once, outputs once, epilogue operands once
template <int EPI>
static double gemm_bytes(const GemmArgs& a, double esz) {
  const double G = a.n_groups, MN = (double)a.M * a.N;
  double b = G * ((a.a_slot_stride ? 1.0 : 1.0 / G) * a.M * a.K * esz + (double)a.N * a.K * esz);
  if (EPI == EPI_STORE) b += G * MN * esz;
  if (EPI == EPI_GELU) b += G * MN * esz * (a.aux ? 2 : 1);
  if (EPI == EPI_DGELU) b += G * MN * esz * 2;
  if (EPI == EPI_STORE_F32) b += G * MN * 4;
  if (EPI == EPI_RESID_INNER) b += G * MN * 4 * (a.base ? 2 : 1);
  if (EPI == EPI_RESID_OUTER) b += G * MN * 4 * (a.RHS.present() ? 4 : 3);
  return b;
}

template <int EPI>
static hipError_t launch_epi(const GemmArgs& a, bool is_bf16, hipStream_t st) {
  if (a.n_groups <= 0 || a.M <= 0) return hipSuccess;
  const double flops = 2.0 * a.n_groups * a.M * (double)a.N * a.K;
  const bool mfma_ok = is_bf16 && !g_force_simple && (a.K % GEMM_BK == 0) && (a.N % 128 == 0);
  ProfScope ps(mfma_ok ? PC_GEMM_MFMA + EPI : PC_GEMM_SIMPLE, flops, gemm_bytes<EPI>(a, is_bf16 ? 2 : 4), st);
  if (!is_bf16) return launch_simple<float, EPI>(a, st);
  if (!mfma_ok) return launch_simple<bf16, EPI>(a, st);
  return launch_mfma<128, 128, 2, 2, EPI>(a, st);
}

hipError_t launch_gemm(const GemmArgs& a, int epi, bool is_bf16, hipStream_t st) {
  switch (epi) {
    case EPI_STORE: return launch_epi<EPI_STORE>(a, is_bf16, st);
    case EPI_GELU: return launch_epi<EPI_GELU>(a, is_bf16, st);
    case EPI_RESID_INNER: return launch_epi<EPI_RESID_INNER>(a, is_bf16, st);
    case EPI_RESID_OUTER: return launch_epi<EPI_RESID_OUTER>(a, is_bf16, st);
    case EPI_DGELU: return launch_epi<EPI_DGELU>(a, is_bf16, st);
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32>(a, is_bf16, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace mg
