// Interval-batched grouped GEMM  C_g[m,n] = sum_k A_g[m,k] * W_g[n,k]  with fused
// epilogues, one launch for all groups of an F-/C-relaxation sweep; every group has
// its own weight matrix (the layer of its coarse interval), found through the
// parameter pointer table.
//
// Three kernels:
//  * gemm_mfma    : bf16 operands, fp32 accumulate on the 32x32x16 MFMA of gfx950; operands
//                   stream global -> LDS directly through a ring of k-tiles, see below.
//  * gemm_f32_mfma: fp32 operands on the 32x32x2 fp32 MFMA (the fp32 configuration).
//  * gemm_simple  : any operand type and shape, LDS-tiled FMA.
#include <type_traits>

#include "common.h"
#include "kernels.h"
#include "prof.h"

namespace mg {

// ---------------------------------------------------------------------------
// Epilogue.  EpiPtrs holds the launch's epilogue operands resolved for one group; apply4
// finishes 4 consecutive columns n..n+3 of row m (idx = m*N + n) from the accumulated
// products `acc` (bias not yet added).
// ---------------------------------------------------------------------------
struct EpiPtrs {
  const float* bias;          // [N] or null
  void* out;                  // packed output (operand type or fp32)
  void* aux;                  // EPI_GELU: z out (optional); EPI_DGELU: z in; EPI_RESID_OUTER: ybar
  void* aux2;                 // EPI_GELU_BOTH: gelu'(z) out
  const float* base;          // EPI_RESID_INNER: optional addend
  const float* X;             // EPI_RESID_OUTER
  const float* RHS;           // EPI_RESID_OUTER, optional
  float* OUT;                 // EPI_RESID_OUTER
};

template <typename TO>
__device__ __forceinline__ EpiPtrs resolve_epi(const GemmArgs& a, int g, int epi) {
  EpiPtrs p;
  p.bias = a.bias_off >= 0 ? reinterpret_cast<const float*>(a.bias.at(g) + a.bias_off) : nullptr;
  const bool f32_out = epi == EPI_STORE_F32 || epi == EPI_RESID_INNER;
  const long osz = f32_out ? 4 : (long)sizeof(TO);
  p.out = a.out ? static_cast<char*>(a.out) + a.out_slots.of(g) * a.out_slot_stride * osz : nullptr;
  if (a.out_tab.tab) p.out = const_cast<char*>(a.out_tab.at(g)) + a.out_tab_off;
  const long asz = epi == EPI_RESID_OUTER ? 4 : (long)sizeof(TO);
  p.aux = a.aux ? static_cast<char*>(a.aux) + a.aux_slots.of(g) * a.aux_slot_stride * asz : nullptr;
  p.aux2 = a.aux2 ? static_cast<char*>(a.aux2) + a.aux2_slots.of(g) * a.aux2_slot_stride * (long)sizeof(TO) : nullptr;
  p.base = a.base ? a.base + a.base_slots.of(g) * a.base_slot_stride : nullptr;
  p.X = a.X.present() ? a.X.at(g) : nullptr;
  p.RHS = a.RHS.present() ? a.RHS.at(g) : nullptr;
  p.OUT = a.OUT.present() ? a.OUT.at(g) : nullptr;
  return p;
}

// Epilogue operands and outputs are touched once per launch: they are moved with the
// non-temporal hint, so that they do not displace the operand panels that the tiles running
// on an XCD share through its L2.
template <typename T> __device__ __forceinline__ void estore4(T* p, f32x4 v);
template <> __device__ __forceinline__ void estore4<float>(float* p, f32x4 v) { st_stream(reinterpret_cast<f32x4*>(p), v); }
template <> __device__ __forceinline__ void estore4<bf16>(bf16* p, f32x4 v) {
  bf16x4 r = {(bf16)v[0], (bf16)v[1], (bf16)v[2], (bf16)v[3]};
  st_stream(reinterpret_cast<bf16x4*>(p), r);
}
template <typename T> __device__ __forceinline__ f32x4 eload4(const T* p);
template <> __device__ __forceinline__ f32x4 eload4<float>(const float* p) { return ld_stream(reinterpret_cast<const f32x4*>(p)); }
template <> __device__ __forceinline__ f32x4 eload4<bf16>(const bf16* p) {
  bf16x4 v = ld_stream(reinterpret_cast<const bf16x4*>(p));
  f32x4 r = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
  return r;
}

// OPT: what is known at compile time about the optional operands of an epilogue: -1 nothing (tested
// per call), else bit 0 = the first one is there (ybar / base / the pre-activation output), bit 1 =
// RHS is there.  With OPT >= 0 a run of items is straight-line code.
template <int OPT> __device__ __forceinline__ bool has_opt(int bit, const void* p) {
  return OPT < 0 ? p != nullptr : ((OPT >> bit) & 1) != 0;
}

template <int EPI, typename TO, int OPT = -1>
__device__ __forceinline__ void apply4(TO* __restrict__ out_op, float* __restrict__ out_f32,
                                       TO* __restrict__ z_out, const TO* __restrict__ z_in,
                                       TO* __restrict__ g_out,
                                       const float* __restrict__ base, const float* __restrict__ X,
                                       const float* __restrict__ ybar, const float* __restrict__ RHS,
                                       float* __restrict__ OUT, float hstep, float sgn, long idx, f32x4 acc) {
  if constexpr (EPI == EPI_STORE) {
    estore4<TO>(out_op + idx, acc);
  } else if constexpr (EPI == EPI_STORE_F32) {
    estore4<float>(out_f32 + idx, hstep * acc);
  } else if constexpr (EPI == EPI_GELU) {
    if (has_opt<OPT>(0, z_out)) estore4<TO>(z_out + idx, acc);
    f32x4 y = {gelu_t<TO>(acc[0]), gelu_t<TO>(acc[1]), gelu_t<TO>(acc[2]), gelu_t<TO>(acc[3])};
    estore4<TO>(out_op + idx, y);
  } else if constexpr (EPI == EPI_GELU_PRIME) {
    if (has_opt<OPT>(0, z_out)) estore4<TO>(z_out + idx, acc);
    f32x4 y = {gelu_prime_t<TO>(acc[0]), gelu_prime_t<TO>(acc[1]), gelu_prime_t<TO>(acc[2]),
               gelu_prime_t<TO>(acc[3])};
    estore4<TO>(out_op + idx, y);
  } else if constexpr (EPI == EPI_GELU_BOTH) {
    if (has_opt<OPT>(0, z_out)) estore4<TO>(z_out + idx, acc);
    f32x4 y = {gelu_t<TO>(acc[0]), gelu_t<TO>(acc[1]), gelu_t<TO>(acc[2]), gelu_t<TO>(acc[3])};
    estore4<TO>(out_op + idx, y);
    f32x4 dy = {gelu_prime_t<TO>(acc[0]), gelu_prime_t<TO>(acc[1]), gelu_prime_t<TO>(acc[2]),
                gelu_prime_t<TO>(acc[3])};
    estore4<TO>(g_out + idx, dy);
  } else if constexpr (EPI == EPI_DGELU) {
    estore4<TO>(out_op + idx, acc * eload4<TO>(z_in + idx));
  } else if constexpr (EPI == EPI_RESID_INNER) {
    if (has_opt<OPT>(0, base)) acc += eload4<float>(base + idx);
    estore4<float>(out_f32 + idx, acc);
  } else if constexpr (EPI == EPI_RESID_OUTER) {
    f32x4 x = eload4<float>(X + idx);
    if (has_opt<OPT>(0, ybar)) acc += eload4<float>(ybar + idx);
    f32x4 r = x + hstep * acc;
    if (has_opt<OPT>(1, RHS)) {
      // sgn = 1: r + rhs; sgn = -1: rhs - r, each a single rounding of the exact value
      const f32x4 rhs = eload4<float>(RHS + idx);
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = __builtin_fmaf(sgn, r[e], rhs[e]);
    }
    estore4<float>(OUT + idx, r);
  }
}

// 8 consecutive columns of a bf16 output (the epilogues whose operands are all bf16)
__device__ __forceinline__ void store8(bf16* p, f32x4 a, f32x4 b) {
  bf16x8 r = {(bf16)a[0], (bf16)a[1], (bf16)a[2], (bf16)a[3], (bf16)b[0], (bf16)b[1], (bf16)b[2], (bf16)b[3]};
  st_stream(reinterpret_cast<bf16x8*>(p), r);
}
template <int EPI, int OPT = -1>
__device__ __forceinline__ void apply8(bf16* __restrict__ out, bf16* __restrict__ z_out,
                                       const bf16* __restrict__ z_in, bf16* __restrict__ g_out, long idx,
                                       f32x4 a, f32x4 b) {
  if constexpr (EPI == EPI_STORE) {
    store8(out + idx, a, b);
  } else if constexpr (EPI == EPI_GELU) {
    if (has_opt<OPT>(0, z_out)) store8(z_out + idx, a, b);
#pragma unroll
    for (int r = 0; r < 4; ++r) { a[r] = gelu_fast(a[r]); b[r] = gelu_fast(b[r]); }
    store8(out + idx, a, b);
  } else if constexpr (EPI == EPI_GELU_PRIME) {
    if (has_opt<OPT>(0, z_out)) store8(z_out + idx, a, b);
#pragma unroll
    for (int r = 0; r < 4; ++r) { a[r] = gelu_prime_fast(a[r]); b[r] = gelu_prime_fast(b[r]); }
    store8(out + idx, a, b);
  } else if constexpr (EPI == EPI_GELU_BOTH) {
    if (has_opt<OPT>(0, z_out)) store8(z_out + idx, a, b);
    f32x4 da, db;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      da[r] = gelu_prime_fast(a[r]); db[r] = gelu_prime_fast(b[r]);
      a[r] = gelu_fast(a[r]); b[r] = gelu_fast(b[r]);
    }
    store8(out + idx, a, b);
    store8(g_out + idx, da, db);
  } else if constexpr (EPI == EPI_DGELU) {
    const bf16x8 g = ld_stream(reinterpret_cast<const bf16x8*>(z_in + idx));
#pragma unroll
    for (int r = 0; r < 4; ++r) { a[r] *= (float)g[r]; b[r] *= (float)g[4 + r]; }
    store8(out + idx, a, b);
  }
}

// one-off form for the generic kernel
template <int EPI, typename TO>
__device__ __forceinline__ void epilogue4(const EpiPtrs& p, float hstep, float sgn, int N, int m, int n, f32x4 acc) {
  if (p.bias) acc += *reinterpret_cast<const f32x4*>(p.bias + n);
  apply4<EPI, TO>(static_cast<TO*>(p.out), static_cast<float*>(p.out), static_cast<TO*>(p.aux),
                  static_cast<const TO*>(p.aux), static_cast<TO*>(p.aux2), p.base, p.X,
                  static_cast<const float*>(p.aux), p.RHS, p.OUT, hstep, sgn, (long)m * N + n, acc);
}

constexpr int ce_gcd(int a, int b) { return b == 0 ? a : ce_gcd(b, a % b); }

// Whole-tile epilogue of one wavefront of the MFMA kernel.  All operand pointers are
// restrict-qualified parameters of this one function, so that the compiler may hoist the
// loads of later rows above the stores of earlier ones (outputs never alias inputs).
template <int EPI, typename TO, int TM, int TN, bool STAGED>
__device__ __forceinline__ void tile_epilogue(
    f32x16 (&acc)[TM][TN], unsigned char* ep, const float* __restrict__ bias, TO* __restrict__ out_op,
    float* __restrict__ out_f32, TO* __restrict__ z_out, const TO* __restrict__ z_in, TO* __restrict__ g_out,
    const float* __restrict__ base, const float* __restrict__ X, const float* __restrict__ ybar,
    const float* __restrict__ RHS, float* __restrict__ OUT, float hstep, float sgn, int N, int M, int mrow0,
    int ncol0, int lane) {
  constexpr int WTN = TN * 32;
  const int lr = lane & 31, lh = lane >> 5;
  if constexpr (STAGED) {
    constexpr int EP_LD = WTN * 4 + 16;                  // bytes per staged row (padded)
    // A lane finishes CW consecutive columns at a time: 8 where the output is bf16 (16-byte
    // stores: four lanes fill a 64-byte sector, so the memory side never has to read a sector
    // back in order to merge a partial write), 4 where it is fp32.
    constexpr bool WIDE = sizeof(TO) == 2 && (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_DGELU ||
                                              EPI == EPI_GELU_PRIME || EPI == EPI_GELU_BOTH);
    constexpr int CW = WIDE ? 8 : 4;
    constexpr int CI = WTN / CW;                         // items per row
    constexpr int NIT = 32 * CI / 64;                    // items per lane in a 32-row block
    static_assert(32 * CI % 64 == 0, "whole passes over a 32-row block");
    // item e = it*64 + lane is column group e % CI of row e / CI.  A lane's column group
    // repeats with period NB in `it` (1 when CI divides 64): one bias vector per phase.
    constexpr int NB = CI / ce_gcd(64, CI);
    f32x4 bv[NB][CW / 4];
#pragma unroll
    for (int p = 0; p < NB; ++p)
#pragma unroll
      for (int h = 0; h < CW / 4; ++h) {
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        bv[p][h] = bias ? *reinterpret_cast<const f32x4*>(bias + ncol0 + CW * ((p * 64 + lane) % CI) + 4 * h) : z;
      }
    // The bias vectors have landed before the first item uses them; saying so once, outside the
    // row guards below, keeps the per-item waits on them from also waiting for every earlier
    // store (stores count on the same counter), which would serialise the stores of a tile.
    if (bias) __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0)
    // GUARD: the wavefront's tile reaches past row M (ragged last tile of a group): per-row tests.
    // Otherwise the items of a 32-row block are straight-line code, whose operand loads the
    // compiler may issue ahead of the stores of earlier items (outputs never alias inputs).
    auto rows32 = [&](auto guard_tag, auto opt_tag, int i) {
      constexpr bool GUARD = decltype(guard_tag)::value;
      constexpr int OPT = decltype(opt_tag)::value;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *reinterpret_cast<f32x4*>(ep + lr * EP_LD + (32 * j + 8 * q + 4 * lh) * 4) = v;
        }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int e = it * 64 + lane;
        const int row = e / CI, ci = e % CI;
        const unsigned char* src = ep + row * EP_LD + ci * CW * 4;
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(src) + bv[it % NB][0];
        const int m = mrow0 + 32 * i + row;
        const long idx = (long)m * N + ncol0 + CW * ci;
        if constexpr (WIDE) {
          const f32x4 v1 = *reinterpret_cast<const f32x4*>(src + 16) + bv[it % NB][1];
          if (!GUARD || m < M)
            apply8<EPI, OPT>(reinterpret_cast<bf16*>(out_op), reinterpret_cast<bf16*>(z_out),
                             reinterpret_cast<const bf16*>(z_in), reinterpret_cast<bf16*>(g_out), idx, v0, v1);
        } else {
          if (!GUARD || m < M)
            apply4<EPI, TO, OPT>(out_op, out_f32, z_out, z_in, g_out, base, X, ybar, RHS, OUT, hstep, sgn, idx, v0);
        }
      }
    };
    // which optional operands this launch has (uniform over the launch): resolved once, so that
    // the items carry no tests of their own
    constexpr int NOPT = EPI == EPI_RESID_OUTER ? 4
                         : (EPI == EPI_RESID_INNER || EPI == EPI_GELU || EPI == EPI_GELU_PRIME ||
                            EPI == EPI_GELU_BOTH) ? 2 : 1;
    const void* first = EPI == EPI_RESID_OUTER ? static_cast<const void*>(ybar)
                        : EPI == EPI_RESID_INNER ? static_cast<const void*>(base) : static_cast<const void*>(z_out);
    const int opt = NOPT == 1 ? 0 : ((first ? 1 : 0) | (NOPT == 4 && RHS ? 2 : 0));
    auto all_rows = [&](auto guard_tag, auto opt_tag) {
#pragma unroll
      for (int i = 0; i < TM; ++i) rows32(guard_tag, opt_tag, i);
    };
    if (mrow0 + 32 * TM <= M) {                            // wave-uniform
      if (opt == 0) all_rows(std::false_type{}, std::integral_constant<int, 0>{});
      else if (opt == 1) all_rows(std::false_type{}, std::integral_constant<int, NOPT >= 2 ? 1 : 0>{});
      else if (opt == 2) all_rows(std::false_type{}, std::integral_constant<int, NOPT == 4 ? 2 : 0>{});
      else all_rows(std::false_type{}, std::integral_constant<int, NOPT == 4 ? 3 : 0>{});
    } else {
      all_rows(std::true_type{}, std::integral_constant<int, -1>{});
    }
  } else {
    // acc[i][j] register 4q+r of lane l  =  C[m = 32i + l%32][n = 32j + 8q + 4*(l/32) + r]
    f32x4 bv[TN][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        bv[j][q] = bias ? *reinterpret_cast<const f32x4*>(bias + ncol0 + j * 32 + q * 8 + lh * 4) : z;
      }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = mrow0 + i * 32 + lr;
      if (m < M) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = ncol0 + j * 32 + q * 8 + lh * 4;
            f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            apply4<EPI, TO>(out_op, out_f32, z_out, z_in, g_out, base, X, ybar, RHS, OUT, hstep, sgn,
                            (long)m * N + n, v + bv[j][q]);
          }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// MFMA kernel.  WM x WN wavefronts, each owning a (BM/WM) x (BN/WN) tile of the output.
//  * Operands go from global memory straight into LDS (global_load_lds, 16 bytes per lane,
//    no register staging) through a ring of STAGES k-tiles of depth BK (32 or 64).
//  * An LDS row holds the BK bf16 of one matrix row (64 or 128 bytes) unpadded; its 16-byte
//    chunks are XOR-swizzled by the row number so that the 16-byte fragment reads of 32
//    consecutive rows are bank-conflict free.  A load instruction of a wavefront fills 1 KB
//    = 8 (or 16) consecutive rows; the lane that will land at position p of row r fetches
//    logical chunk p ^ f(r) of that row.
//  * MFMA fragments are double-buffered in registers (LDS reads of k-step s+1 overlap the
//    MFMAs of s) and the next tile's load instructions are issued one at a time between
//    MFMA groups, so their issue time overlaps matrix work.
//  * The weight fragment is the first MFMA operand: a lane then holds 4 consecutive output
//    columns per register quad.
//  * Epilogue, STAGED: each wavefront transposes 32 rows at a time through a private padded
//    LDS region and walks them row-major (32 lanes per row), so every global access of the
//    epilogue covers whole contiguous rows.  Otherwise: straight from the MFMA layout.
// ---------------------------------------------------------------------------
typedef __attribute__((address_space(1))) const void* gas_ptr;
typedef __attribute__((address_space(3))) void* las_ptr;

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else if constexpr (N == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
  else if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if constexpr (N == 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
  else if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  else if constexpr (N == 18) asm volatile("s_waitcnt vmcnt(18)" ::: "memory");
  else if constexpr (N == 24) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
  else if constexpr (N == 32) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// LDS has 64 four-byte banks (256 bytes per clock); a 16-byte read is served 16 lanes at a
// time, so 16 consecutive rows must land on 16 distinct 16-byte slots modulo 256 bytes.  With
// 128-byte rows two rows share a 256-byte bank row: swizzle by the row pair; with 64-byte
// rows four rows share it: swizzle by the row quad.
template <int BK> __device__ __forceinline__ int swz(int row) {
  return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

template <int BM, int BN, int BK, int STAGES, int OCC, bool STAGED, int EPI, typename TO, int WM = 2, int WN = 2>
__global__ void __launch_bounds__(64 * WM * WN, OCC)
gemm_mfma_kernel(const GemmArgs a, int tiles_m, int tiles_n, int total_tiles, int per_xcd, int pm, int pn) {
  constexpr int NW = WM * WN;                            // wavefronts per block
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int RB = BK * 2;                             // bytes per LDS row
  constexpr int CPR = RB / 16;                           // 16-byte chunks per row
  constexpr int RPL = 1024 / RB;                         // rows per load instruction
  constexpr int KS = BK / 16;                            // MFMA k-steps per tile
  constexpr int A_BYTES = BM * RB, B_BYTES = BN * RB, STAGE = A_BYTES + B_BYTES;
  constexpr int A_LD = BM / RPL / NW, B_LD = BN / RPL / NW; // load instructions per wave per k-tile
  static_assert(A_LD >= 1 && B_LD >= 1 && A_LD * RPL * NW == BM && B_LD * RPL * NW == BN, "tile/wave split");
  constexpr int PER_TILE = A_LD + B_LD;
  constexpr int SLOTS = KS * TM;                         // MFMA groups per k-tile
  constexpr int PER_SLOT = (PER_TILE + SLOTS - 1) / SLOTS;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem2[];

  // XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, so give each
  // XCD one contiguous range of tiles.  Inside a group's tile grid the order runs over
  // pm x pn patches (pn = 0: plain row-major): the tiles an XCD runs at the same time then
  // share pm activation row panels and a pn-tile-wide slice of the weight matrix, which fit
  // that XCD's L2 together, and successive patches keep the row panels.
  const int pid = blockIdx.x;
  const int tile = (pid & 7) * per_xcd + (pid >> 3);
  if (tile >= total_tiles) return;
  const int tiles_per_group = tiles_m * tiles_n;
  const int g = tile / tiles_per_group;
  const int tg = tile - g * tiles_per_group;
  int tm, tn;
  if (pn > 0) {
    const int patch = pm * pn, patches_n = tiles_n / pn;
    const int b = tg / patch, w = tg - b * patch;
    const int bm = b / patches_n, bn = b - bm * patches_n;
    tm = bm * pm + w / pn;
    tn = bn * pn + w % pn;
  } else {
    tm = tg / tiles_n;
    tn = tg - tm * tiles_n;
  }
  const int m0 = tm * BM, n0 = tn * BN;

  const bf16* A = reinterpret_cast<const bf16*>(a.A) + a.a_slots.of(g) * a.a_slot_stride;
  const char* pblock = a.B.at(g);
  const bf16* B = reinterpret_cast<const bf16*>(pblock + a.b_off);
  const int K = a.K, M = a.M;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int lr = lane & 31, lh = lane >> 5;
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  // global -> LDS: this lane's element offsets (row clamped at the ragged tail of M)
  const int lrow = lane / CPR, lpos = lane % CPR;
  unsigned aoff[A_LD], boff[B_LD];
#pragma unroll
  for (int j = 0; j < A_LD; ++j) {
    const int row = (wave * A_LD + j) * RPL + lrow;            // row inside the tile
    int gm = m0 + row;
    gm = gm < M ? gm : M - 1;
    aoff[j] = (unsigned)gm * (unsigned)K + (lpos ^ swz<BK>(row)) * 8;
  }
#pragma unroll
  for (int j = 0; j < B_LD; ++j) {
    const int row = (wave * B_LD + j) * RPL + lrow;
    boff[j] = (unsigned)(n0 + row) * (unsigned)K + (lpos ^ swz<BK>(row)) * 8;
  }

  auto issue_one = [&](int stage, int k0, int idx) {
    unsigned char* sa = smem2 + stage * STAGE;
    if (idx < A_LD)
      __builtin_amdgcn_global_load_lds((gas_ptr)(A + aoff[idx] + k0), (las_ptr)(sa + (wave * A_LD + idx) * 1024),
                                       16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((gas_ptr)(B + boff[idx - A_LD] + k0),
                                       (las_ptr)(sa + A_BYTES + (wave * B_LD + idx - A_LD) * 1024), 16, 0, 0);
  };
  auto issue = [&](int stage, int k0) {
#pragma unroll
    for (int idx = 0; idx < PER_TILE; ++idx) issue_one(stage, k0, idx);
  };

  // fragment byte offsets inside a tile region: row lr, swizzled chunk of k-step ks
  int foff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) foff[ks] = lr * RB + (((2 * ks + lh) ^ swz<BK>(lr)) << 4);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = K / BK;
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < KT) issue(s, s * BK);
  if (KT > STAGES - 2) wait_vmcnt<(STAGES - 2) * PER_TILE>(); else wait_vmcnt<0>();
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt % STAGES;
    const bool pf = kt + STAGES - 1 < KT;
    const int pstage = (kt + STAGES - 1) % STAGES, pk0 = (kt + STAGES - 1) * BK;
    const unsigned char* sA = smem2 + cur * STAGE + wm0 * RB;
    const unsigned char* sB = smem2 + cur * STAGE + A_BYTES + wn0 * RB;
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = *reinterpret_cast<const bf16x8*>(sA + i * 32 * RB + foff[0]);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = *reinterpret_cast<const bf16x8*>(sB + j * 32 * RB + foff[0]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cb = ks & 1, nb = cb ^ 1;
      if (ks + 1 < KS) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
          fa[nb][i] = *reinterpret_cast<const bf16x8*>(sA + i * 32 * RB + foff[ks + 1 < KS ? ks + 1 : 0]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fb[nb][j] = *reinterpret_cast<const bf16x8*>(sB + j * 32 * RB + foff[ks + 1 < KS ? ks + 1 : 0]);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cb][j], fa[cb][i], acc[i][j], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < PER_SLOT; ++u) {
          const int idx = (ks * TM + i) * PER_SLOT + u;
          if (idx < PER_TILE && pf) issue_one(pstage, pk0, idx);
        }
      }
    }
    // tile kt+1 must have landed (later tiles may still be in flight), and every wave must be
    // done reading this stage before it is refilled
    if (kt + STAGES - 1 < KT) wait_vmcnt<(STAGES - 2) * PER_TILE>(); else wait_vmcnt<0>();
    __syncthreads();
  }

  // the staging regions reuse the (now idle) k-tile ring; the launcher sizes LDS for both
  constexpr int EP_BYTES = (32 * (WTN * 4 + 16) + 1023) / 1024 * 1024;
  const EpiPtrs P = resolve_epi<TO>(a, g, EPI);
  tile_epilogue<EPI, TO, TM, TN, STAGED>(acc, smem2 + wave * EP_BYTES, P.bias, static_cast<TO*>(P.out),
                                         static_cast<float*>(P.out), static_cast<TO*>(P.aux),
                                         static_cast<const TO*>(P.aux), static_cast<TO*>(P.aux2), P.base, P.X,
                                         static_cast<const float*>(P.aux), P.RHS, P.OUT, a.hstep, a.rhs_sign, a.N,
                                         M, m0 + wm0, n0 + wn0, lane);
}

// ---------------------------------------------------------------------------
// fp32 MFMA kernel (fp32 parameters and operands): 64x64 block tile, 4 wavefronts of 32x32 on
// the 32x32x2 fp32 MFMA, k-tiles of 16 staged through LDS.  As in the bf16 kernel the weight
// fragment is the first MFMA operand, so a lane ends up with 4 consecutive output columns of one
// row per register quad and the shared epilogue code applies.  Needs N % 64 == 0 and K % 16 == 0;
// M may be ragged (rows are clamped on load and guarded on store).
// ---------------------------------------------------------------------------
template <int EPI>
__global__ void __launch_bounds__(256)
gemm_f32_mfma_kernel(const GemmArgs a, int tiles_m, int tiles_n) {
  constexpr int BT = 64, BKF = 16, LD = BKF + 4;       // row pitch 20 floats: 16-byte aligned vector stores
  __shared__ __attribute__((aligned(16))) float As[BT * LD];
  __shared__ __attribute__((aligned(16))) float Bs[BT * LD];
  const int g = blockIdx.z;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x - tm * tiles_n;
  const int m0 = tm * BT, n0 = tn * BT;
  const float* A = reinterpret_cast<const float*>(a.A) + a.a_slots.of(g) * a.a_slot_stride;
  const float* B = reinterpret_cast<const float*>(a.B.at(g) + a.b_off);
  const int M = a.M, K = a.K;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane & 31, lh = lane >> 5;
  const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
  const int srow = tid >> 2, sk = (tid & 3) * 4;       // staging: one float4 of each operand per thread
  int am = m0 + srow;
  am = am < M ? am : M - 1;
  const float* ap = A + (long)am * K + sk;
  const float* bp = B + (long)(n0 + srow) * K + sk;
  f32x16 acc[1][1];
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[0][0][r] = 0.f;
  f32x4 va = *reinterpret_cast<const f32x4*>(ap), vb = *reinterpret_cast<const f32x4*>(bp);
  for (int k0 = 0; k0 < K; k0 += BKF) {
    __syncthreads();                                   // the previous k-tile has been read by every wavefront
    *reinterpret_cast<f32x4*>(&As[srow * LD + sk]) = va;
    *reinterpret_cast<f32x4*>(&Bs[srow * LD + sk]) = vb;
    __syncthreads();
    if (k0 + BKF < K) {                                // next k-tile's loads fly while this one is multiplied
      va = *reinterpret_cast<const f32x4*>(ap + k0 + BKF);
      vb = *reinterpret_cast<const f32x4*>(bp + k0 + BKF);
    }
#pragma unroll
    for (int ks = 0; ks < BKF; ks += 2)
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(Bs[(wn0 + lr) * LD + ks + lh], As[(wm0 + lr) * LD + ks + lh],
                                                      acc[0][0], 0, 0, 0);
  }
  const EpiPtrs P = resolve_epi<float>(a, g, EPI);
  tile_epilogue<EPI, float, 1, 1, false>(acc, nullptr, P.bias, static_cast<float*>(P.out), static_cast<float*>(P.out),
                                         static_cast<float*>(P.aux), static_cast<const float*>(P.aux),
                                         static_cast<float*>(P.aux2), P.base, P.X,
                                         static_cast<const float*>(P.aux), P.RHS, P.OUT, a.hstep, a.rhs_sign, a.N, M,
                                         m0 + wm0, n0 + wn0, lane);
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
    const EpiPtrs P = resolve_epi<TO>(a, g, EPI);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + ty * 4 + i;
      if (m < M) {
        f32x4 v = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
        epilogue4<EPI, TO>(P, a.hstep, a.rhs_sign, N, m, n, v);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------
static int g_force_simple = 0;
static int g_tile_cfg = 0;                 // 0 = choose by shape
void gemm_force_simple(int on) { g_force_simple = on; }
void gemm_set_tile_config(int cfg) { g_tile_cfg = cfg; }

// Compute units of the current device (256 if the query fails).
static int compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
      cus = 256;
    n = cus;
  }
  return n;
}

template <int BM, int BN, int BK, int STAGES, int OCC, bool STAGED, int EPI, int WM = 2, int WN = 2>
static hipError_t launch_mfma(const GemmArgs& a, hipStream_t st) {
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = a.N / BN;
  const int total = tiles_m * tiles_n * a.n_groups;
  const int per_xcd = (total + 7) / 8;
  const size_t ring = (size_t)STAGES * (BM + BN) * BK * 2;
  const size_t staging = STAGED ? (size_t)WM * WN * ((32 * (BN / WN * 4 + 16) + 1023) / 1024 * 1024) : 0;
  const size_t smem = ring > staging ? ring : staging;
  // patch shape of the tile order: 4 tiles wide, half of what one XCD runs at a time (two patches next
  // to each other are resident together; measured against whole-resident-set patches: the bias+GELU
  // launches 5 % faster at the GPT-2 and BERT shapes, the others unchanged)
  int pm = 0, pn = 0;
  const int resident = compute_units() / 8 * OCC;
  if (tiles_n > 4 && tiles_n % 4 == 0 && resident % 8 == 0 && tiles_m % (resident / 8) == 0) {
    pn = 4;
    pm = resident / 8;
  }
  auto kern = gemm_mfma_kernel<BM, BN, BK, STAGES, OCC, STAGED, EPI, bf16, WM, WN>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(per_xcd * 8), dim3(64 * WM * WN), smem, st, a, tiles_m, tiles_n, total,
                     per_xcd, pm, pn);
  return hipGetLastError();
}

template <int EPI>
static hipError_t launch_f32_mfma(const GemmArgs& a, hipStream_t st) {
  const int tiles_m = (a.M + 63) / 64, tiles_n = a.N / 64;
  hipLaunchKernelGGL((gemm_f32_mfma_kernel<EPI>), dim3(tiles_m * tiles_n, 1, a.n_groups), dim3(256), 0, st, a,
                     tiles_m, tiles_n);
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
  if (EPI == EPI_GELU || EPI == EPI_GELU_PRIME) b += G * MN * esz * (a.aux ? 2 : 1);
  if (EPI == EPI_GELU_BOTH) b += G * MN * esz * (a.aux ? 3 : 2);
  if (EPI == EPI_DGELU) b += G * MN * esz * 2;
  if (EPI == EPI_STORE_F32) b += G * MN * 4;
  if (EPI == EPI_RESID_INNER) b += G * MN * 4 * (a.base ? 2 : 1);
  if (EPI == EPI_RESID_OUTER) b += G * MN * 4 * (a.RHS.present() ? 4 : 3);
  return b;
}

// Tile configurations of the MFMA kernel (BK = 64, two stages, unless noted):
//  1: 256x256, 8 wavefronts 2x4 (128x64 each, two per SIMD), one block per CU;
//  3: 256x192, 8 wavefronts 4x2 (64x96 each), one block per CU;
//  4: 128x128, 4 wavefronts (64x64 each), two blocks per CU;
//  2: 256x128x32, three stages, 4 wavefronts (128x64 each), two blocks per CU: any N % 128 == 0.
// A launch runs in rounds of (CUs x blocks per CU) tiles.  Measured on MI355X at 768..3072 wide
// operands, the time of a round hardly depends on how full it is, and relative to a round of
// 256x256 tiles a round of 256x192 tiles takes 0.9 and a (double) round of 128x128 tiles 0.62:
// pick the configuration with the cheapest sum of rounds.
static int choose_tile_config(int n_groups, int M, int N, double* cost_out = nullptr) {
  struct Cand { int cfg, bm, bn, occ; double round_cost; };
  static const Cand cands[] = {{1, 256, 256, 1, 1.0}, {3, 256, 192, 1, 0.9}, {4, 128, 128, 2, 0.62}};
  const long cus = compute_units();
  int best = 2;
  double best_cost = 1e30;
  for (const Cand& c : cands) {
    if (N % c.bn != 0) continue;
    const long tiles = (long)((M + c.bm - 1) / c.bm) * (N / c.bn) * n_groups;
    const long rounds = (tiles + cus * c.occ - 1) / (cus * c.occ);
    const double cost = rounds * c.round_cost;
    if (cost < best_cost) { best_cost = cost; best = c.cfg; }
  }
  if (best == 2) {                                       // 256x128x32, two blocks per CU
    const long tiles = (long)((M + 255) / 256) * ((N + 127) / 128) * n_groups;
    best_cost = (double)((tiles + cus * 2 - 1) / (cus * 2));
  }
  if (cost_out) *cost_out = best_cost;
  return best;
}

// Modelled time of one grouped launch, in rounds of 256x256 tiles per 64 of reduction length (the
// driver sizes its launch chunks with it).
double gemm_model_cost(int n_groups, int M, int N, int K) {
  double c = 0.0;
  choose_tile_config(n_groups, M, N, &c);
  return c * K / 64.0;
}

template <int EPI>
static hipError_t launch_epi(const GemmArgs& a, bool is_bf16, hipStream_t st) {
  if (a.n_groups <= 0 || a.M <= 0) return hipSuccess;
  const double flops = 2.0 * a.n_groups * a.M * (double)a.N * a.K;
  // the MFMA kernel needs whole 64-deep k-tiles and 128-wide column tiles, and 32-bit element offsets
  const bool mfma_ok = is_bf16 && !g_force_simple && (a.K % 64 == 0) && (a.N % 128 == 0) &&
                       (double)a.M * a.K < 4e9 && (double)a.N * a.K < 4e9;
  const int cls = mfma_ok ? (a.n_groups > 1 ? PC_GEMM_MFMA : PC_GEMM_MFMA_SINGLE) + EPI : PC_GEMM_SIMPLE;
  ProfScope ps(cls, flops, gemm_bytes<EPI>(a, is_bf16 ? 2 : 4), st);
  if (!is_bf16) {
    // fp32: the 32x32x2 fp32 MFMA where the shape allows it (whole 64-column tiles, whole 16-deep k-tiles)
    if (!g_force_simple && a.N % 64 == 0 && a.K % 16 == 0) return launch_f32_mfma<EPI>(a, st);
    return launch_simple<float, EPI>(a, st);
  }
  if (!mfma_ok) return launch_simple<bf16, EPI>(a, st);
  int cfg = g_tile_cfg;
  if (cfg == 0) cfg = choose_tile_config(a.n_groups, a.M, a.N);
  switch (cfg) {
    case 1: if (a.N % 256 == 0) return launch_mfma<256, 256, 64, 2, 1, true, EPI, 2, 4>(a, st); break;
    case 2: return launch_mfma<256, 128, 32, 3, 2, true, EPI>(a, st);
    case 3: if (a.N % 192 == 0) return launch_mfma<256, 192, 64, 2, 1, true, EPI, 4, 2>(a, st); break;
    case 4:
      // long reductions: 8 wavefronts of 32x64 (four per SIMD with two blocks resident) hide the
      // k-loop's latencies better than 4 of 64x64; short ones are all epilogue, where 4 do better
      if (a.K >= 512) return launch_mfma<128, 128, 64, 2, 2, true, EPI, 4, 2>(a, st);
      return launch_mfma<128, 128, 64, 2, 2, true, EPI>(a, st);
    default: break;
  }
  return launch_mfma<256, 128, 32, 3, 2, true, EPI>(a, st);
}

hipError_t launch_gemm(const GemmArgs& a, int epi, bool is_bf16, hipStream_t st) {
  switch (epi) {
    case EPI_STORE: return launch_epi<EPI_STORE>(a, is_bf16, st);
    case EPI_GELU: return launch_epi<EPI_GELU>(a, is_bf16, st);
    case EPI_RESID_INNER: return launch_epi<EPI_RESID_INNER>(a, is_bf16, st);
    case EPI_RESID_OUTER: return launch_epi<EPI_RESID_OUTER>(a, is_bf16, st);
    case EPI_DGELU: return launch_epi<EPI_DGELU>(a, is_bf16, st);
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32>(a, is_bf16, st);
    case EPI_GELU_PRIME: return launch_epi<EPI_GELU_PRIME>(a, is_bf16, st);
    case EPI_GELU_BOTH: return a.aux2 ? launch_epi<EPI_GELU_BOTH>(a, is_bf16, st) : hipErrorInvalidValue;
  }
  return hipErrorInvalidValue;
}

}  // namespace mg
