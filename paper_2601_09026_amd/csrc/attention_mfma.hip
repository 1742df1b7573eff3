// Fused softmax attention on the 32x32x16 bf16 MFMA (d_head = 64 or 128), forward and backward.
//
// Every product is arranged as  D[i][j] = sum_k A[i][k] B[k][j]  with the wavefront's own 32
// rows (queries in the forward and dQ kernels, keys in the dK/dV kernel) on the j axis.  In
// the MFMA result layout lane l then owns column j = l%32 and its 16 registers hold rows
// i = 8q + 4*(l/32) + r  (q, r = 0..3).  Consequences:
//   * the softmax statistics of a query are private to a lane (plus one exchange between
//     lanes l and l+32): no cross-lane reductions over the score tile;
//   * a score / probability tile, converted to bf16, already IS the B operand of the next
//     product (registers 8t..8t+7 feed k-step t), provided the A operand enumerates the
//     reduction index the same way: k-slot (half, e) <-> row 16t + 8*(e/4) + 4*half + e%4.
//     A operands of that kind are read from a transposed LDS tile as two 8-byte pieces;
//   * per-row scalars (running max, denominator, lse, D) scale whole accumulators in place.
// A operands come from LDS (row-major tile, or the transposed copy made while staging), B
// operands stay in registers for the whole kernel.
//
// Forward :  S^T = K Q^T,  P^T = exp2(c S^T - m),  O^T += V^T P^T           (online softmax)
// dQ pass :  S^T, dP^T = V dO^T,  dA^T = P^T (dP^T - D),  dQ^T += K^T dA^T
// dKV pass:  S = Q K^T, dP = dO V^T, P, dA;  dV^T += dO^T P,  dK^T += Q^T dA
// No atomics: dQ and dK/dV are separate passes, so results are bit-reproducible.
#include "common.h"
#include "kernels.h"

namespace mg {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

// LDS has 64 four-byte banks.  Row-major tiles are read 16 bytes per lane (16 lanes per
// clock): rows of DH + 8 bf16 (144 or 272 bytes, an odd number of 16-byte units) put 16
// consecutive rows on 16 distinct 16-byte slots.  Transposed tiles are read 8 bytes per lane
// (32 lanes per clock): 136-byte rows (an odd number of 8-byte units) put 32 consecutive rows
// on 32 distinct 8-byte slots.
template <int DH> constexpr int fa_ld() { return DH + 8; }     // row-major tile [64][DH + 8 pad]
constexpr int FA_LDT = 68;                // transposed tile [DH][64 + 4 pad]
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// 64 rows x DH cols of bf16 from global (rows clamped to nrows-1) into a row-major LDS tile
// and/or its transpose.  Work item = (row pair, 8-column chunk); the chunk varies fastest so
// that DH/8 consecutive lanes fetch one whole row (coalesced global reads matter more
// here than the two-way bank conflict the transposed 4-byte stores then have).
template <int NT, int DH, bool PLAIN, bool TRANS>
__device__ __forceinline__ void stage64(bf16* plain, bf16* trans, const bf16* src, long rs, int row0, int nrows) {
  constexpr int FA_LD = fa_ld<DH>(), CH = DH / 8;
#pragma unroll
  for (int item = threadIdx.x; item < 32 * CH; item += NT) {
    const int cc = item % CH, rp = item / CH;
    int r0 = row0 + 2 * rp, r1 = r0 + 1;
    r0 = r0 < nrows ? r0 : nrows - 1;
    r1 = r1 < nrows ? r1 : nrows - 1;
    const bf16x8 v0 = *reinterpret_cast<const bf16x8*>(src + (long)r0 * rs + 8 * cc);
    const bf16x8 v1 = *reinterpret_cast<const bf16x8*>(src + (long)r1 * rs + 8 * cc);
    if (PLAIN) {
      *reinterpret_cast<bf16x8*>(plain + (2 * rp) * FA_LD + 8 * cc) = v0;
      *reinterpret_cast<bf16x8*>(plain + (2 * rp + 1) * FA_LD + 8 * cc) = v1;
    }
    if (TRANS) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        bf16x2 pr = {v0[i], v1[i]};
        *reinterpret_cast<bf16x2*>(trans + (8 * cc + i) * FA_LDT + 2 * rp) = pr;
      }
    }
  }
}

// The same staging in two halves, for double-buffered tiles: tile_load leaves the 64 x DH values
// in registers (global loads in flight while the current tile is being used), tile_store writes
// them to the row-major tile and/or its transpose.
template <int NT, int DH>
struct TileRegs {
  static constexpr int N = (32 * (DH / 8) + NT - 1) / NT;
  bf16x8 v0[N], v1[N];
};
template <int NT, int DH>
__device__ __forceinline__ void tile_load(TileRegs<NT, DH>& r, const bf16* src, long rs, int row0, int nrows) {
  constexpr int CH = DH / 8;
#pragma unroll
  for (int j = 0; j < TileRegs<NT, DH>::N; ++j) {
    const int item = threadIdx.x + j * NT;
    if (32 * CH % NT == 0 || item < 32 * CH) {   // (no test where the items divide evenly)
      const int cc = item % CH, rp = item / CH;
      int r0 = row0 + 2 * rp, r1 = r0 + 1;
      r0 = r0 < nrows ? r0 : nrows - 1;
      r1 = r1 < nrows ? r1 : nrows - 1;
      r.v0[j] = *reinterpret_cast<const bf16x8*>(src + (long)r0 * rs + 8 * cc);
      r.v1[j] = *reinterpret_cast<const bf16x8*>(src + (long)r1 * rs + 8 * cc);
    }
  }
}
template <int NT, int DH, bool PLAIN, bool TRANS>
__device__ __forceinline__ void tile_store(const TileRegs<NT, DH>& r, bf16* plain, bf16* trans) {
  constexpr int FA_LD = fa_ld<DH>(), CH = DH / 8;
#pragma unroll
  for (int j = 0; j < TileRegs<NT, DH>::N; ++j) {
    const int item = threadIdx.x + j * NT;
    if (32 * CH % NT == 0 || item < 32 * CH) {   // (no test where the items divide evenly)
      const int cc = item % CH, rp = item / CH;
      if (PLAIN) {
        *reinterpret_cast<bf16x8*>(plain + (2 * rp) * FA_LD + 8 * cc) = r.v0[j];
        *reinterpret_cast<bf16x8*>(plain + (2 * rp + 1) * FA_LD + 8 * cc) = r.v1[j];
      }
      if (TRANS) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          bf16x2 pr = {r.v0[j][i], r.v1[j][i]};
          *reinterpret_cast<bf16x2*>(trans + (8 * cc + i) * FA_LDT + 2 * rp) = pr;
        }
      }
    }
  }
}

// A operand from a row-major tile: row `row`, reduction chunk of k-step ks
template <int DH>
__device__ __forceinline__ bf16x8 frag_plain(const bf16* tile, int row, int ks, int lh) {
  return *reinterpret_cast<const bf16x8*>(tile + row * fa_ld<DH>() + 16 * ks + 8 * lh);
}
// A operand from a transposed tile: row `row` (a feature), reduction over the tile's 64
// staged rows, k-step t of 32-row tile rt, in the register-order enumeration
__device__ __forceinline__ bf16x8 frag_trans(const bf16* tile, int row, int rt, int t, int lh) {
  const bf16* p = tile + row * FA_LDT + 32 * rt + 16 * t + 4 * lh;
  const bf16x4 lo = *reinterpret_cast<const bf16x4*>(p);
  const bf16x4 hi = *reinterpret_cast<const bf16x4*>(p + 8);
  bf16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return r;
}
// registers 8t..8t+7 of a result tile as the bf16 B operand of k-step t
__device__ __forceinline__ bf16x8 regs_to_b(const f32x16& v, int t) {
  bf16x8 r = {(bf16)v[8 * t], (bf16)v[8 * t + 1], (bf16)v[8 * t + 2], (bf16)v[8 * t + 3],
              (bf16)v[8 * t + 4], (bf16)v[8 * t + 5], (bf16)v[8 * t + 6], (bf16)v[8 * t + 7]};
  return r;
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}
// 2^x as the bare hardware instruction: the library routine wraps it in a range reduction for
// results below 2^-126, which a probability that small does not need (it is 0 in bf16 anyway)
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

struct HeadPtrs {
  const bf16 *Q, *K, *V, *O, *dO;
  bf16 *Ow, *dQ, *dK, *dV;
  float *lse, *D;
};

__device__ __forceinline__ HeadPtrs head_ptrs(const AttnArgs& a, int g, int b, int h) {
  HeadPtrs p;
  const int dh = a.dh;
  p.Q = reinterpret_cast<const bf16*>(a.q) + a.q_slots.of(g) * a.q_slot_stride + (long)b * a.Sq * a.q_row_stride + h * dh;
  p.K = reinterpret_cast<const bf16*>(a.k) + a.k_slots.of(g) * a.k_slot_stride + (long)b * a.Sk * a.k_row_stride + h * dh;
  p.V = reinterpret_cast<const bf16*>(a.v) + a.k_slots.of(g) * a.v_slot_stride + (long)b * a.Sk * a.v_row_stride + h * dh;
  p.O = reinterpret_cast<const bf16*>(a.o) + a.o_slots.of(g) * a.o_slot_stride + (long)b * a.Sq * a.o_row_stride + h * dh;
  p.Ow = const_cast<bf16*>(p.O);
  p.lse = a.lse ? a.lse + a.lse_slots.of(g) * a.lse_slot_stride + ((long)b * a.H + h) * a.Sq : nullptr;
  p.dO = nullptr; p.dQ = p.dK = p.dV = nullptr; p.D = nullptr;
  if (a.dO) {
    p.dO = reinterpret_cast<const bf16*>(a.dO) + a.do_slots.of(g) * a.do_slot_stride + (long)b * a.Sq * a.do_row_stride + h * dh;
    const long base = a.dqkv_slots.of(g) * a.dqkv_slot_stride;
    p.dQ = reinterpret_cast<bf16*>(a.dq) + base + (long)b * a.Sq * a.dqkv_row_stride + h * dh;
    if (a.dk) {
      const long kv_rs = a.dkv_row_stride ? a.dkv_row_stride : a.dqkv_row_stride;
      const long kv_base = a.dqkv_slots.of(g) * (a.dkv_slot_stride ? a.dkv_slot_stride : a.dqkv_slot_stride);
      p.dK = reinterpret_cast<bf16*>(a.dk) + kv_base + (long)b * a.Sk * kv_rs + h * dh;
      p.dV = reinterpret_cast<bf16*>(a.dv) + kv_base + (long)b * a.Sk * kv_rs + h * dh;
    }
    p.D = a.D + a.D_slots.of(g) * a.D_slot_stride + ((long)b * a.H + h) * a.Sq;
  }
  return p;
}

// store [DH features][32 rows] accumulators (transposed result) as rows of DH bf16
template <int DH>
__device__ __forceinline__ void store_rows_T(bf16* dst, long row_stride, int row, const f32x16* acc, float mul,
                                             int lh) {
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 v = {acc[dt][4 * q] * mul, acc[dt][4 * q + 1] * mul, acc[dt][4 * q + 2] * mul, acc[dt][4 * q + 3] * mul};
      store4<bf16>(dst + (long)row * row_stride + 32 * dt + 8 * q + 4 * lh, v);
    }
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
// Which (row block, batch*head, group) a workgroup takes.  Workgroups are dispatched in linear order
// of their index (x fastest), consecutive ones to consecutive XCDs (8, each with an L2 of its own).
// Causal mask: the work of a row block grows (query blocks) or shrinks (key blocks) with its
// position, 4 : 1 between the two ends of a 512-token sequence, so in the natural order some XCDs get
// only heavy blocks.  The linear index is re-read as (rank of the row block, head), heaviest rank
// first: every XCD gets the same mix and the launch ends on its lightest blocks.
// No mask: all blocks are equal; the index is re-read so that the row blocks of one head go to ONE
// XCD one after the other (they run together and share the head's K and V, or Q and dO, in its L2).
struct BlockTask { int tile, bh, g; };
__device__ __forceinline__ BlockTask block_task(bool causal, bool last_tile_heaviest) {
  const int nx = gridDim.x, ny = gridDim.y;
  if (nx == 1) return {0, (int)blockIdx.y, (int)blockIdx.z};
  const int heads = ny * gridDim.z;
  const int lin = blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z);
  int tile, head;
  if (causal) {
    const int rank = lin / heads;
    head = lin - rank * heads;
    tile = last_tile_heaviest ? nx - 1 - rank : rank;
  } else {
    const int whole = (heads >> 3) << 3;                  // heads that fill all 8 XCDs evenly
    if (lin < whole * nx) {
      const int s = lin >> 3, hs = s / nx;
      tile = s - hs * nx;
      head = (hs << 3) + (lin & 7);
    } else {
      const int rem = lin - whole * nx, hs = rem / nx;
      tile = rem - hs * nx;
      head = whole + hs;
    }
  }
  const int g = head / ny;
  return {tile, head - g * ny, g};
}

// Resident blocks per CU the register budget is set for: the accumulators grow with DH.
template <int DH, int NW = 4> constexpr int fa_fwd_blocks() { return NW == 8 ? 1 : DH == 64 ? 4 : 2; }
template <int DH, int NW = 4> constexpr int fa_bwd_blocks() { return NW == 8 ? 1 : 2; }

template <int NW, int DH>
__global__ void __launch_bounds__(NW * 64, (fa_fwd_blocks<DH, NW>())) attn_fwd_mfma_kernel(const AttnArgs a) {
  constexpr int KS = DH / 16, DT = DH / 32;
  // d_head = 128, blocks of 128 queries or more: two buffers per tile, the next key tile is
  // fetched while this one is used and written after it, one barrier per tile (forward time -14 %
  // at 2048 keys; at d_head = 64 the gain is within noise and costs a resident block)
  constexpr bool DB = NW >= 4 && DH == 128;
  __shared__ __attribute__((aligned(16))) bf16 Ksb[DB ? 2 : 1][64 * fa_ld<DH>()];    // [key][d]
  __shared__ __attribute__((aligned(16))) bf16 Vtb[DB ? 2 : 1][DH * FA_LDT];          // [d][key]
  const BlockTask bt = block_task(a.causal, true);
  const int g = bt.g;
  const int b = bt.bh / a.H, h = bt.bh - b * a.H;
  const int q0 = bt.tile * (NW * 32);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 31, lh = lane >> 5;
  const HeadPtrs P = head_ptrs(a, g, b, h);
  const int qi = q0 + wave * 32 + lr;
  const int qc = qi < a.Sq ? qi : a.Sq - 1;
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(P.Q + (long)qc * a.q_row_stride + 16 * ks + 8 * lh);

  const float c = rsqrtf((float)DH) * LOG2E;
  float m = -INFINITY, l = 0.f;
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = zero16();
  const int q_blk_last = min(q0 + NW * 32, a.Sq) - 1;
  const int k_end = a.causal ? min(a.Sk, q_blk_last + 1) : a.Sk;
  const int q_wave_first = q0 + wave * 32, q_wave_last = q_wave_first + 31;
  TileRegs<NW * 64, DH> kr, vr;
  if constexpr (DB) {                                    // k_end >= 1: the launcher rejects empty sequences
    tile_load(kr, P.K, a.k_row_stride, 0, a.Sk);
    tile_load(vr, P.V, a.v_row_stride, 0, a.Sk);
    tile_store<NW * 64, DH, true, false>(kr, Ksb[0], nullptr);
    tile_store<NW * 64, DH, false, true>(vr, nullptr, Vtb[0]);
    __syncthreads();
    // every load issued so far has landed (the tile was waited for and loads return in order);
    // saying so keeps the loop's waits on the query fragments from also covering its prefetches
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
  }
  int cur = 0;
  for (int k0 = 0; k0 < k_end; k0 += 64, cur ^= DB ? 1 : 0) {
    const bool more = DB && k0 + 64 < k_end;               // block-uniform
    if constexpr (!DB) {
      __syncthreads();
      stage64<NW * 64, DH, true, false>(Ksb[0], nullptr, P.K, a.k_row_stride, k0, a.Sk);
      stage64<NW * 64, DH, false, true>(nullptr, Vtb[0], P.V, a.v_row_stride, k0, a.Sk);
      __syncthreads();
    } else if (more) {
      tile_load(kr, P.K, a.k_row_stride, k0 + 64, a.Sk);
      tile_load(vr, P.V, a.v_row_stride, k0 + 64, a.Sk);
    }
    const bf16* Ks = Ksb[cur];
    const bf16* Vt = Vtb[cur];
    if (!(a.causal && k0 > q_wave_last)) {               // wave-uniform: the tile lies above the diagonal
    f32x16 s[2] = {zero16(), zero16()};
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) s[kt] = MFMA(frag_plain<DH>(Ks, 32 * kt + lr, ks, lh), qf[ks], s[kt]);
    // a tile whose 64 keys all exist and precede every query of the wavefront needs no mask
    // (wave-uniform test); masked scores become -inf, whose exp2 is 0
    const bool full = k0 + 64 <= a.Sk && (!a.causal || k0 + 63 <= q_wave_first);
    if (!full) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + 32 * kt + 8 * (i >> 2) + 4 * lh + (i & 3);
          const bool valid = key < a.Sk && (!a.causal || key <= qi);
          s[kt][i] = valid ? s[kt][i] : -INFINITY;
        }
    }
    float mloc = -INFINITY;                                // of the raw scores; the scale c is positive
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mloc = fmaxf(mloc, s[kt][i]);
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float mn = fmaxf(m, mloc * c);
    const float ms = mn == -INFINITY ? 0.f : mn;         // fully masked so far: keep exp2 finite
    const float corr = exp2_raw(m - ms);
    float lsum = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = exp2_raw(fmaf(s[kt][i], c, -ms));
        s[kt][i] = p;
        lsum += p;
      }
    lsum += __shfl_xor(lsum, 32, 64);
    l = l * corr + lsum;
    m = mn;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= corr;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pb = regs_to_b(s[kt], t);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = MFMA(frag_trans(Vt, 32 * dt + lr, kt, t, lh), pb, o[dt]);
      }
    }
    if constexpr (DB) {
      if (more) {
        tile_store<NW * 64, DH, true, false>(kr, Ksb[cur ^ 1], nullptr);
        tile_store<NW * 64, DH, false, true>(vr, nullptr, Vtb[cur ^ 1]);
      }
      __syncthreads();    // the other buffer is complete, and nobody reads this one any more
    }
  }
  if (qi < a.Sq) {
    store_rows_T<DH>(P.Ow, a.o_row_stride, qi, o, 1.0f / l, lh);
    if (P.lse && lh == 0) P.lse[qi] = (m + log2f(l)) * LN2;
  }
}

// ---------------------------------------------------------------------------
// backward pass 1: D and dQ, one wavefront per 32 query rows
// ---------------------------------------------------------------------------
// LDS of the two backward passes (bf16 elements): pass 1 stages K, V row-major and K transposed;
// pass 2 stages Q, dO both ways.  The fused kernel runs them one after the other in the same buffer.
template <int DH> constexpr int bwd_dq_lds() { return 2 * 64 * fa_ld<DH>() + DH * FA_LDT; }
template <int DH> constexpr int bwd_dkv_lds() { return 2 * 64 * fa_ld<DH>() + 2 * DH * FA_LDT; }

// d_local: if not null, D of the block's query rows is also left there (index = row - q0)
// DB: `lds` holds two sets of tiles; the next key tile is fetched while the current one is used
// and written after it, one barrier per tile
template <int NW, int DH, bool DB = false>
__device__ __forceinline__ void attn_bwd_dq_body(const AttnArgs& a, bf16* lds, float* d_local) {
  constexpr int KS = DH / 16, DT = DH / 32, FA_LD = fa_ld<DH>();
  // one set of tiles: K [key][d], V [key][d], K transposed [d][key]
  constexpr int V_OFF = 64 * FA_LD, KT_OFF = 2 * 64 * FA_LD, SET = bwd_dq_lds<DH>();
  const BlockTask bt = block_task(a.causal, true);
  const int g = bt.g;
  const int b = bt.bh / a.H, h = bt.bh - b * a.H;
  const int q0 = bt.tile * (NW * 32);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 31, lh = lane >> 5;
  const HeadPtrs P = head_ptrs(a, g, b, h);
  const int qi = q0 + wave * 32 + lr;
  const int qc = qi < a.Sq ? qi : a.Sq - 1;
  bf16x8 qf[KS], dof[KS];
  float Dq = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8*>(P.Q + (long)qc * a.q_row_stride + 16 * ks + 8 * lh);
    dof[ks] = *reinterpret_cast<const bf16x8*>(P.dO + (long)qc * a.do_row_stride + 16 * ks + 8 * lh);
    const bf16x8 of = *reinterpret_cast<const bf16x8*>(P.O + (long)qc * a.o_row_stride + 16 * ks + 8 * lh);
#pragma unroll
    for (int e = 0; e < 8; ++e) Dq = fmaf((float)dof[ks][e], (float)of[e], Dq);
  }
  Dq += __shfl_xor(Dq, 32, 64);
  const float lse2 = P.lse[qc] * LOG2E;
  if (qi < a.Sq && lh == 0) P.D[qi] = Dq;
  if (d_local && lh == 0) d_local[wave * 32 + lr] = Dq;

  const float c = rsqrtf((float)DH) * LOG2E;
  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) dq[dt] = zero16();
  const int q_blk_last = min(q0 + NW * 32, a.Sq) - 1;
  const int k_end = a.causal ? min(a.Sk, q_blk_last + 1) : a.Sk;
  const int q_wave_first = q0 + wave * 32, q_wave_last = q_wave_first + 31;
  TileRegs<NW * 64, DH> kr, vr;
  if constexpr (DB) {                                    // k_end >= 1: the launcher rejects empty sequences
    tile_load(kr, P.K, a.k_row_stride, 0, a.Sk);
    tile_load(vr, P.V, a.v_row_stride, 0, a.Sk);
    tile_store<NW * 64, DH, true, true>(kr, lds, lds + KT_OFF);
    tile_store<NW * 64, DH, true, false>(vr, lds + V_OFF, nullptr);
    __syncthreads();
    // every load issued so far has landed (the tile was waited for and loads return in order);
    // saying so keeps the loop's waits on the query fragments from also covering its prefetches
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)
  }
  int cur = 0;
  for (int k0 = 0; k0 < k_end; k0 += 64, cur ^= DB ? 1 : 0) {
    bf16* Ks = lds + cur * SET;
    bf16* Vs = Ks + V_OFF;
    bf16* Kt = Ks + KT_OFF;
    const bool more = DB && k0 + 64 < k_end;               // block-uniform
    if constexpr (!DB) {
      __syncthreads();
      stage64<NW * 64, DH, true, true>(Ks, Kt, P.K, a.k_row_stride, k0, a.Sk);
      stage64<NW * 64, DH, true, false>(Vs, nullptr, P.V, a.v_row_stride, k0, a.Sk);
      __syncthreads();
    } else if (more) {
      tile_load(kr, P.K, a.k_row_stride, k0 + 64, a.Sk);
      tile_load(vr, P.V, a.v_row_stride, k0 + 64, a.Sk);
    }
    const bool full = k0 + 64 <= a.Sk && (!a.causal || k0 + 63 <= q_wave_first);   // no mask needed
    if (!(a.causal && k0 > q_wave_last)) {                 // wave-uniform: the tile lies above the diagonal
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      f32x16 s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s = MFMA(frag_plain<DH>(Ks, 32 * kt + lr, ks, lh), qf[ks], s);
        dp = MFMA(frag_plain<DH>(Vs, 32 * kt + lr, ks, lh), dof[ks], dp);
      }
      if (full) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = exp2_raw(fmaf(s[i], c, -lse2)) * (dp[i] - Dq);      // dA^T
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + 32 * kt + 8 * (i >> 2) + 4 * lh + (i & 3);
          const bool valid = key < a.Sk && (!a.causal || key <= qi);
          const float p = valid ? exp2_raw(fmaf(s[i], c, -lse2)) : 0.f;
          s[i] = p * (dp[i] - Dq);
        }
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 ab = regs_to_b(s, t);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) dq[dt] = MFMA(frag_trans(Kt, 32 * dt + lr, kt, t, lh), ab, dq[dt]);
      }
    }
    }
    if constexpr (DB) {
      if (more) {
        bf16* other = lds + (cur ^ 1) * SET;
        tile_store<NW * 64, DH, true, true>(kr, other, other + KT_OFF);
        tile_store<NW * 64, DH, true, false>(vr, other + V_OFF, nullptr);
      }
      __syncthreads();    // the other set is complete, and nobody reads this one any more
    }
  }
  if (qi < a.Sq) store_rows_T<DH>(P.dQ, a.dqkv_row_stride, qi, dq, rsqrtf((float)DH), lh);
}

template <int NW, int DH>
__global__ void __launch_bounds__(NW * 64, (fa_bwd_blocks<DH, NW>())) attn_bwd_dq_mfma_kernel(const AttnArgs a) {
  // the 256-row blocks at d_head = 128 (one block per CU) double-buffer their key tiles
  constexpr bool DB = NW == 8 && DH == 128;
  __shared__ __attribute__((aligned(16))) bf16 lds[(DB ? 2 : 1) * bwd_dq_lds<DH>()];
  attn_bwd_dq_body<NW, DH, DB>(a, lds, nullptr);
}

// ---------------------------------------------------------------------------
// backward pass 2: dK and dV, one wavefront per 32 key rows
// ---------------------------------------------------------------------------
// d_src: D of query row i at d_src[i] (the global array of pass 1, or the fused kernel's LDS copy)
// VLDS: the wavefronts keep their V fragments there (64 lanes x 16 bytes per k-step and
// wavefront in `vpriv`, each lane reading back what it wrote) instead of in registers: at d_head = 128 the two
// accumulator sets and both fragment sets do not fit the 256 registers of two waves per SIMD, and a
// register spilled to scratch costs far more than an LDS read
template <int NW, int DH, bool VLDS = false>
__device__ __forceinline__ void attn_bwd_dkv_body(const AttnArgs& a, bf16* lds, float* Ls, float* Ds,
                                                  const float* d_src, bf16* vpriv = nullptr) {
  constexpr int KS = DH / 16, DT = DH / 32, FA_LD = fa_ld<DH>();
  bf16* Qs = lds;                        // [query][d]
  bf16* dOs = Qs + 64 * FA_LD;           // [query][d]
  bf16* Qt = dOs + 64 * FA_LD;           // [d][query]
  bf16* dOt = Qt + DH * FA_LDT;          // [d][query]
  const BlockTask bt = block_task(a.causal, false);
  const int g = bt.g;
  const int b = bt.bh / a.H, h = bt.bh - b * a.H;
  const int j0 = bt.tile * (NW * 32);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 31, lh = lane >> 5;
  const HeadPtrs P = head_ptrs(a, g, b, h);
  const int kj = j0 + wave * 32 + lr;
  const int kc = kj < a.Sk ? kj : a.Sk - 1;
  bf16x8 kf[KS], vf[VLDS ? 1 : KS];
  bf16* vmine = VLDS ? vpriv + (wave * KS * 64 + lane) * 8 : nullptr;          // + ks * 512 per k-step
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *reinterpret_cast<const bf16x8*>(P.K + (long)kc * a.k_row_stride + 16 * ks + 8 * lh);
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(P.V + (long)kc * a.v_row_stride + 16 * ks + 8 * lh);
    if constexpr (VLDS) *reinterpret_cast<bf16x8*>(vmine + ks * 512) = v;
    else vf[ks] = v;
  }
  const float c = rsqrtf((float)DH) * LOG2E;
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) { dk[dt] = zero16(); dv[dt] = zero16(); }
  // causal: key j only receives from queries i >= j
  const int i_begin = a.causal ? (j0 / 64) * 64 : 0;
  const int k_wave_first = j0 + wave * 32;
  for (int i0 = i_begin; i0 < a.Sq; i0 += 64) {
    __syncthreads();
    stage64<NW * 64, DH, true, true>(Qs, Qt, P.Q, a.q_row_stride, i0, a.Sq);
    stage64<NW * 64, DH, true, true>(dOs, dOt, P.dO, a.do_row_stride, i0, a.Sq);
    if (threadIdx.x < 64) {
      const int qq = i0 + threadIdx.x;
      const int qcl = qq < a.Sq ? qq : a.Sq - 1;
      Ls[threadIdx.x] = P.lse[qcl] * LOG2E;
      Ds[threadIdx.x] = d_src ? d_src[qcl] : P.D[qcl];
    }
    __syncthreads();
    if (a.causal && i0 + 63 < k_wave_first) continue;      // every query of the tile precedes this wave's keys
    // no mask needed: all 64 queries exist, the wavefront's keys exist and (causal) precede them all
    const bool full = i0 + 64 <= a.Sq && k_wave_first + 32 <= a.Sk && (!a.causal || k_wave_first + 31 <= i0);
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      f32x16 s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s = MFMA(frag_plain<DH>(Qs, 32 * qt + lr, ks, lh), kf[ks], s);
        bf16x8 vk;
        if constexpr (VLDS) vk = *reinterpret_cast<const bf16x8*>(vmine + ks * 512);
        else vk = vf[ks];
        dp = MFMA(frag_plain<DH>(dOs, 32 * qt + lr, ks, lh), vk, dp);
      }
      if (full) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int ql = 32 * qt + 8 * (i >> 2) + 4 * lh + (i & 3);
          const float p = exp2_raw(fmaf(s[i], c, -Ls[ql]));
          s[i] = p;
          dp[i] = p * (dp[i] - Ds[ql]);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int ql = 32 * qt + 8 * (i >> 2) + 4 * lh + (i & 3);
          const int qq = i0 + ql;
          const bool valid = qq < a.Sq && kj < a.Sk && (!a.causal || kj <= qq);
          // computed for every pair and zeroed afterwards: a conditional evaluation would put the
          // LDS read of the row's lse behind a branch per element
          const float e = exp2_raw(fmaf(s[i], c, -Ls[ql]));
          const float p = valid ? e : 0.f;
          s[i] = p;
          dp[i] = p * (dp[i] - Ds[ql]);
        }
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pb = regs_to_b(s, t), ab = regs_to_b(dp, t);
        if constexpr (DH == 128) {
          // d_head = 128 runs at the register limit: the fragments of one feature tile are fetched
          // while the products of the tile before it run, and a fence per tile keeps the scheduler
          // from fetching all of them ahead (it then spills the key fragments to scratch)
          bf16x8 fo = frag_trans(dOt, lr, qt, t, lh), fq = frag_trans(Qt, lr, qt, t, lh);
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            bf16x8 fo_n = fo, fq_n = fq;
            if (dt + 1 < DT) {
              fo_n = frag_trans(dOt, 32 * (dt + 1) + lr, qt, t, lh);
              fq_n = frag_trans(Qt, 32 * (dt + 1) + lr, qt, t, lh);
            }
            dv[dt] = MFMA(fo, pb, dv[dt]);
            dk[dt] = MFMA(fq, ab, dk[dt]);
            __builtin_amdgcn_sched_barrier(0);
            fo = fo_n; fq = fq_n;
          }
        } else {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            dv[dt] = MFMA(frag_trans(dOt, 32 * dt + lr, qt, t, lh), pb, dv[dt]);
            dk[dt] = MFMA(frag_trans(Qt, 32 * dt + lr, qt, t, lh), ab, dk[dt]);
          }
        }
      }
    }
  }
  if (kj < a.Sk) {
    const long kv_rs = a.dkv_row_stride ? a.dkv_row_stride : a.dqkv_row_stride;
    store_rows_T<DH>(P.dK, kv_rs, kj, dk, rsqrtf((float)DH), lh);
    store_rows_T<DH>(P.dV, kv_rs, kj, dv, 1.0f, lh);
  }
}

template <int NW, int DH>
__global__ void __launch_bounds__(NW * 64, (fa_bwd_blocks<DH, NW>())) attn_bwd_dkv_mfma_kernel(const AttnArgs a) {
  // the 256-row blocks at d_head = 128 (one block per CU) park their V fragments in LDS
  constexpr bool VLDS = NW == 8 && DH == 128;
  __shared__ __attribute__((aligned(16))) bf16 lds[bwd_dkv_lds<DH>() + (VLDS ? NW * (DH / 16) * 64 * 8 : 0)];
  __shared__ float Ls[64], Ds[64];
  attn_bwd_dkv_body<NW, DH, VLDS>(a, lds, Ls, Ds, nullptr, lds + bwd_dkv_lds<DH>());
}

// Sequences that fit one block (Sq, Sk <= 32 NW): both passes in one launch.  The head's Q, K, V,
// dO are then read from HBM once (pass 2 finds them in L2) and D never leaves the CU.
template <int NW, int DH>
__global__ void __launch_bounds__(NW * 64, (fa_bwd_blocks<DH, NW>())) attn_bwd_fused_mfma_kernel(const AttnArgs a) {
  constexpr int LDS = bwd_dq_lds<DH>() > bwd_dkv_lds<DH>() ? bwd_dq_lds<DH>() : bwd_dkv_lds<DH>();
  __shared__ __attribute__((aligned(16))) bf16 lds[LDS];
  __shared__ float Ls[64], Ds[64], Dall[NW * 32];
  attn_bwd_dq_body<NW, DH>(a, lds, Dall);
  __syncthreads();
  attn_bwd_dkv_body<NW, DH>(a, lds, Ls, Ds, Dall);
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
bool attn_mfma_supported(const AttnArgs& a) {
  return (a.dh == 64 || a.dh == 128) && (a.q_row_stride % 8 == 0) && (a.k_row_stride % 8 == 0) &&
         (a.v_row_stride % 8 == 0) && (a.o_row_stride % 8 == 0);
}

// Blocks of 256 rows halve the K/V (Q/dO) bytes staged from L2 per flop, which is what bounds these
// kernels once a head no longer fits a block of 128.  Mask bits 0-2: forward, dQ pass, dK/dV pass at
// d_head = 128, where these blocks also double-buffer their tiles (forward, dQ) or keep their V
// fragments in LDS (dK/dV): they win from 129 tokens on; the two backward passes keep 128-row
// blocks when the last 256-row block would be at most half full.  Bits 4-6: the same at d_head = 64
// (from 512 tokens; measured slower, off).  Default: all three passes at d_head = 128.
int g_attn_wide = 7;
void attn_set_wide_blocks(int mask) { g_attn_wide = mask & 0x77; }
template <int DH> static bool attn_wide(int pass, int seq) {
  if (DH == 64) return seq >= 512 && ((g_attn_wide >> (4 + pass)) & 1);
  if (!((g_attn_wide >> pass) & 1) || seq <= 128) return false;
  const int tail = seq % 256;
  return pass == 0 || tail == 0 || tail > 128;
}

template <int DH>
static hipError_t attn_fwd_mfma_dh(const AttnArgs& a, hipStream_t st) {
  if (a.Sq <= 0 || a.Sk <= 0) return hipErrorInvalidValue;
  if (a.Sq <= 64) {
    dim3 grid((a.Sq + 63) / 64, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<2, DH>), grid, dim3(128), 0, st, a);
  } else if (attn_wide<DH>(0, a.Sq)) {
    dim3 grid((a.Sq + 255) / 256, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<8, DH>), grid, dim3(512), 0, st, a);
  } else {
    dim3 grid((a.Sq + 127) / 128, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<4, DH>), grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t attn_fwd_mfma(const AttnArgs& a, hipStream_t st) {
  return a.dh == 64 ? attn_fwd_mfma_dh<64>(a, st) : attn_fwd_mfma_dh<128>(a, st);
}

template <int DH>
static hipError_t attn_bwd_mfma_dh(const AttnArgs& a, hipStream_t st) {
  if (a.Sq <= 0 || a.Sk <= 0) return hipErrorInvalidValue;
  if (a.dk && a.Sq <= 128 && a.Sk <= 128) {
    dim3 grid(1, a.B * a.H, a.n_groups);
    if (a.Sq <= 64 && a.Sk <= 64) hipLaunchKernelGGL((attn_bwd_fused_mfma_kernel<2, DH>), grid, dim3(128), 0, st, a);
    else hipLaunchKernelGGL((attn_bwd_fused_mfma_kernel<4, DH>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
  }
  if (a.Sq <= 64) {
    dim3 grid((a.Sq + 63) / 64, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<2, DH>), grid, dim3(128), 0, st, a);
  } else if (attn_wide<DH>(1, a.Sq)) {
    dim3 grid((a.Sq + 255) / 256, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<8, DH>), grid, dim3(512), 0, st, a);
  } else {
    dim3 grid((a.Sq + 127) / 128, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<4, DH>), grid, dim3(256), 0, st, a);
  }
  if (!a.dk) return hipGetLastError();           // only dQ wanted (cross-attention: dK, dV feed the memory gradient)
  if (a.Sk <= 64) {
    dim3 grid((a.Sk + 63) / 64, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<2, DH>), grid, dim3(128), 0, st, a);
  } else if (attn_wide<DH>(2, a.Sk)) {
    dim3 grid((a.Sk + 255) / 256, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<8, DH>), grid, dim3(512), 0, st, a);
  } else {
    dim3 grid((a.Sk + 127) / 128, a.B * a.H, a.n_groups);
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<4, DH>), grid, dim3(256), 0, st, a);
  }
  return hipGetLastError();
}

hipError_t attn_bwd_mfma(const AttnArgs& a, hipStream_t st) {
  return a.dh == 64 ? attn_bwd_mfma_dh<64>(a, st) : attn_bwd_mfma_dh<128>(a, st);
}

}  // namespace mg
