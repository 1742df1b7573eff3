// C ABI, batched layer step (forward and adjoint) and the MGRIT driver.
//
// Everything here is host code that only enqueues kernels on the caller's stream.
//
// Layer step (paper sec. 3.1, eq. "encoder" / "decoder"), per launch chunk of groups:
//   LN1 -> QKV projection -> fused attention -> output projection            (s, fp32)
//   [-> LN3(X+s) -> cross-attention projections -> fused attention -> projection (ybar = s + c)]
//   -> LN2(X+ybar) -> FFN1 (+GELU) -> FFN2 with the Euler update  out = X + h(ybar + m) + rhs
// Adjoint step (the discrete transpose, sec. 3.1 backward problem): the block internals at
// the linearisation state are produced once per layer by a forward pass that stops before
// FFN2 ("linearisation cache": qkv, attention output and log-sum-exp, s, pre-GELU z);
// each adjoint evaluation then runs only the transposed chain.  The cache is independent
// of the step size, so coarse-level adjoint steps reuse the fine layer's entry.
//
// MGRIT driver (sec. 3.2, Fig. 2, Appendix A / Algorithm 1), full-approximation form.
// All levels live in the one [(N+1),T,d] state array: point j of level l is row j*cf^l
// (the reversed row for the adjoint).  Injection and correction are therefore free:
// the coarse solve overwrites the C-points in place.  With R_k = Phi(w_{k cf-1}) + g_{k cf}
// the coarse right-hand side g'_k = what_k - Phi'(what_{k-1}) + (R_k - w_{k cf}) collapses to
// R_k - Phi'(w_{(k-1) cf}) because what_k = w_{k cf}.
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "../../include/mgrit.h"
#include "common.h"
#include "kernels.h"

using namespace mg;

namespace mg { int resnorm_partials_per_group(); }

namespace {

thread_local int g_last_hip_error = 0;
int g_max_groups = 0;                       // 0 = default
constexpr int DEFAULT_MAX_GROUPS = 4;

// Groups per launch chunk for sweeps of `sweep` groups when the caller has not fixed it.  A launch
// runs in whole rounds of tiles over the CUs, so the group count decides how full the last round of
// every projection GEMM is (at d = 768, 5 groups of 4096 tokens make 240 tiles of 256x256 for the
// d-wide outputs, one round; 4 groups need the smaller 256x192 tiles): take the count in 3..6 with the
// smallest modelled GEMM time over the sweep, near-ties (1 %) going to the larger count.
inline int default_groups(const mgrit_model_desc* md, int sweep) {
  if (md->dtype != MGRIT_DTYPE_BF16 || sweep < 2) return DEFAULT_MAX_GROUPS;
  const int T = md->batch * md->seq, d = md->d_model, f = md->d_ff;
  double cost[7] = {0};
  double best = 1e300;
  for (int gc = 3; gc <= 6; ++gc) {
    const int chunk = gc < (sweep + 1) / 2 ? gc : (sweep + 1) / 2;       // as run_chunks splits a sweep over two lanes
    double c = 0.0;
    for (int k = 0; k < sweep; k += chunk) {
      const int n = sweep - k < chunk ? sweep - k : chunk;
      c += gemm_model_cost(n, T, 3 * d, d) + gemm_model_cost(n, T, d, d) + gemm_model_cost(n, T, f, d) +
           gemm_model_cost(n, T, d, f);
    }
    cost[gc] = c;
    if (c < best) best = c;
  }
  int pick = DEFAULT_MAX_GROUPS;
  for (int gc = 3; gc <= 6; ++gc)
    if (cost[gc] <= 1.01 * best) pick = gc;
  return pick;
}
inline int max_groups(const mgrit_model_desc* md, int sweep) {
  return g_max_groups > 0 ? g_max_groups : default_groups(md, sweep);
}

#define HIPCHK(expr)                                   \
  do {                                                 \
    hipError_t e_ = (expr);                            \
    if (e_ != hipSuccess) {                            \
      g_last_hip_error = (int)e_;                      \
      return MGRIT_HIP_ERROR;                          \
    }                                                  \
  } while (0)

#define STCHK(expr)                                    \
  do {                                                 \
    int s_ = (expr);                                   \
    if (s_ != MGRIT_OK) return s_;                     \
  } while (0)

// ---------------------------------------------------------------------------
// parameter block layout
// ---------------------------------------------------------------------------
int compute_layout(const mgrit_model_desc* md, mgrit_theta_layout_t* L) {
  const int d = md->d_model, f = md->d_ff;
  const bool cross = md->arch == MGRIT_ARCH_CROSS;
  const int wbytes = md->dtype == MGRIT_DTYPE_BF16 ? 2 : 4;
  for (int i = 0; i < MGRIT_P_COUNT; ++i) { L->offset[i] = -1; L->rows[i] = L->cols[i] = L->elem_bytes[i] = 0; }
  int64_t off = 0;
  auto vec = [&](int id, int n) {
    L->offset[id] = off; L->rows[id] = n; L->cols[id] = 1; L->elem_bytes[id] = 4;
    off += ((int64_t)n * 4 + 15) / 16 * 16;
  };
  auto mat = [&](int id, int r, int c) {
    L->offset[id] = off; L->rows[id] = r; L->cols[id] = c; L->elem_bytes[id] = wbytes;
    off += ((int64_t)r * c * wbytes + 15) / 16 * 16;
  };
  vec(MGRIT_P_LN1_G, d); vec(MGRIT_P_LN1_B, d); vec(MGRIT_P_BQKV, 3 * d); vec(MGRIT_P_BO, d);
  vec(MGRIT_P_LN2_G, d); vec(MGRIT_P_LN2_B, d); vec(MGRIT_P_B1, f); vec(MGRIT_P_B2, d);
  if (cross) {
    vec(MGRIT_P_LN3_G, d); vec(MGRIT_P_LN3_B, d); vec(MGRIT_P_BQ_C, d); vec(MGRIT_P_BKV_C, 2 * d);
    vec(MGRIT_P_BO_C, d);
  }
  mat(MGRIT_P_WQKV, 3 * d, d); mat(MGRIT_P_WO, d, d); mat(MGRIT_P_W1, f, d); mat(MGRIT_P_W2, d, f);
  if (cross) { mat(MGRIT_P_WQ_C, d, d); mat(MGRIT_P_WKV_C, 2 * d, d); mat(MGRIT_P_WO_C, d, d); }
  L->block_bytes = (off + 255) / 256 * 256;
  return MGRIT_OK;
}

int validate_desc(const mgrit_model_desc* md) {
  if (!md) return MGRIT_INVALID_ARG;
  if (md->arch < 0 || md->arch > 2) return MGRIT_INVALID_ARG;
  if (md->dtype != MGRIT_DTYPE_F32 && md->dtype != MGRIT_DTYPE_BF16) return MGRIT_INVALID_ARG;
  if (md->d_model <= 0 || md->n_heads <= 0 || md->d_ff <= 0 || md->batch <= 0 || md->seq <= 0)
    return MGRIT_INVALID_ARG;
  if (md->d_model % md->n_heads != 0) return MGRIT_INVALID_ARG;
  if (md->arch == MGRIT_ARCH_CROSS ? md->mem_seq <= 0 : md->mem_seq != 0) return MGRIT_INVALID_ARG;
  if (!(md->ln_eps > 0.f) || !isfinite(md->ln_eps)) return MGRIT_INVALID_ARG;
  const int dh = md->d_model / md->n_heads;
  // kernel limits of this build
  if (md->d_model % 8 || md->d_ff % 8 || dh % 4 || dh > 128 || md->d_model > 2048) return MGRIT_UNSUPPORTED;
  if ((int64_t)md->batch * md->seq > (1 << 24)) return MGRIT_UNSUPPORTED;
  return MGRIT_OK;
}

int validate_opts(const mgrit_opts* o) {
  if (!o) return MGRIT_INVALID_ARG;
  if (o->N < 1 || o->cf < 1 || o->levels < 1 || o->iters < 0) return MGRIT_INVALID_ARG;
  if (!isfinite(o->h)) return MGRIT_INVALID_ARG;
  if (o->relax != MGRIT_RELAX_F && o->relax != MGRIT_RELAX_FCF) return MGRIT_INVALID_ARG;
  if (o->init_guess != 0 && o->init_guess != 1) return MGRIT_INVALID_ARG;
  if (o->levels > 1 && o->cf > 1) {
    int64_t p = 1;
    for (int l = 1; l < o->levels; ++l) {
      p *= o->cf;
      if (p > o->N) return MGRIT_INVALID_ARG;
    }
    if (o->N % p != 0) return MGRIT_INVALID_ARG;
    // without a V-cycle the F-points of the output would never be written
    if (o->iters < 1) return MGRIT_INVALID_ARG;
  }
  return MGRIT_OK;
}

inline bool serial_run(const mgrit_opts* o) { return o->levels == 1 || o->cf == 1; }

// ---------------------------------------------------------------------------
// workspace carving (same code measures and allocates)
// ---------------------------------------------------------------------------
struct Bump {
  char* base;
  size_t off = 0;
  explicit Bump(void* b) : base(static_cast<char*>(b)) {}
  template <typename T> T* take(size_t count) {
    off = (off + 255) / 256 * 256;
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
  void* take_bytes(size_t bytes) { return take<char>(bytes); }
};

struct Engine {
  mgrit_model_desc md;
  mgrit_theta_layout_t lay;
  bool bf16;
  int T, Tm, d, f, H, dh;
  size_t esz;                      // operand element size
  hipStream_t st;
  int Gc;                          // groups per launch chunk
  // forward work buffers, Gc slots each
  void *u, *qkv, *o, *act, *qc, *kvc, *memb;
  float *xin, *x3;
  // adjoint: linearisation cache (n_cache slots) and work buffers (Gc slots)
  int n_cache;
  void *c_qkv, *c_o, *c_z;         // c_z holds gelu'(z): the adjoint only needs the derivative
  void* c_zraw = nullptr;          // z itself, kept when parameter gradients are wanted (W2's needs GELU(z))
  bool keep_z = false;
  float *c_lse, *c_xin;
  void *c_xh1, *c_xh2;             // normalised LN1 / LN2 inputs (operand type) ...
  float *c_rs1, *c_rs2;            // ... and their 1/std, one per token
  void *c_qc, *c_kvc, *c_oc;       // cross-attention decoder only
  float *c_lsec, *c_x3;
  void *cb, *dz, *du, *ds, *da, *dqkv;
  float *dxin, *Dbuf;
  // parameter-gradient pass: transposed operands (Gc slots each), token-sum partials, table of tB slots
  mgrit_theta_layout_t glay;       // layout of a gradient block: the fp32 parameter block of the model
  void *tA = nullptr, *tB = nullptr;
  float* gpart = nullptr;
  void** tabTB = nullptr;
  void* dkvc = nullptr;            // cross-attention decoder: dK | dV of the cross attention, [Tm, 2d] per slot
  // decoder half of a stacked encoder-decoder grid: every group attends to the X part of its own
  // input state, so the operand-type copy of the memory is per launch slot ([Tm, d] each)
  bool per_group_mem = false;
  void* membG = nullptr;
  // adjoint without the N-layer linearisation cache: the cache arrays hold one launch chunk (Gc slots,
  // one set per lane) and every chunk of transposed steps first recomputes the internals of its layers
  bool recompute = false;
  // sign of the step inside OUT = RHS + sign * (step): -1 while the driver forms a coarse right-hand side
  float rhs_sign = 1.f;
  int Tmax() const { return T > Tm ? T : Tm; }
  long tA_stride() const { return (long)(f > 3 * d ? f : 3 * d) * Tmax(); }   // elements per slot
  long tB_stride() const { return (long)(f > d ? f : d) * Tmax(); }

  long Td() const { return (long)T * d; }

  void init(const mgrit_model_desc* m, hipStream_t s) {
    md = *m;
    compute_layout(m, &lay);
    bf16 = m->dtype == MGRIT_DTYPE_BF16;
    T = m->batch * m->seq; Tm = m->batch * m->mem_seq; d = m->d_model; f = m->d_ff; H = m->n_heads;
    dh = d / H; esz = bf16 ? 2 : 4; st = s;
    mgrit_model_desc m32 = *m;
    m32.dtype = MGRIT_DTYPE_F32;
    compute_layout(&m32, &glay);
  }
  // work buffers of one lane (a lane = a stream with its own intermediates)
  void carve_forward_work(Bump& b, int gc) {
    Gc = gc;
    const size_t G = gc;
    u = b.take_bytes(G * T * d * esz);
    qkv = b.take_bytes(G * T * 3 * d * esz);
    o = b.take_bytes(G * T * d * esz);
    xin = b.take<float>(G * T * d);
    act = b.take_bytes(G * T * f * esz);
    x3 = nullptr; qc = kvc = nullptr;
    if (md.arch == MGRIT_ARCH_CROSS) {
      x3 = b.take<float>(G * T * d);
      qc = b.take_bytes(G * T * d * esz);
      kvc = b.take_bytes(G * Tm * 2 * d * esz);
      if (per_group_mem) membG = b.take_bytes(G * Tm * d * esz);
    }
  }
  void carve_forward(Bump& b, int gc) {
    memb = md.arch == MGRIT_ARCH_CROSS ? b.take_bytes((size_t)Tm * d * esz) : nullptr;
    carve_forward_work(b, gc);
  }
  void carve_cache(Bump& b, int ncache) {
    n_cache = ncache;
    const size_t C = ncache;
    c_qkv = b.take_bytes(C * T * 3 * d * esz);
    c_o = b.take_bytes(C * T * d * esz);
    c_z = b.take_bytes(C * T * f * esz);
    c_zraw = keep_z ? b.take_bytes(C * T * f * esz) : nullptr;
    c_lse = b.take<float>(C * md.batch * H * md.seq);
    c_xin = b.take<float>(C * T * d);
    c_xh1 = b.take_bytes(C * T * d * esz);
    c_xh2 = b.take_bytes(C * T * d * esz);
    c_rs1 = b.take<float>(C * T);
    c_rs2 = b.take<float>(C * T);
    c_qc = c_kvc = c_oc = nullptr; c_lsec = c_x3 = nullptr;
    if (md.arch == MGRIT_ARCH_CROSS) {
      c_qc = b.take_bytes(C * T * d * esz);
      c_kvc = b.take_bytes(C * Tm * 2 * d * esz);
      c_oc = b.take_bytes(C * T * d * esz);
      c_lsec = b.take<float>(C * md.batch * H * md.seq);
      c_x3 = b.take<float>(C * T * d);
    }
  }
  // the cache pointers of an engine laid out elsewhere (a forward plan that fills an adjoint plan's cache)
  void take_cache_from(const Engine& o) {
    n_cache = o.n_cache; keep_z = o.keep_z;
    c_qkv = o.c_qkv; c_o = o.c_o; c_z = o.c_z; c_zraw = o.c_zraw; c_lse = o.c_lse; c_xin = o.c_xin;
    c_xh1 = o.c_xh1; c_xh2 = o.c_xh2; c_rs1 = o.c_rs1; c_rs2 = o.c_rs2;
    c_qc = o.c_qc; c_kvc = o.c_kvc; c_oc = o.c_oc; c_lsec = o.c_lsec; c_x3 = o.c_x3;
  }
  void carve_adjoint(Bump& b, int gc, int ncache) {
    carve_cache(b, recompute ? gc : ncache);
    memb = md.arch == MGRIT_ARCH_CROSS ? b.take_bytes((size_t)Tm * d * esz) : nullptr;
    carve_adjoint_work(b, gc);
  }
  void carve_adjoint_work(Bump& b, int gc) {
    Gc = gc;
    const size_t G = gc;
    u = b.take_bytes(G * T * d * esz);
    cb = b.take_bytes(G * T * d * esz);
    dz = b.take_bytes(G * T * f * esz);
    du = b.take_bytes(G * T * d * esz);
    ds = b.take_bytes(G * T * d * esz);
    da = b.take_bytes(G * T * d * esz);
    dqkv = b.take_bytes(G * T * 3 * d * esz);
    dxin = b.take<float>(G * T * d);
    Dbuf = b.take<float>(G * md.batch * H * md.seq);
    qkv = o = act = nullptr; xin = nullptr;
    if (per_group_mem) {
      membG = b.take_bytes(G * Tm * d * esz);
      dkvc = b.take_bytes(G * Tm * 2 * d * esz);
    }
  }
  void carve_grad_work(Bump& b) {
    const size_t G = Gc;
    tA = b.take_bytes(G * tA_stride() * esz);
    tB = b.take_bytes(G * tB_stride() * esz);
    const size_t widest = f > 3 * d ? f : 3 * d;
    const size_t p1 = G * transpose_row_blocks(Tmax()) * widest, p2 = G * ln_param_partial_rows() * 2 * (size_t)d;
    gpart = b.take<float>(p1 > p2 ? p1 : p2);
    tabTB = b.take<void*>(G);
    if (!per_group_mem) dkvc = md.arch == MGRIT_ARCH_CROSS ? b.take_bytes(G * Tm * 2 * d * esz) : nullptr;
  }
};

// Second lane: independent chunks of a sweep alternate between the caller's stream and one
// helper stream (forked from and joined back into the caller's stream with events), so that
// the bandwidth-bound kernels of one chunk overlap the matrix kernels of the other.  The
// helper stream and its events (fork, join and a pool for the hand-overs of the overlapped coarse
// solve) are created once per device, on first use.
constexpr int PIPE_EVENTS = 32;
struct AuxStream {
  hipStream_t s = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  hipEvent_t pipe[PIPE_EVENTS] = {};     // hand-overs from the serial coarse solve to the helper lane
  bool tried = false, ok = false;
};
// One helper lane per device, created on first use with that device current.  Calls are serialised on
// the host while they enqueue (g_call_mutex, taken by every entry point that launches work), so the
// lane's stream and events are never used by two calls at once: hipStreamWaitEvent takes the event's
// state when it is enqueued, and a call has enqueued all its waits before the next call records again.
constexpr int MAX_AUX_DEVICES = 64;
std::recursive_mutex g_call_mutex;
AuxStream& aux_stream() {
  static AuxStream table[MAX_AUX_DEVICES];
  static AuxStream none;                    // ok == false: no second lane
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_AUX_DEVICES) return none;
  AuxStream& a = table[dev];
  if (!a.tried) {
    a.tried = true;
    a.ok = hipStreamCreateWithFlags(&a.s, hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&a.fork, hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&a.join, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; a.ok && i < PIPE_EVENTS; ++i)
      a.ok = hipEventCreateWithFlags(&a.pipe[i], hipEventDisableTiming) == hipSuccess;
  }
  return a;
}
int g_adjoint_cache = 1;                    // 0 = no N-layer linearisation cache: recompute per launch chunk
int g_lanes = 2;                            // 1 = everything on the caller's stream
int g_pipeline = 1;                         // overlap the serial coarse solve with the F-relaxation that follows it
int g_pipe_chunk = 0;                       // intervals per hand-over (0 = the launch chunk)

// Engine of the second lane: same model and shared buffers, own work buffers and stream.
inline bool make_lane(Engine& E2, const Engine& E, Bump& b, bool adjoint, bool measure_only) {
  if (g_lanes < 2) return false;
  E2 = E;
  if (adjoint && E.recompute) E2.carve_cache(b, E.Gc);      // lanes run at the same time: one chunk-sized cache each
  if (adjoint) E2.carve_adjoint_work(b, E.Gc); else E2.carve_forward_work(b, E.Gc);
  if (measure_only) return true;
  AuxStream& a = aux_stream();
  if (!a.ok) return false;
  E2.st = a.s;
  return true;
}

inline Rows shift(Rows r, int c0) { if (r.tab) r.i0 += c0 * r.is; return r; }
inline Params shift(Params p, int c0) { p.i0 += c0 * p.is; return p; }
inline Slots shift(Slots s, int c0) { s.s0 += c0 * s.ss; return s; }
const Rows NO_ROWS = {nullptr, 0, 0};

GemmArgs gemm_base(int n, int M, int N, int K, const void* A, long a_stride, Slots a_slots, Params B, long b_off,
                   long bias_off) {
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.n_groups = n; g.M = M; g.N = N; g.K = K;
  g.A = A; g.a_slot_stride = a_stride; g.a_slots = a_slots;
  g.B = B; g.b_off = b_off; g.bias = B; g.bias_off = bias_off;
  g.rhs_sign = 1.f;
  return g;
}

// One chunk (n <= Gc groups) of the forward layer step.  `cache`: write the linearisation
// cache at `cslots` instead of advancing the state (stops before FFN2).
// MEM (decoder of a stacked grid): group g's cross-attention memory is the fp32 rows MEM.at(g).
// cache: 0 = the plain step; 1 = fill the layers' entries of the linearisation cache (slots cslots)
// and stop before the second feed-forward product (no state written); 2 = the whole step, leaving
// those entries on the way (the step's intermediates live in the cache slots instead of the lane's
// work buffers, and the first feed-forward product writes gelu(z) and gelu'(z) in one epilogue).
int forward_chunk(Engine& E, int n, Rows IN, Rows OUT, Rows RHS, Params TH, float hstep, int cache,
                  Slots cslots, Rows MEM = NO_ROWS) {
  const int T = E.T, d = E.d, f = E.f;
  const auto& L = E.lay;
  const Slots loc = {0, 1};
  const Slots cs = cache ? cslots : loc;
  void* qkv = cache ? E.c_qkv : E.qkv;
  void* ob = cache ? E.c_o : E.o;
  float* xin = cache ? E.c_xin : E.xin;
  const size_t esz = E.esz;
  const bool causal = E.md.arch != MGRIT_ARCH_ENCODER;

  LnFwdArgs ln;
  memset(&ln, 0, sizeof(ln));
  ln.n_groups = n; ln.T = T; ln.d = d; ln.X = IN; ln.P = TH;
  ln.gamma_off = L.offset[MGRIT_P_LN1_G]; ln.beta_off = L.offset[MGRIT_P_LN1_B];
  ln.out = E.u; ln.out_slot_stride = E.Td(); ln.out_slots = loc; ln.eps = E.md.ln_eps;
  if (cache) { ln.xhat = E.c_xh1; ln.xhat_slot_stride = E.Td(); ln.xhat_slots = cs; ln.rstd = E.c_rs1; }
  HIPCHK(launch_ln_fwd(ln, E.bf16, E.st));
  ln.xhat = nullptr; ln.rstd = nullptr;

  GemmArgs g = gemm_base(n, T, 3 * d, d, E.u, E.Td(), loc, TH, L.offset[MGRIT_P_WQKV], L.offset[MGRIT_P_BQKV]);
  g.out = qkv; g.out_slot_stride = (long)T * 3 * d; g.out_slots = cs;
  HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));

  AttnArgs at;
  memset(&at, 0, sizeof(at));
  at.n_groups = n; at.B = E.md.batch; at.H = E.H; at.dh = E.dh; at.Sq = E.md.seq; at.Sk = E.md.seq;
  at.causal = causal;
  at.q = qkv; at.k = (char*)qkv + (size_t)d * esz; at.v = (char*)qkv + (size_t)2 * d * esz;
  at.q_row_stride = at.k_row_stride = at.v_row_stride = 3 * d;
  at.q_slot_stride = at.k_slot_stride = at.v_slot_stride = (long)T * 3 * d;
  at.q_slots = at.k_slots = cs;
  at.o = ob; at.o_row_stride = d; at.o_slot_stride = E.Td(); at.o_slots = cs;
  if (cache) { at.lse = E.c_lse; at.lse_slot_stride = (long)E.md.batch * E.H * E.md.seq; at.lse_slots = cs; }
  HIPCHK(launch_attn_fwd(at, E.bf16, E.st));

  const bool cross = E.md.arch == MGRIT_ARCH_CROSS;
  float* x3 = cache ? E.c_x3 : E.x3;
  // s = SA(LN1(X)) kept in fp32 (never X + s: the Euler sum must not lose the small increment)
  g = gemm_base(n, T, d, d, ob, E.Td(), cs, TH, L.offset[MGRIT_P_WO], L.offset[MGRIT_P_BO]);
  g.out = cross ? x3 : xin; g.out_slot_stride = E.Td(); g.out_slots = cs;
  HIPCHK(launch_gemm(g, EPI_RESID_INNER, E.bf16, E.st));

  if (cross) {
    void* qc = cache ? E.c_qc : E.qc;
    void* kvc = cache ? E.c_kvc : E.kvc;
    void* oc = cache ? E.c_oc : E.o;
    ln.X = IN; ln.xp = x3; ln.xp_slot_stride = E.Td(); ln.xp_slots = cs;         // LN3(X + s)
    ln.gamma_off = L.offset[MGRIT_P_LN3_G]; ln.beta_off = L.offset[MGRIT_P_LN3_B];
    HIPCHK(launch_ln_fwd(ln, E.bf16, E.st));
    g = gemm_base(n, T, d, d, E.u, E.Td(), loc, TH, L.offset[MGRIT_P_WQ_C], L.offset[MGRIT_P_BQ_C]);
    g.out = qc; g.out_slot_stride = E.Td(); g.out_slots = cs;
    HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));
    if (MEM.present()) HIPCHK(launch_cast_rows(n, (long)E.Tm * d, MEM, E.membG, (long)E.Tm * d, loc, E.bf16, E.st));
    g = gemm_base(n, E.Tm, 2 * d, d, MEM.present() ? E.membG : E.memb, MEM.present() ? (long)E.Tm * d : 0, loc, TH,
                  L.offset[MGRIT_P_WKV_C], L.offset[MGRIT_P_BKV_C]);
    g.out = kvc; g.out_slot_stride = (long)E.Tm * 2 * d; g.out_slots = cs;
    HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));
    memset(&at, 0, sizeof(at));
    at.n_groups = n; at.B = E.md.batch; at.H = E.H; at.dh = E.dh; at.Sq = E.md.seq; at.Sk = E.md.mem_seq;
    at.causal = 0;
    at.q = qc; at.q_row_stride = d; at.q_slot_stride = E.Td(); at.q_slots = cs;
    at.k = kvc; at.v = (char*)kvc + (size_t)d * esz;
    at.k_row_stride = at.v_row_stride = 2 * d;
    at.k_slot_stride = at.v_slot_stride = (long)E.Tm * 2 * d; at.k_slots = cs;
    at.o = oc; at.o_row_stride = d; at.o_slot_stride = E.Td(); at.o_slots = cs;
    if (cache) { at.lse = E.c_lsec; at.lse_slot_stride = (long)E.md.batch * E.H * E.md.seq; at.lse_slots = cs; }
    HIPCHK(launch_attn_fwd(at, E.bf16, E.st));
    g = gemm_base(n, T, d, d, oc, E.Td(), cs, TH, L.offset[MGRIT_P_WO_C], L.offset[MGRIT_P_BO_C]);
    g.base = x3; g.base_slot_stride = E.Td(); g.base_slots = cs;
    g.out = xin; g.out_slot_stride = E.Td(); g.out_slots = cs;
    HIPCHK(launch_gemm(g, EPI_RESID_INNER, E.bf16, E.st));
  }

  ln.X = IN; ln.xp = xin; ln.xp_slot_stride = E.Td(); ln.xp_slots = cs;          // LN2(X + ybar)
  ln.gamma_off = L.offset[MGRIT_P_LN2_G]; ln.beta_off = L.offset[MGRIT_P_LN2_B];
  if (cache) { ln.xhat = E.c_xh2; ln.xhat_slot_stride = E.Td(); ln.xhat_slots = cs; ln.rstd = E.c_rs2; }
  HIPCHK(launch_ln_fwd(ln, E.bf16, E.st));

  g = gemm_base(n, T, f, d, E.u, E.Td(), loc, TH, L.offset[MGRIT_P_W1], L.offset[MGRIT_P_B1]);
  if (cache == 1) {
    g.out = E.c_z; g.out_slot_stride = (long)T * f; g.out_slots = cs;
    g.aux = E.c_zraw; g.aux_slot_stride = (long)T * f; g.aux_slots = cs;
    HIPCHK(launch_gemm(g, EPI_GELU_PRIME, E.bf16, E.st));
    return MGRIT_OK;
  }
  g.out = E.act; g.out_slot_stride = (long)T * f; g.out_slots = loc;
  if (cache) {
    g.aux2 = E.c_z; g.aux2_slot_stride = (long)T * f; g.aux2_slots = cs;
    g.aux = E.c_zraw; g.aux_slot_stride = (long)T * f; g.aux_slots = cs;
    HIPCHK(launch_gemm(g, EPI_GELU_BOTH, E.bf16, E.st));
  } else {
    HIPCHK(launch_gemm(g, EPI_GELU, E.bf16, E.st));
  }

  g = gemm_base(n, T, d, f, E.act, (long)T * f, loc, TH, L.offset[MGRIT_P_W2], L.offset[MGRIT_P_B2]);
  g.aux = xin; g.aux_slot_stride = E.Td(); g.aux_slots = cs;                    // ybar
  g.X = IN; g.OUT = OUT; g.RHS = RHS; g.hstep = hstep; g.rhs_sign = E.rhs_sign;
  HIPCHK(launch_gemm(g, EPI_RESID_OUTER, E.bf16, E.st));
  return MGRIT_OK;
}

// Weight and bias gradient of one linear map y = u W^T + b of the chunk's layers:
//   dW[out,in] = scale * dY^T U,  db[out] = scale * sum over tokens of dY,
// dY [T,out] and U [T,in] packed operand-type buffers.  The product runs on the same
// "both operands reduction-contiguous" GEMM, on transposed copies of dY and U (reduction over
// the T tokens); gelu_u: U = GELU(given buffer).  Results go into the layers' gradient blocks.
int linear_param_grads(Engine& E, int n, const void* dY, long dy_stride, Slots dy_slots, int out_dim,
                       const void* U, long u_stride, Slots u_slots, int in_dim, bool gelu_u, Params DT,
                       int w_id, int b_id, float scale, int tokens = 0) {
  const Slots loc = {0, 1};
  const int T = tokens ? tokens : E.T;
  const Params none = {nullptr, 0, 0};
  HIPCHK(launch_transpose_slots(n, dY, dy_stride, dy_slots, T, out_dim, E.tA, E.tA_stride(), loc, false, E.bf16,
                                E.gpart, DT, E.glay.offset[b_id], scale, E.st));
  HIPCHK(launch_transpose_slots(n, U, u_stride, u_slots, T, in_dim, E.tB, E.tB_stride(), loc, gelu_u, E.bf16,
                                nullptr, none, 0, 0.f, E.st));
  GemmArgs g = gemm_base(n, out_dim, in_dim, T, E.tA, E.tA_stride(), loc, Params{(const void* const*)E.tabTB, 0, 1},
                         0, -1);
  g.out_tab = DT; g.out_tab_off = E.glay.offset[w_id]; g.hstep = scale;
  HIPCHK(launch_gemm(g, EPI_STORE_F32, E.bf16, E.st));
  return MGRIT_OK;
}

// One chunk of the adjoint step:  OUT = IN + hstep * J(LIN; theta)^T IN (+ RHS), from the cache.
// THT: parameter blocks whose matrices are stored transposed; TH: the original blocks.
// With DT (gradient blocks of the chunk's layers) the chunk is a parameter-gradient pass instead:
// the same backward chain with IN = lambda_{n+1}, every linear map and LayerNorm also emitting
// hstep * (its parameter cotangent), and no state written (paper section 3.1: theta enters the
// step only through h F, so dtheta_n = h (dF/dtheta_n (Z_n))^T lambda_{n+1}).
struct GradPass {
  const Params* DT = nullptr;      // gradient blocks of the chunk's layers, or null
  float* dE_all = nullptr;         // cross-attention decoder: [layer slot, Tm, d] fp32 memory-gradient terms, or null
  Slots dE_slots = {0, 1};         // layer slots of the chunk's groups in dE_all
  bool write_state = false;        // also finish the step (OUT written): a relaxation step that emits its layer's gradients
};
// Decoder step of a stacked encoder-decoder grid (paper section 3.1, eq. "fp_transformer"): the
// memory of group g is the X part of its linearisation state, and the transposed step adds the
// memory cotangent to the X part of the adjoint state:  OUTX = INX + hstep * dE (+ RHSX).
struct StackedDec {
  Rows MEM, INX, OUTX, RHSX;
};
inline StackedDec shift(StackedDec s, int c0) {
  s.MEM = shift(s.MEM, c0); s.INX = shift(s.INX, c0); s.OUTX = shift(s.OUTX, c0); s.RHSX = shift(s.RHSX, c0);
  return s;
}

// Operand-type copies of adjoint states, one [T, d] slot per grid point (index of the driver's point table):
// a transposed step starts from the operand-type copy of its input, and the kernel that writes a step's
// output state can write that copy on the way.  in: the copies of this chunk's inputs are there (no cast
// needed); out: where to leave the copies of its outputs.
struct CastShadow {
  const void* in = nullptr; Slots in_slots = {0, 1};
  void* out = nullptr; Slots out_slots = {0, 1};
  const char* valid = nullptr;            // per grid point: its copy is current (checked per launch chunk)
  bool have_inputs(int n) const {
    if (!in || !valid) return false;
    for (int g = 0; g < n; ++g) if (!valid[in_slots.of(g)]) return false;
    return true;
  }
};
inline CastShadow shift(CastShadow c, int c0) { c.in_slots = shift(c.in_slots, c0); c.out_slots = shift(c.out_slots, c0); return c; }

int adjoint_chunk(Engine& E, int n, Rows IN, Rows OUT, Rows RHS, Params TH, Params THT, Rows LIN, Slots cs,
                  float hstep, const GradPass* gp = nullptr, const StackedDec* sd = nullptr,
                  const CastShadow* sh = nullptr) {
  const Params* DT = gp ? gp->DT : nullptr;
  const int T = E.T, d = E.d, f = E.f;
  const auto& L = E.lay;
  const Slots loc = {0, 1};
  const size_t esz = E.esz;

  const void* cbuf = E.cb;                 // operand-type copy of the inputs
  Slots cbs = loc;
  if (sh && sh->have_inputs(n)) { cbuf = sh->in; cbs = sh->in_slots; }
  else HIPCHK(launch_cast_rows(n, E.Td(), IN, E.cb, E.Td(), loc, E.bf16, E.st));
  LnFwdArgs lf;
  LnParamArgs lp;
  memset(&lf, 0, sizeof(lf));
  memset(&lp, 0, sizeof(lp));
  if (DT) {
    // m = GELU(z) W2^T + b2
    STCHK(linear_param_grads(E, n, cbuf, E.Td(), cbs, d, E.c_zraw, (long)T * f, cs, f, true, *DT, MGRIT_P_W2,
                             MGRIT_P_B2, hstep));
    lf.n_groups = n; lf.T = T; lf.d = d; lf.X = LIN; lf.P = TH; lf.eps = E.md.ln_eps;
    lf.out = E.u; lf.out_slot_stride = E.Td(); lf.out_slots = loc;
    lp.n_groups = n; lp.T = T; lp.d = d; lp.X = LIN; lp.out = *DT; lp.scale = hstep; lp.eps = E.md.ln_eps;
    lp.dy = E.du; lp.dy_slot_stride = E.Td(); lp.dy_slots = loc;
  }

  // dz = (c W2) * gelu'(z)        [T,d] x [d,f]: transposed W2 is [f,d]; gelu'(z) comes from the cache
  GemmArgs g = gemm_base(n, T, f, d, cbuf, E.Td(), cbs, THT, L.offset[MGRIT_P_W2], -1);
  g.out = E.dz; g.out_slot_stride = (long)T * f; g.out_slots = loc;
  g.aux = E.c_z; g.aux_slot_stride = (long)T * f; g.aux_slots = cs;
  HIPCHK(launch_gemm(g, EPI_DGELU, E.bf16, E.st));
  if (DT) {
    // z = LN2(X + ybar) W1^T + b1
    lf.xp = E.c_xin; lf.xp_slot_stride = E.Td(); lf.xp_slots = cs;
    lf.gamma_off = L.offset[MGRIT_P_LN2_G]; lf.beta_off = L.offset[MGRIT_P_LN2_B];
    HIPCHK(launch_ln_fwd(lf, E.bf16, E.st));
    STCHK(linear_param_grads(E, n, E.dz, (long)T * f, loc, f, E.u, E.Td(), loc, d, false, *DT, MGRIT_P_W1,
                             MGRIT_P_B1, hstep));
  }

  // du2 = dz W1                   [T,f] x [f,d]: transposed W1 is [d,f]
  g = gemm_base(n, T, d, f, E.dz, (long)T * f, loc, THT, L.offset[MGRIT_P_W1], -1);
  g.out = E.du; g.out_slot_stride = E.Td(); g.out_slots = loc;
  HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));

  if (DT) {
    lp.xp = E.c_xin; lp.xp_slot_stride = E.Td(); lp.xp_slots = cs;
    lp.gamma_off = E.glay.offset[MGRIT_P_LN2_G]; lp.beta_off = E.glay.offset[MGRIT_P_LN2_B];
    HIPCHK(launch_ln_param_grad(lp, E.gpart, E.bf16, E.st));
  }

  // dX' = LN2^T du2 ;  ds = c + dX'
  LnBwdArgs lb;
  memset(&lb, 0, sizeof(lb));
  lb.n_groups = n; lb.T = T; lb.d = d; lb.eps = E.md.ln_eps;
  lb.dy = E.du; lb.dy_slot_stride = E.Td(); lb.dy_slots = loc;
  lb.xhat = E.c_xh2; lb.xhat_slot_stride = E.Td(); lb.xhat_slots = cs; lb.rstd = E.c_rs2;   // LN2 input X + ybar
  lb.P = TH; lb.gamma_off = L.offset[MGRIT_P_LN2_G];
  lb.out_f32 = E.dxin; lb.of_slot_stride = E.Td(); lb.of_slots = loc;
  lb.cop = cbuf; lb.cop_slot_stride = E.Td(); lb.cop_slots = cbs;
  lb.out_op = E.ds; lb.oo_slot_stride = E.Td(); lb.oo_slots = loc;
  HIPCHK(launch_ln_bwd(lb, E.bf16, E.st));

  if (E.md.arch == MGRIT_ARCH_CROSS) {
    // Here ds = c + dx2 is the cotangent of ybar = s + CA(LN3(Y + s), E); dxin = dx2.
    // c = o_c Wo_c^T + bo_c
    if (DT)
      STCHK(linear_param_grads(E, n, E.ds, E.Td(), loc, d, E.c_oc, E.Td(), cs, d, false, *DT, MGRIT_P_WO_C,
                               MGRIT_P_BO_C, hstep));
    // do_c = ds Wo_c
    g = gemm_base(n, T, d, d, E.ds, E.Td(), loc, THT, L.offset[MGRIT_P_WO_C], -1);
    g.out = E.da; g.out_slot_stride = E.Td(); g.out_slots = loc;
    HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));
    // cross-attention backward: lambda needs dQ only; dK, dV feed the gradients of Wkv_c and of the memory
    AttnArgs ac;
    memset(&ac, 0, sizeof(ac));
    ac.n_groups = n; ac.B = E.md.batch; ac.H = E.H; ac.dh = E.dh; ac.Sq = E.md.seq; ac.Sk = E.md.mem_seq;
    ac.causal = 0;
    ac.q = E.c_qc; ac.q_row_stride = d; ac.q_slot_stride = E.Td(); ac.q_slots = cs;
    ac.k = E.c_kvc; ac.v = (char*)E.c_kvc + (size_t)d * esz;
    ac.k_row_stride = ac.v_row_stride = 2 * d;
    ac.k_slot_stride = ac.v_slot_stride = (long)E.Tm * 2 * d; ac.k_slots = cs;
    ac.o = E.c_oc; ac.o_row_stride = d; ac.o_slot_stride = E.Td(); ac.o_slots = cs;
    ac.lse = E.c_lsec; ac.lse_slot_stride = (long)E.md.batch * E.H * E.md.seq; ac.lse_slots = cs;
    ac.dO = E.da; ac.do_row_stride = d; ac.do_slot_stride = E.Td(); ac.do_slots = loc;
    ac.dq = E.dqkv; ac.dk = nullptr; ac.dv = nullptr;
    ac.dqkv_row_stride = d; ac.dqkv_slot_stride = (long)T * 3 * d; ac.dqkv_slots = loc;
    if (gp || sd) {
      ac.dk = E.dkvc; ac.dv = (char*)E.dkvc + (size_t)d * esz;
      ac.dkv_row_stride = 2 * d; ac.dkv_slot_stride = (long)E.Tm * 2 * d;
    }
    ac.D = E.Dbuf; ac.D_slot_stride = (long)E.md.batch * E.H * E.md.seq; ac.D_slots = loc;
    HIPCHK(launch_attn_bwd(ac, E.bf16, E.st));
    if (DT) {
      // q_c = LN3(Y + s) Wq_c^T + bq_c ;  [k_c | v_c] = E Wkv_c^T + bkv_c
      lf.xp = E.c_x3; lf.xp_slot_stride = E.Td(); lf.xp_slots = cs;
      lf.gamma_off = L.offset[MGRIT_P_LN3_G]; lf.beta_off = L.offset[MGRIT_P_LN3_B];
      HIPCHK(launch_ln_fwd(lf, E.bf16, E.st));
      STCHK(linear_param_grads(E, n, E.dqkv, (long)T * 3 * d, loc, d, E.u, E.Td(), loc, d, false, *DT,
                               MGRIT_P_WQ_C, MGRIT_P_BQ_C, hstep));
      if (sd) HIPCHK(launch_cast_rows(n, (long)E.Tm * d, sd->MEM, E.membG, (long)E.Tm * d, loc, E.bf16, E.st));
      STCHK(linear_param_grads(E, n, E.dkvc, (long)E.Tm * 2 * d, loc, 2 * d, sd ? E.membG : E.memb,
                               sd ? (long)E.Tm * d : 0, loc, d, false, *DT, MGRIT_P_WKV_C, MGRIT_P_BKV_C, hstep, E.Tm));
    }
    if (sd && (!gp || gp->write_state)) {
      // lambda_X <- lambda_X + hstep * [dK | dV] Wkv_c (+ rhs)    [Tm,2d] x [2d,d]: transposed Wkv_c is [d,2d]
      g = gemm_base(n, E.Tm, d, 2 * d, E.dkvc, (long)E.Tm * 2 * d, loc, THT, L.offset[MGRIT_P_WKV_C], -1);
      g.X = sd->INX; g.OUT = sd->OUTX; g.RHS = sd->RHSX; g.hstep = hstep;
      HIPCHK(launch_gemm(g, EPI_RESID_OUTER, E.bf16, E.st));
    }
    if (gp && gp->dE_all) {
      // this layer's term of dL/dE:  hstep * [dK | dV] Wkv_c       [Tm,2d] x [2d,d]: transposed Wkv_c is [d,2d]
      g = gemm_base(n, E.Tm, d, 2 * d, E.dkvc, (long)E.Tm * 2 * d, loc, THT, L.offset[MGRIT_P_WKV_C], -1);
      g.out = gp->dE_all; g.out_slot_stride = (long)E.Tm * d; g.out_slots = gp->dE_slots; g.hstep = hstep;
      HIPCHK(launch_gemm(g, EPI_STORE_F32, E.bf16, E.st));
    }
    // du3 = dq_c Wq_c
    g = gemm_base(n, T, d, d, E.dqkv, (long)T * 3 * d, loc, THT, L.offset[MGRIT_P_WQ_C], -1);
    g.out = E.du; g.out_slot_stride = E.Td(); g.out_slots = loc;
    HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));
    if (DT) {
      lp.xp = E.c_x3; lp.xp_slot_stride = E.Td(); lp.xp_slots = cs;
      lp.gamma_off = E.glay.offset[MGRIT_P_LN3_G]; lp.beta_off = E.glay.offset[MGRIT_P_LN3_B];
      HIPCHK(launch_ln_param_grad(lp, E.gpart, E.bf16, E.st));
    }
    // dx3 = LN3^T du3 at Y + s;  dxin <- dx2 + dx3 (in place);  ds <- c + dx2 + dx3
    memset(&lb, 0, sizeof(lb));
    lb.n_groups = n; lb.T = T; lb.d = d; lb.eps = E.md.ln_eps;
    lb.dy = E.du; lb.dy_slot_stride = E.Td(); lb.dy_slots = loc;
    lb.X = LIN; lb.xp = E.c_x3; lb.xp_slot_stride = E.Td(); lb.xp_slots = cs;
    lb.P = TH; lb.gamma_off = L.offset[MGRIT_P_LN3_G];
    lb.add = E.dxin; lb.add_slot_stride = E.Td(); lb.add_slots = loc;
    lb.out_f32 = E.dxin; lb.of_slot_stride = E.Td(); lb.of_slots = loc;
    lb.C = IN; lb.out_op = E.ds; lb.oo_slot_stride = E.Td(); lb.oo_slots = loc;
    HIPCHK(launch_ln_bwd(lb, E.bf16, E.st));
  }

  // s = o Wo^T + bo
  if (DT)
    STCHK(linear_param_grads(E, n, E.ds, E.Td(), loc, d, E.c_o, E.Td(), cs, d, false, *DT, MGRIT_P_WO,
                             MGRIT_P_BO, hstep));

  // da = ds Wo
  g = gemm_base(n, T, d, d, E.ds, E.Td(), loc, THT, L.offset[MGRIT_P_WO], -1);
  g.out = E.da; g.out_slot_stride = E.Td(); g.out_slots = loc;
  HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));

  // attention backward
  AttnArgs at;
  memset(&at, 0, sizeof(at));
  at.n_groups = n; at.B = E.md.batch; at.H = E.H; at.dh = E.dh; at.Sq = E.md.seq; at.Sk = E.md.seq;
  at.causal = E.md.arch != MGRIT_ARCH_ENCODER;
  at.q = E.c_qkv; at.k = (char*)E.c_qkv + (size_t)d * esz; at.v = (char*)E.c_qkv + (size_t)2 * d * esz;
  at.q_row_stride = at.k_row_stride = at.v_row_stride = 3 * d;
  at.q_slot_stride = at.k_slot_stride = at.v_slot_stride = (long)T * 3 * d;
  at.q_slots = at.k_slots = cs;
  at.o = E.c_o; at.o_row_stride = d; at.o_slot_stride = E.Td(); at.o_slots = cs;
  at.lse = E.c_lse; at.lse_slot_stride = (long)E.md.batch * E.H * E.md.seq; at.lse_slots = cs;
  at.dO = E.da; at.do_row_stride = d; at.do_slot_stride = E.Td(); at.do_slots = loc;
  at.dq = E.dqkv; at.dk = (char*)E.dqkv + (size_t)d * esz; at.dv = (char*)E.dqkv + (size_t)2 * d * esz;
  at.dqkv_row_stride = 3 * d; at.dqkv_slot_stride = (long)T * 3 * d; at.dqkv_slots = loc;
  at.D = E.Dbuf; at.D_slot_stride = (long)E.md.batch * E.H * E.md.seq; at.D_slots = loc;
  HIPCHK(launch_attn_bwd(at, E.bf16, E.st));

  if (DT) {
    // qkv = LN1(X) Wqkv^T + bqkv
    lf.xp = nullptr;
    lf.gamma_off = L.offset[MGRIT_P_LN1_G]; lf.beta_off = L.offset[MGRIT_P_LN1_B];
    HIPCHK(launch_ln_fwd(lf, E.bf16, E.st));
    STCHK(linear_param_grads(E, n, E.dqkv, (long)T * 3 * d, loc, 3 * d, E.u, E.Td(), loc, d, false, *DT,
                             MGRIT_P_WQKV, MGRIT_P_BQKV, hstep));
  }

  // du1 = dqkv Wqkv               [T,3d] x [3d,d]: transposed Wqkv is [d,3d]
  g = gemm_base(n, T, d, 3 * d, E.dqkv, (long)T * 3 * d, loc, THT, L.offset[MGRIT_P_WQKV], -1);
  g.out = E.du; g.out_slot_stride = E.Td(); g.out_slots = loc;
  HIPCHK(launch_gemm(g, EPI_STORE, E.bf16, E.st));

  if (DT) {
    lp.xp = nullptr;
    lp.gamma_off = E.glay.offset[MGRIT_P_LN1_G]; lp.beta_off = E.glay.offset[MGRIT_P_LN1_B];
    HIPCHK(launch_ln_param_grad(lp, E.gpart, E.bf16, E.st));
  }
  if (gp && !gp->write_state) return MGRIT_OK;           // a pure gradient pass writes no state

  // dX = dX' + LN1^T du1 ;  OUT = c + hstep dX (+ RHS)
  memset(&lb, 0, sizeof(lb));
  lb.n_groups = n; lb.T = T; lb.d = d; lb.eps = E.md.ln_eps;
  lb.dy = E.du; lb.dy_slot_stride = E.Td(); lb.dy_slots = loc;
  lb.xhat = E.c_xh1; lb.xhat_slot_stride = E.Td(); lb.xhat_slots = cs; lb.rstd = E.c_rs1;
  lb.P = TH; lb.gamma_off = L.offset[MGRIT_P_LN1_G];
  lb.add = E.dxin; lb.add_slot_stride = E.Td(); lb.add_slots = loc;
  lb.C = IN; lb.OUT = OUT; lb.RHS = RHS; lb.hstep = hstep; lb.rhs_sign = E.rhs_sign;
  if (sh && sh->out) { lb.out_cast = sh->out; lb.oc_slot_stride = E.Td(); lb.oc_slots = sh->out_slots; }
  HIPCHK(launch_ln_bwd(lb, E.bf16, E.st));
  return MGRIT_OK;
}

// Runs `fn(lane engine, first group, count)` over chunks of a sweep; with a second lane the
// chunks alternate between the two streams.
template <typename F>
int run_chunks(Engine& E, Engine* E2, int G, F fn) {
  const bool two = E2 != nullptr && G >= 2;
  int chunk = E.Gc;
  if (two && (G + 1) / 2 < chunk) chunk = (G + 1) / 2;
  if (!two) {
    for (int c0 = 0; c0 < G; c0 += chunk) STCHK(fn(E, c0, G - c0 < chunk ? G - c0 : chunk));
    return MGRIT_OK;
  }
  AuxStream& a = aux_stream();
  HIPCHK(hipEventRecord(a.fork, E.st));
  HIPCHK(hipStreamWaitEvent(E2->st, a.fork, 0));
  int lane = 0, status = MGRIT_OK;
  for (int c0 = 0; c0 < G && status == MGRIT_OK; c0 += chunk, lane ^= 1)
    status = fn(lane ? *E2 : E, c0, G - c0 < chunk ? G - c0 : chunk);
  // the helper lane is joined back whatever happened, so that a failed call leaves no work behind
  // that the caller's stream does not wait for
  const hipError_t e1 = hipEventRecord(a.join, E2->st);
  const hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(E.st, a.join, 0) : e1;
  STCHK(status);
  HIPCHK(e2);
  return MGRIT_OK;
}

int forward_groups(Engine& E, Engine* E2, int G, Rows IN, Rows OUT, Rows RHS, Params TH, float hstep, int cache,
                   Slots cslots, Rows MEM = NO_ROWS) {
  return run_chunks(E, E2, G, [&](Engine& L, int c0, int n) {
    return forward_chunk(L, n, shift(IN, c0), shift(OUT, c0), shift(RHS, c0), shift(TH, c0), hstep, cache,
                         shift(cslots, c0), shift(MEM, c0));
  });
}

// emit: the steps also write the parameter gradients of their layers (DT, may be null) and the
// memory-gradient terms (dE_all, may be null); the caller guarantees that IN holds final values
int adjoint_groups(Engine& E, Engine* E2, int G, Rows IN, Rows OUT, Rows RHS, Params TH, Params THT, Rows LIN,
                   Slots cs, float hstep, const StackedDec* sd = nullptr, bool emit = false,
                   const Params* DT = nullptr, float* dE_all = nullptr, const CastShadow* sh = nullptr) {
  return run_chunks(E, E2, G, [&](Engine& L, int c0, int n) {
    StackedDec s;
    if (sd) s = shift(*sd, c0);
    CastShadow shc;
    if (sh) shc = shift(*sh, c0);
    Params dt = {nullptr, 0, 0};
    GradPass gp;
    if (emit) {
      if (DT) { dt = shift(*DT, c0); gp.DT = &dt; }
      gp.dE_all = dE_all;
      gp.write_state = true;
    }
    Slots slots = shift(cs, c0);
    gp.dE_slots = slots;
    if (L.recompute) {                    // the internals of this chunk's layers, into the lane's chunk-sized cache
      slots = Slots{0, 1};
      STCHK(forward_chunk(L, n, shift(LIN, c0), NO_ROWS, NO_ROWS, shift(TH, c0), 0.f, 1, slots,
                          sd ? s.MEM : NO_ROWS));
    }
    return adjoint_chunk(L, n, shift(IN, c0), shift(OUT, c0), shift(RHS, c0), shift(TH, c0), shift(THT, c0),
                         shift(LIN, c0), slots, hstep, emit ? &gp : nullptr, sd ? &s : nullptr, sh ? &shc : nullptr);
  });
}

// parameter gradients of G layers: group g has IN = lambda_{n+1}, LIN = Z_n, gradient block DT[g]
int gradient_groups(Engine& E, Engine* E2, int G, Rows IN, Params TH, Params THT, Rows LIN, Slots cs,
                    const Params* DT, float* dE_all, float hstep, const StackedDec* sd = nullptr) {
  return run_chunks(E, E2, G, [&](Engine& L, int c0, int n) {
    Params dt = {nullptr, 0, 0};
    GradPass gp;
    if (DT) { dt = shift(*DT, c0); gp.DT = &dt; }
    gp.dE_all = dE_all;
    StackedDec s;
    if (sd) s = shift(*sd, c0);
    Slots slots = shift(cs, c0);
    gp.dE_slots = slots;
    if (L.recompute) {
      slots = Slots{0, 1};
      STCHK(forward_chunk(L, n, shift(LIN, c0), NO_ROWS, NO_ROWS, shift(TH, c0), 0.f, 1, slots,
                          sd ? s.MEM : NO_ROWS));
    }
    return adjoint_chunk(L, n, shift(IN, c0), NO_ROWS, NO_ROWS, shift(TH, c0), shift(THT, c0), shift(LIN, c0),
                         slots, hstep, &gp, sd ? &s : nullptr);
  });
}

int transpose_blocks(Engine& E, int n, Params TH, Params THT) {
  static const int mats[] = {MGRIT_P_WQKV, MGRIT_P_WO, MGRIT_P_W1, MGRIT_P_W2, MGRIT_P_WQ_C, MGRIT_P_WO_C,
                             MGRIT_P_WKV_C};
  for (int id : mats) {
    if (E.lay.offset[id] < 0) continue;
    HIPCHK(launch_transpose(n, TH, THT, E.lay.offset[id], E.lay.rows[id], E.lay.cols[id], E.lay.elem_bytes[id],
                            E.st));
  }
  return MGRIT_OK;
}

// ---------------------------------------------------------------------------
// MGRIT driver
// ---------------------------------------------------------------------------
struct Driver {
  Engine* E = nullptr;             // null: dry run that only counts evaluations
  Engine* E2 = nullptr;            // second lane, or null
  bool adjoint = false;
  int N = 0, cf = 1, L = 1, relax = MGRIT_RELAX_FCF;
  float h = 0.f;
  // device pointer tables
  void** tabW = nullptr;           // level-0 point m -> state row (forward: m, adjoint: N-m)
  void** tabZ = nullptr;           // adjoint: forward state n (linearisation)
  void** tabTh = nullptr;          // layer n -> parameter block
  void** tabThT = nullptr;         // layer n -> transposed block (adjoint)
  std::vector<void**> tabG;        // level l >= 1: point j -> right-hand side g^l_j
  void** tabR = nullptr;           // k -> scratch state R_k
  double* partial = nullptr;
  int max_partial = 0;
  float* resnorm = nullptr;
  int64_t evals = 0;
  int64_t sweeps = 0;              // batched sweeps enqueued: each depends on the one before it
  // stacked encoder-decoder grid (paper section 3.1, eq. "fp_transformer"): E, E2 are the encoder's
  // engines, Ed, Ed2 the decoder's; layers below n_enc are encoder layers.  A state is the X rows
  // (x_elems floats) followed by the Y rows (y_elems floats).
  Engine* Ed = nullptr;
  Engine* Ed2 = nullptr;
  int n_enc = 0;
  long x_elems = 0, y_elems = 0;
  long state_elems() const { return Ed ? x_elems + y_elems : E->Td(); }

  static int ipow(int b, int e) { int r = 1; while (e-- > 0) r *= b; return r; }
  static Rows part(Rows r, long off) { if (r.tab) r.off += off; return r; }

  // Stacked grid: the groups of a sweep start at increasing (forward) or decreasing (adjoint)
  // layers, so they split into one run of encoder steps and one run of decoder steps.  An
  // encoder step advances the X rows and copies the Y rows (+ right-hand side), a decoder step
  // the other way round, reading the X rows of its input (forward) or of its linearisation
  // state (adjoint) as cross-attention memory.
  int step_stacked(int cnt, int n0, int ns, Rows IN, Rows OUT, Rows RHS, float hstep, bool fill = false) {
    // groups k = 0..cnt-1 act on layer n0 + k*ns
    int n_first = 0;                                 // groups of the first run
    const bool first_is_enc = adjoint ? false : true;
    if (!adjoint) {                                  // ns >= 0: encoder while n0 + k ns < n_enc
      if (n0 >= n_enc) n_first = 0;
      else if (ns <= 0) n_first = cnt;
      else n_first = (n_enc - 1 - n0) / ns + 1;
    } else {                                         // ns <= 0: decoder while n0 + k ns >= n_enc
      if (n0 < n_enc) n_first = 0;
      else if (ns >= 0) n_first = cnt;
      else n_first = (n0 - n_enc) / (-ns) + 1;
    }
    if (n_first > cnt) n_first = cnt;
    // engines of this call: both lanes with fork / join, or one lane alone (see `only`)
    const bool helper = only != nullptr && only == E2;
    Engine& Le = helper ? *E2 : *E;
    Engine& Ld = helper ? *Ed2 : *Ed;
    Engine* Le2 = only ? nullptr : E2;
    Engine* Ld2 = only ? nullptr : Ed2;
    for (int run = 0; run < 2; ++run) {
      const int c0 = run == 0 ? 0 : n_first, n = run == 0 ? n_first : cnt - n_first;
      if (n <= 0) continue;
      const bool enc = (run == 0) == first_is_enc;
      const int nl = n0 + c0 * ns;
      const Rows in = shift(IN, c0), out = shift(OUT, c0), rhs = shift(RHS, c0);
      const Rows inx = in, outx = out, rhsx = rhs;
      const Rows iny = part(in, x_elems), outy = part(out, x_elems), rhsy = part(rhs, x_elems);
      Params TH = {(const void* const*)tabTh, nl, ns};
      if (!adjoint) {
        // fill: these level-0 steps read final states and leave their layers' cache entries (see fill_cache)
        if (enc) {
          STCHK(forward_groups(Le, Le2, n, inx, outx, rhsx, TH, hstep, fill ? 2 : 0, fill ? Slots{nl, ns} : Slots{0, 0}));
          HIPCHK(launch_add_rows(n, y_elems, iny, rhsy, outy, Le.st));
        } else {
          STCHK(forward_groups(Ld, Ld2, n, iny, outy, rhsy, TH, hstep, fill ? 2 : 0,
                               fill ? Slots{nl - n_enc, ns} : Slots{0, 0}, inx));
          HIPCHK(launch_add_rows(n, x_elems, inx, rhsx, outx, Le.st));
        }
        continue;
      }
      Params THT = {(const void* const*)tabThT, nl, ns};
      Rows LIN = {(const void* const*)tabZ, nl, ns};
      const bool emit = emit_now && tabDT != nullptr;         // see step(): these steps read final values
      const Params DT = {(const void* const*)tabDT, nl, ns};
      if (emit) emitted = true;
      if (enc) {
        STCHK(adjoint_groups(Le, Le2, n, inx, outx, rhsx, TH, THT, LIN, Slots{nl, ns}, hstep, nullptr, emit, &DT));
        HIPCHK(launch_add_rows(n, y_elems, iny, rhsy, outy, Le.st));
      } else {
        StackedDec sd = {LIN, inx, outx, rhsx};
        STCHK(adjoint_groups(Ld, Ld2, n, iny, outy, rhsy, TH, THT, part(LIN, x_elems), Slots{nl - n_enc, ns}, hstep,
                             &sd, emit, &DT));
      }
    }
    return MGRIT_OK;
  }

  Engine* only = nullptr;          // when set, step() enqueues on this engine's stream alone (no fork / join)
  // Parameter gradients (adjoint only): dtheta_n = h (dF/dtheta_n (Z_n))^T lambda_{n+1} needs the final
  // lambda_{n+1}, which is exactly the input of the level-0 steps of the last cycle's closing
  // F-relaxation (and of every step of a serial run): those steps emit their layer's gradients on
  // the way (emit_final), the remaining N / cf layers get a pass of their own afterwards.
  void** tabDT = nullptr;          // layer n -> gradient block, or null
  float* dE_all = nullptr;         // per-layer memory-gradient terms, or null
  bool want_grads = false, last_cycle = false, emit_now = false, emitted = false;
  // Forward solve on behalf of an adjoint that follows: the level-0 steps of the last cycle's closing
  // F-relaxation (of every step in a serial run) read final states, so they leave their layers'
  // entries of the adjoint's linearisation cache on the way (the engines' cache pointers then point
  // into the adjoint's workspace).  The layers n = cf-1, 2cf-1, .. are left to the adjoint.
  bool fill_cache = false, cache_now = false;
  // adjoint: operand-type copy of every grid point's state, [N+1][T,d], and which of them hold the point's
  // current value (host-side bookkeeping at enqueue time: grid points are written by steps only)
  void* shadow = nullptr;
  std::vector<char> shadow_valid;

  // cnt steps of level `lvl`, group k starting at point j = j0 + k*js
  int step(int lvl, int j0, int js, int cnt, Rows OUT, Rows RHS) {
    evals += cnt;
    ++sweeps;
    if (!E) return MGRIT_OK;
    Engine& L1 = only ? *only : *E;
    Engine* L2 = only ? nullptr : E2;
    const int s = ipow(cf, lvl);
    const float hstep = (float)((double)s * (double)h);
    Rows IN = {(const void* const*)tabW, j0 * s, js * s};
    if (Ed) {
      if (!adjoint) return step_stacked(cnt, j0 * s, js * s, IN, OUT, RHS, hstep, cache_now && lvl == 0);
      const bool keep = emit_now;
      emit_now = keep && lvl == 0;
      const int st = step_stacked(cnt, N - (j0 + 1) * s, -js * s, IN, OUT, RHS, hstep);
      emit_now = keep;
      return st;
    }
    if (!adjoint) {
      Params TH = {(const void* const*)tabTh, j0 * s, js * s};
      if (cache_now && lvl == 0) return forward_groups(L1, L2, cnt, IN, OUT, RHS, TH, hstep, 2, Slots{j0, js});
      return forward_groups(L1, L2, cnt, IN, OUT, RHS, TH, hstep, 0, Slots{0, 0});
    }
    const int n0 = N - (j0 + 1) * s, ns = -js * s;       // layer the coarse step lands on
    Params TH = {(const void* const*)tabTh, n0, ns};
    Params THT = {(const void* const*)tabThT, n0, ns};
    Rows LIN = {(const void* const*)tabZ, n0, ns};
    // operand-type copies of the states (see CastShadow): the inputs' copies exist if every input point was
    // written by a step of this call; the outputs' copies are left when the outputs are grid points
    CastShadow sh;
    const bool out_is_point = OUT.tab == (const void* const*)tabW;
    if (shadow) {
      sh.in = shadow; sh.in_slots = Slots{j0 * s, js * s}; sh.valid = shadow_valid.data();
      if (out_is_point) { sh.out = shadow; sh.out_slots = Slots{OUT.i0, OUT.is}; }
    }
    int st;
    if (emit_now && lvl == 0) {
      emitted = true;
      const Params DT = {(const void* const*)tabDT, n0, ns};
      st = adjoint_groups(L1, L2, cnt, IN, OUT, RHS, TH, THT, LIN, Slots{n0, ns}, hstep, nullptr, true,
                          tabDT ? &DT : nullptr, dE_all, shadow ? &sh : nullptr);
    } else {
      st = adjoint_groups(L1, L2, cnt, IN, OUT, RHS, TH, THT, LIN, Slots{n0, ns}, hstep, nullptr, false, nullptr,
                          nullptr, shadow ? &sh : nullptr);
    }
    if (shadow && out_is_point && st == MGRIT_OK)
      for (int k = 0; k < cnt; ++k) shadow_valid[(size_t)OUT.i0 + (size_t)k * OUT.is] = 1;
    return st;
  }

  // g'_k = R_k - Phi'(w_{(k-1) cf}) for the groups g0 .. g0+n-1 of level lvl+1 (Gn, R already shifted to g0).
  // The step that evaluates Phi' takes R as its right-hand side with the sign of the step reversed, which
  // gives the same rounded values as the step followed by a subtraction.  The stacked grid copies the half
  // of the state a step leaves alone, so there the subtraction stays a kernel of its own.
  int coarse_rhs(int lvl, int g0, int n, Rows R, Rows Gn, Engine* lane) {
    if (Ed || !E) {
      STCHK(step(lvl + 1, g0, 1, n, Gn, NO_ROWS));
      if (E) HIPCHK(launch_sub_rows(n, state_elems(), R, Gn, Gn, lane ? lane->st : E->st));
      return MGRIT_OK;
    }
    E->rhs_sign = -1.f;
    if (E2) E2->rhs_sign = -1.f;
    const int st = step(lvl + 1, g0, 1, n, Gn, R);
    E->rhs_sign = 1.f;
    if (E2) E2->rhs_sign = 1.f;
    return st;
  }

  // The coarse right-hand sides, the serial solve on the coarsest level (level lvl + 1, M steps) and
  // the F-relaxation of level lvl that follows it, overlapped on the two lanes.  The coarse steps
  // are single groups, which leave much of the chip idle, and they form MGRIT's serial chain:
  //  * the right-hand sides g'_k = R_k - Phi'(w_{(k-1) cf}) are formed chunk by chunk, the first
  //    chunk on the caller's stream, the others on the helper lane; coarse step j reads g'_j and
  //    overwrites C-point j, which the right-hand side of group j still has to read, so it waits
  //    (by event) for the chunk that holds group j and no more;
  //  * interval k of level lvl may relax as soon as its C-point v_k is final, i.e. after coarse
  //    step k: after every `chunk` steps an event hands the finished intervals to the helper lane,
  //    which runs their cf-1 dependent F-steps meanwhile; the last chunk relaxes on this stream.
  // Same kernels on the same data as the sequential order: results are identical.
  int coarse_solve_with_relaxation(int lvl, int M, Rows R, Rows Gn) {
    AuxStream& a = aux_stream();
    const int status = coarse_solve_pipeline(lvl, M, R, Gn);
    // join the helper lane whatever happened (see run_chunks)
    only = nullptr;
    emit_now = cache_now = false;
    const hipError_t e1 = hipEventRecord(a.join, E2->st);
    const hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(E->st, a.join, 0) : e1;
    STCHK(status);
    HIPCHK(e2);
    return MGRIT_OK;
  }
  int coarse_solve_pipeline(int lvl, int M, Rows R, Rows Gn) {
    AuxStream& a = aux_stream();
    const int chunk = g_pipe_chunk > 0 && g_pipe_chunk < E2->Gc ? g_pipe_chunk : E2->Gc;
    const int n_chunks = (M + chunk - 1) / chunk;
    constexpr int HALF = PIPE_EVENTS / 2;                // events 0..HALF-1: right-hand sides; the others: hand-overs
    auto rhs_chunk = [&](Engine* lane, int g0, int n) -> int {
      only = lane;
      const int st = coarse_rhs(lvl, g0, n, shift(R, g0), shift(Gn, g0), lane);
      only = nullptr;
      return st;
    };
    const bool split_rhs = n_chunks >= 2 && n_chunks <= HALF;
    if (!split_rhs) {
      STCHK(coarse_rhs(lvl, 0, M, R, Gn, nullptr));
    } else {
      // the helper lane starts from everything enqueued so far (relaxation, residual)
      HIPCHK(hipEventRecord(a.fork, E->st));
      HIPCHK(hipStreamWaitEvent(E2->st, a.fork, 0));
      STCHK(rhs_chunk(E, 0, chunk));
      for (int c = 1; c < n_chunks; ++c) {
        const int g0 = c * chunk;
        STCHK(rhs_chunk(E2, g0, M - g0 < chunk ? M - g0 : chunk));
        HIPCHK(hipEventRecord(a.pipe[c], E2->st));
      }
    }
    auto relax = [&](Engine* lane, int ka, int kb) -> int {   // F-relaxation of intervals ka .. kb-1 on one lane
      only = lane;
      emit_now = want_grads && last_cycle && lvl == 0;
      cache_now = fill_cache && last_cycle && lvl == 0;
      int st = MGRIT_OK;
      for (int i = 0; i + 1 < cf && st == MGRIT_OK; ++i)
        st = step(lvl, ka * cf + i, cf, kb - ka, W(lvl, ka * cf + i + 1, cf), Gr(lvl, ka * cf + i + 1, cf));
      only = nullptr;
      emit_now = cache_now = false;
      return st;
    };
    int k0 = 0, ev = 0;
    for (int j = 0; j <= M; ++j) {                       // j coarse steps done: v_0 .. v_j are final
      if (j >= 1) {
        const int need = j < M ? j : M - 1;              // groups 0 .. need must have read their C-point
        if (split_rhs && need % chunk == 0 && need >= chunk)
          HIPCHK(hipStreamWaitEvent(E->st, a.pipe[need / chunk], 0));
        STCHK(step(lvl + 1, j - 1, 1, 1, W(lvl + 1, j, 1), Gr(lvl + 1, j, 1)));
      }
      const int k1 = j + 1;                              // intervals k0 .. k1-1 can relax now
      if (k1 >= M || k1 % chunk != 0) continue;          // the last chunk stays on this lane, see below
      hipEvent_t e = a.pipe[HALF + ev++ % HALF];
      HIPCHK(hipEventRecord(e, E->st));
      HIPCHK(hipStreamWaitEvent(E2->st, e, 0));
      STCHK(relax(E2, k0, k1));
      k0 = k1;
    }
    // the helper lane still has its chunks to finish: the remaining intervals relax on this lane
    return relax(E, k0, M);
  }

  Rows W(int lvl, int j0, int js) const {
    const int s = ipow(cf, lvl);
    return Rows{(const void* const*)tabW, j0 * s, js * s};
  }
  Rows Gr(int lvl, int j0, int js) const {
    if (lvl == 0) return NO_ROWS;
    return Rows{(const void* const*)tabG[lvl], j0, js};
  }

  int f_relax(int lvl, int M) {
    for (int i = 0; i + 1 < cf; ++i) STCHK(step(lvl, i, cf, M, W(lvl, i + 1, cf), Gr(lvl, i + 1, cf)));
    return MGRIT_OK;
  }

  int vcycle(int lvl, int iter, bool skip_first_f) {
    const int Nl = N / ipow(cf, lvl);
    if (lvl == L - 1) {
      for (int j = 1; j <= Nl; ++j) STCHK(step(lvl, j - 1, 1, 1, W(lvl, j, 1), Gr(lvl, j, 1)));
      return MGRIT_OK;
    }
    const int M = Nl / cf;
    if (!skip_first_f) STCHK(f_relax(lvl, M));
    if (relax == MGRIT_RELAX_FCF) {
      STCHK(step(lvl, cf - 1, cf, M, W(lvl, cf, cf), Gr(lvl, cf, cf)));
      STCHK(f_relax(lvl, M));
    }
    // R_k = Phi(w_{k cf - 1}) + g_{k cf}
    Rows R = {(const void* const*)tabR, 0, 1};
    STCHK(step(lvl, cf - 1, cf, M, R, Gr(lvl, cf, cf)));
    if (E && lvl == 0 && resnorm)
      HIPCHK(launch_resnorm(M, state_elems(), R, W(lvl, cf, cf), partial, max_partial, resnorm + iter, E->st));
    // g'_k = R_k - Phi'(w_{(k-1) cf}),  k = 1..M
    Rows Gn = {(const void* const*)(E ? tabG[lvl + 1] : nullptr), 1, 1};
    if (E && E2 && g_pipeline && lvl + 1 == L - 1 && M >= 2 && cf >= 2)
      return coarse_solve_with_relaxation(lvl, M, R, Gn);
    STCHK(coarse_rhs(lvl, 0, M, R, Gn, nullptr));
    STCHK(vcycle(lvl + 1, iter, false));
    emit_now = want_grads && last_cycle && lvl == 0;
    cache_now = fill_cache && last_cycle && lvl == 0;
    const int st = f_relax(lvl, M);
    emit_now = cache_now = false;
    return st;
  }

  int run(int iters) {
    if (L == 1 || cf == 1) {
      emit_now = want_grads;
      cache_now = fill_cache;
      int st = MGRIT_OK;
      for (int n = 0; n < N && st == MGRIT_OK; ++n) st = step(0, n, 1, 1, W(0, n + 1, 1), NO_ROWS);
      emit_now = cache_now = false;
      return st;
    }
    for (int it = 0; it < iters; ++it) {
      last_cycle = it == iters - 1;
      STCHK(vcycle(0, it, it > 0));
    }
    return MGRIT_OK;
  }
  bool serial() const { return L == 1 || cf == 1; }
};

struct Plan {                       // workspace of mgrit_forward / mgrit_adjoint
  Engine E, E2;
  bool two_lanes = false;
  Driver D;
  void* thT_blocks = nullptr;
  void** tabDT = nullptr;           // layer n -> gradient block (adjoint with parameter gradients)
  float* dE_all = nullptr;          // cross-attention decoder: per-layer terms of the memory gradient
  size_t bytes = 0;
};

// mode: 0 forward, 1 adjoint, 2 adjoint followed by the parameter-gradient pass
// share_ws, share_mode: a forward plan whose closing relaxation fills the linearisation cache of the
// adjoint plan (mode 1 or 2) that will be laid out in share_ws: the cache is the first thing an adjoint
// plan carves, so carving it again from the same base gives the same addresses.
int make_plan(Plan& P, const mgrit_model_desc* md, const mgrit_opts* op, int mode, void* ws, hipStream_t st,
              void* share_ws = nullptr, int share_mode = 0) {
  const bool adjoint = mode != 0;
  Bump b(ws);
  Engine& E = P.E;
  E.init(md, st);
  const int N = op->N;
  const bool serial = serial_run(op);
  const int M0 = serial ? 1 : N / op->cf;
  int gc = max_groups(md, M0);
  const int widest = adjoint ? (N > M0 ? N : M0) : M0;      // the cache pass batches over all N layers
  if (gc > widest) gc = widest;
  E.keep_z = mode == 2;
  E.recompute = adjoint && !g_adjoint_cache;
  if (adjoint) E.carve_adjoint(b, gc, N); else E.carve_forward(b, gc);
  if (!adjoint && share_ws) {
    Bump shared(share_ws);
    E.keep_z = share_mode == 2;
    E.carve_cache(shared, N);
    P.D.fill_cache = true;
  }
  P.two_lanes = widest >= 2 && make_lane(P.E2, E, b, adjoint, ws == nullptr);
  Driver& D = P.D;
  D.E = &E; D.E2 = P.two_lanes ? &P.E2 : nullptr; D.adjoint = adjoint; D.N = N; D.cf = op->cf; D.L = serial ? 1 : op->levels; D.relax = op->relax;
  D.h = op->h;
  D.tabW = b.take<void*>(N + 1);
  D.tabTh = b.take<void*>(N);
  if (adjoint) {
    D.tabZ = b.take<void*>(N + 1);
    D.tabThT = b.take<void*>(N);
    P.thT_blocks = b.take_bytes((size_t)N * E.lay.block_bytes);
  }
  if (mode == 2) {
    P.tabDT = b.take<void*>(N);
    if (md->arch == MGRIT_ARCH_CROSS) P.dE_all = b.take<float>((size_t)N * E.Tm * E.d);
    for (Engine* L : {&E, P.two_lanes ? &P.E2 : nullptr}) {
      if (!L) continue;
      L->carve_grad_work(b);
      if (ws && launch_fill_table(L->tabTB, static_cast<char*>(L->tB), L->tB_stride() * (long)L->esz, L->Gc, st) !=
                    hipSuccess)
        return MGRIT_HIP_ERROR;
    }
  }
  if (adjoint) {
    D.shadow = b.take_bytes((size_t)(N + 1) * E.T * E.d * E.esz);
    D.shadow_valid.assign((size_t)N + 1, 0);
  }
  D.tabG.assign(D.L, nullptr);
  if (!serial) {
    D.tabR = b.take<void*>(M0);
    D.max_partial = M0 * resnorm_partials_per_group();
    D.partial = b.take<double>(D.max_partial);
    const size_t state = (size_t)E.T * E.d * sizeof(float);
    char* Rbuf = static_cast<char*>(b.take_bytes(M0 * state));
    std::vector<char*> Gbuf(D.L, nullptr);
    for (int l = 1; l < D.L; ++l) {
      const int Nl = N / Driver::ipow(op->cf, l);
      D.tabG[l] = b.take<void*>(Nl + 1);
      Gbuf[l] = static_cast<char*>(b.take_bytes((size_t)(Nl + 1) * state));
    }
    if (ws) {
      if (launch_fill_table(D.tabR, Rbuf, (long)state, M0, st) != hipSuccess) return MGRIT_HIP_ERROR;
      for (int l = 1; l < D.L; ++l) {
        const int Nl = N / Driver::ipow(op->cf, l);
        if (launch_fill_table(D.tabG[l], Gbuf[l], (long)state, Nl + 1, st) != hipSuccess) return MGRIT_HIP_ERROR;
      }
    }
  }
  P.bytes = (b.off + 255) / 256 * 256;
  return MGRIT_OK;
}

int check_ptr_array(const void* const* a, int n) {
  if (!a) return MGRIT_INVALID_ARG;
  for (int i = 0; i < n; ++i) if (!a[i]) return MGRIT_INVALID_ARG;
  return MGRIT_OK;
}

// Scratch need of one batched layer step; second_lane: the helper lane's work buffers included
// (when two lanes are switched on and there are at least two groups).
size_t layer_step_bytes(const mgrit_model_desc* desc, int adjoint, int n_groups, bool second_lane) {
  if (validate_desc(desc) != MGRIT_OK || n_groups < 1) return 0;
  Engine E;
  E.init(desc, nullptr);
  Bump b(nullptr);
  int gc = max_groups(desc, n_groups) < n_groups ? max_groups(desc, n_groups) : n_groups;
  Engine E2;
  if (adjoint) {
    E.carve_adjoint(b, gc, n_groups);
    if (second_lane && n_groups >= 2) make_lane(E2, E, b, true, true);
    b.take_bytes((size_t)n_groups * E.lay.block_bytes);
    b.take<void*>((size_t)n_groups * 6);
  } else {
    E.carve_forward(b, gc);
    if (second_lane && n_groups >= 2) make_lane(E2, E, b, false, true);
    b.take<void*>((size_t)n_groups * 4);
  }
  return (b.off + 255) / 256 * 256;
}

// The batched layer step on scratch memory of `workspace_bytes` at `workspace`; second_lane as above
// (false: every launch goes to `stream`, no helper stream or event is touched).
int layer_step_on(const mgrit_model_desc* desc, int adjoint, int n_groups, const void* const* in,
                  void* const* out, const void* const* theta, const void* const* lin_state,
                  const void* const* rhs, const void* memory, float hstep, void* workspace,
                  size_t workspace_bytes, void* stream, bool second_lane) {
  std::lock_guard<std::recursive_mutex> call_lock(g_call_mutex);
  STCHK(validate_desc(desc));
  if (n_groups < 1 || !workspace || !isfinite(hstep)) return MGRIT_INVALID_ARG;
  STCHK(check_ptr_array(in, n_groups));
  STCHK(check_ptr_array((const void* const*)out, n_groups));
  STCHK(check_ptr_array(theta, n_groups));
  if (rhs) STCHK(check_ptr_array(rhs, n_groups));
  if (adjoint) STCHK(check_ptr_array(lin_state, n_groups));
  if (desc->arch == MGRIT_ARCH_CROSS && !memory) return MGRIT_INVALID_ARG;
  const size_t need = layer_step_bytes(desc, adjoint, n_groups, second_lane);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (workspace_bytes < need) return MGRIT_WORKSPACE_TOO_SMALL;
  hipStream_t st = static_cast<hipStream_t>(stream);

  Engine E;
  E.init(desc, st);
  Bump b(workspace);
  const int gc = max_groups(desc, n_groups) < n_groups ? max_groups(desc, n_groups) : n_groups;
  const int G = n_groups;
  Engine E2;
  Engine* L2 = nullptr;
  if (adjoint) {
    E.carve_adjoint(b, gc, G);
    if (second_lane && G >= 2 && make_lane(E2, E, b, true, false)) L2 = &E2;
    char* tblocks = static_cast<char*>(b.take_bytes((size_t)G * E.lay.block_bytes));
    void** tabs = b.take<void*>((size_t)G * 6);
    void **tIn = tabs, **tOut = tabs + G, **tTh = tabs + 2 * G, **tLin = tabs + 3 * G, **tRhs = tabs + 4 * G,
         **tThT = tabs + 5 * G;
    HIPCHK(upload_pointers(tIn, in, G, st));
    HIPCHK(upload_pointers(tOut, (const void* const*)out, G, st));
    HIPCHK(upload_pointers(tTh, theta, G, st));
    HIPCHK(upload_pointers(tLin, lin_state, G, st));
    if (rhs) HIPCHK(upload_pointers(tRhs, rhs, G, st));
    HIPCHK(launch_fill_table(tThT, tblocks, (long)E.lay.block_bytes, G, st));
    Params TH = {(const void* const*)tTh, 0, 1}, THT = {(const void* const*)tThT, 0, 1};
    Rows IN = {(const void* const*)tIn, 0, 1}, OUT = {(const void* const*)tOut, 0, 1};
    Rows LIN = {(const void* const*)tLin, 0, 1};
    Rows RHS = rhs ? Rows{(const void* const*)tRhs, 0, 1} : NO_ROWS;
    STCHK(transpose_blocks(E, G, TH, THT));
    if (desc->arch == MGRIT_ARCH_CROSS)
      HIPCHK(launch_cast_flat(static_cast<const float*>(memory), E.memb, (long)E.Tm * E.d, E.bf16, st));
    STCHK(forward_groups(E, L2, G, LIN, NO_ROWS, NO_ROWS, TH, 0.f, 1, Slots{0, 1}));
    return adjoint_groups(E, L2, G, IN, OUT, RHS, TH, THT, LIN, Slots{0, 1}, hstep);
  }
  E.carve_forward(b, gc);
  if (second_lane && G >= 2 && make_lane(E2, E, b, false, false)) L2 = &E2;
  void** tabs = b.take<void*>((size_t)G * 4);
  void **tIn = tabs, **tOut = tabs + G, **tTh = tabs + 2 * G, **tRhs = tabs + 3 * G;
  HIPCHK(upload_pointers(tIn, in, G, st));
  HIPCHK(upload_pointers(tOut, (const void* const*)out, G, st));
  HIPCHK(upload_pointers(tTh, theta, G, st));
  if (rhs) HIPCHK(upload_pointers(tRhs, rhs, G, st));
  if (desc->arch == MGRIT_ARCH_CROSS)
    HIPCHK(launch_cast_flat(static_cast<const float*>(memory), E.memb, (long)E.Tm * E.d, E.bf16, st));
  Params TH = {(const void* const*)tTh, 0, 1};
  Rows IN = {(const void* const*)tIn, 0, 1}, OUT = {(const void* const*)tOut, 0, 1};
  Rows RHS = rhs ? Rows{(const void* const*)tRhs, 0, 1} : NO_ROWS;
  return forward_groups(E, L2, G, IN, OUT, RHS, TH, hstep, 0, Slots{0, 0});
}

}  // namespace

// Scratch memory of layer_step_batched_static: one array per GPU, part of the loaded code object (the
// runtime places it when the library is loaded on a device; nothing is allocated at call time).
// On the host this name is only a handle for hipGetSymbolAddress: the device address is looked up once
// per device and that pointer, never the name, is what host code passes on.
static __device__ __align__(256) unsigned char scratch[MGRIT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device.
int static_scratch(void** out) {
  int dev = -1;
  HIPCHK(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return MGRIT_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return MGRIT_HIP_ERROR;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MGRIT_OK;
}
}  // namespace

// ---------------------------------------------------------------------------
// exported functions
// ---------------------------------------------------------------------------
extern "C" {

int mgrit_theta_layout(const mgrit_model_desc* desc, mgrit_theta_layout_t* out) {
  if (!out) return MGRIT_INVALID_ARG;
  int s = validate_desc(desc);
  if (s != MGRIT_OK) return s;
  return compute_layout(desc, out);
}

size_t mgrit_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts, int adjoint) {
  if (validate_desc(desc) != MGRIT_OK || validate_opts(opts) != MGRIT_OK) return 0;
  if (adjoint < 0 || adjoint > 2) return 0;
  Plan P;
  if (make_plan(P, desc, opts, adjoint, nullptr, nullptr) != MGRIT_OK) return 0;
  return P.bytes;
}

size_t mgrit_layer_step_workspace_bytes(const mgrit_model_desc* desc, int adjoint, int n_groups) {
  return layer_step_bytes(desc, adjoint, n_groups, true);
}

int64_t mgrit_step_evaluations(const mgrit_opts* opts) {
  if (validate_opts(opts) != MGRIT_OK) return -1;
  Driver D;
  D.N = opts->N; D.cf = opts->cf; D.L = serial_run(opts) ? 1 : opts->levels; D.relax = opts->relax;
  D.tabG.assign(D.L, nullptr);
  D.run(opts->iters);
  return D.evals;
}

int64_t mgrit_step_depth(const mgrit_opts* opts) {
  if (validate_opts(opts) != MGRIT_OK) return -1;
  Driver D;
  D.N = opts->N; D.cf = opts->cf; D.L = serial_run(opts) ? 1 : opts->levels; D.relax = opts->relax;
  D.tabG.assign(D.L, nullptr);
  D.run(opts->iters);
  return D.sweeps;
}

}  // extern "C"

namespace {
// share_ws != null: the forward solve also fills the linearisation cache of the adjoint workspace share_ws
int forward_impl(const mgrit_model_desc* desc, const mgrit_opts* opts, const void* Z0,
                 const void* const* theta, const void* memory, void* Z_all, float* resnorm, void* workspace,
                 size_t workspace_bytes, void* share_ws, size_t share_bytes, int share_mode, void* stream) {
  std::lock_guard<std::recursive_mutex> call_lock(g_call_mutex);
  STCHK(validate_desc(desc));
  STCHK(validate_opts(opts));
  if (!Z0 || !Z_all || !workspace) return MGRIT_INVALID_ARG;
  STCHK(check_ptr_array(theta, opts->N));
  if (desc->arch == MGRIT_ARCH_CROSS && !memory) return MGRIT_INVALID_ARG;
  const size_t need = mgrit_workspace_bytes(desc, opts, 0);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (workspace_bytes < need) return MGRIT_WORKSPACE_TOO_SMALL;
  if (share_ws) {
    if (!g_adjoint_cache) return MGRIT_INVALID_ARG;       // there is no N-layer cache to fill
    const size_t need_adj = mgrit_workspace_bytes(desc, opts, share_mode);
    if (need_adj == 0) return MGRIT_INVALID_ARG;
    if (share_bytes < need_adj) return MGRIT_WORKSPACE_TOO_SMALL;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);

  Plan P;
  STCHK(make_plan(P, desc, opts, 0, workspace, st, share_ws, share_mode));
  Engine& E = P.E;
  Driver& D = P.D;
  const int N = opts->N;
  const size_t state = (size_t)E.T * E.d * sizeof(float);
  HIPCHK(launch_fill_table(D.tabW, static_cast<char*>(Z_all), (long)state, N + 1, st));
  HIPCHK(upload_pointers(D.tabTh, theta, N, st));
  if (desc->arch == MGRIT_ARCH_CROSS)
    HIPCHK(launch_cast_flat(static_cast<const float*>(memory), E.memb, (long)E.Tm * E.d, E.bf16, st));
  // initial values (Z0 may be row 0 of Z_all itself)
  if (Z0 != Z_all) HIPCHK(hipMemcpyAsync(Z_all, Z0, state, hipMemcpyDeviceToDevice, st));
  if (!serial_run(opts) && opts->init_guess == 0) {
    for (int k = 1; k <= N / opts->cf; ++k)
      HIPCHK(hipMemcpyAsync(static_cast<char*>(Z_all) + (size_t)k * opts->cf * state, Z0, state,
                            hipMemcpyDeviceToDevice, st));
  }
  D.resnorm = resnorm;
  return D.run(opts->iters);
}

// prefilled: the cache already holds the entries that a forward solve with share_ws = workspace leaves
int adjoint_impl(const mgrit_model_desc* desc, const mgrit_opts* opts, const void* Z_all,
                 const void* const* theta, const void* memory, const void* lambda_N, void* lambda_all,
                 void* dmemory, void* const* dtheta, float* resnorm, void* workspace, size_t workspace_bytes,
                 bool prefilled, void* stream) {
  std::lock_guard<std::recursive_mutex> call_lock(g_call_mutex);
  if (prefilled && !g_adjoint_cache) return MGRIT_INVALID_ARG;
  STCHK(validate_desc(desc));
  STCHK(validate_opts(opts));
  if (dmemory && desc->arch != MGRIT_ARCH_CROSS) return MGRIT_INVALID_ARG;
  if (desc->arch == MGRIT_ARCH_CROSS && !memory) return MGRIT_INVALID_ARG;
  if (!Z_all || !lambda_N || !lambda_all || !workspace) return MGRIT_INVALID_ARG;
  STCHK(check_ptr_array(theta, opts->N));
  if (dtheta) STCHK(check_ptr_array((const void* const*)dtheta, opts->N));
  const int mode = (dtheta || dmemory) ? 2 : 1;
  const size_t need = mgrit_workspace_bytes(desc, opts, mode);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (workspace_bytes < need) return MGRIT_WORKSPACE_TOO_SMALL;
  hipStream_t st = static_cast<hipStream_t>(stream);

  Plan P;
  STCHK(make_plan(P, desc, opts, mode, workspace, st));
  Engine& E = P.E;
  Driver& D = P.D;
  const int N = opts->N;
  const size_t state = (size_t)E.T * E.d * sizeof(float);
  // reversed index: point m lives in row N-m
  HIPCHK(launch_fill_table(D.tabW, static_cast<char*>(lambda_all) + (size_t)N * state, -(long)state, N + 1, st));
  HIPCHK(launch_fill_table(D.tabZ, static_cast<char*>(const_cast<void*>(Z_all)), (long)state, N + 1, st));
  HIPCHK(upload_pointers(D.tabTh, theta, N, st));
  HIPCHK(launch_fill_table(D.tabThT, static_cast<char*>(P.thT_blocks), (long)E.lay.block_bytes, N, st));
  Params TH = {(const void* const*)D.tabTh, 0, 1};
  Params THT = {(const void* const*)D.tabThT, 0, 1};
  if (desc->arch == MGRIT_ARCH_CROSS)
    HIPCHK(launch_cast_flat(static_cast<const float*>(memory), E.memb, (long)E.Tm * E.d, E.bf16, st));
  // linearisation cache for all N layers, batched over layers (unless every chunk recomputes its own)
  Rows Zrows = {(const void* const*)D.tabZ, 0, 1};
  if (prefilled && D.E2 && !serial_run(opts)) {
    // The forward solve's closing relaxation has left every layer it stepped through: all but the last
    // layer of each interval (n = cf-1, 2cf-1, ..).  That short pass does not touch the transposed weights,
    // so it runs on this lane while the helper lane transposes them (bandwidth-bound, a lane of its own).
    const int cf = opts->cf;
    AuxStream& a = aux_stream();
    HIPCHK(hipEventRecord(a.fork, st));
    HIPCHK(hipStreamWaitEvent(D.E2->st, a.fork, 0));
    int status = transpose_blocks(*D.E2, N, TH, THT);
    if (status == MGRIT_OK)
      status = forward_groups(E, nullptr, N / cf, Rows{(const void* const*)D.tabZ, cf - 1, cf}, NO_ROWS, NO_ROWS,
                              Params{(const void* const*)D.tabTh, cf - 1, cf}, 0.f, 1, Slots{cf - 1, cf});
    // the helper lane is joined back whatever happened
    const hipError_t e1 = hipEventRecord(a.join, D.E2->st);
    const hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(st, a.join, 0) : e1;
    STCHK(status);
    HIPCHK(e2);
  } else {
    STCHK(transpose_blocks(E, N, TH, THT));
    if (prefilled) {
      // a serial run's forward solve has left all layers; with one lane the few missing ones follow here
      const int cf = opts->cf;
      if (!serial_run(opts))
        STCHK(forward_groups(E, D.E2, N / cf, Rows{(const void* const*)D.tabZ, cf - 1, cf}, NO_ROWS, NO_ROWS,
                             Params{(const void* const*)D.tabTh, cf - 1, cf}, 0.f, 1, Slots{cf - 1, cf}));
    } else if (!E.recompute) {
      STCHK(forward_groups(E, D.E2, N, Zrows, NO_ROWS, NO_ROWS, TH, 0.f, 1, Slots{0, 1}));
    }
  }
  // initial values
  if (lambda_N != static_cast<char*>(lambda_all) + (size_t)N * state)     // may be row N of lambda_all itself
    HIPCHK(hipMemcpyAsync(static_cast<char*>(lambda_all) + (size_t)N * state, lambda_N, state,
                          hipMemcpyDeviceToDevice, st));
  if (!serial_run(opts) && opts->init_guess == 0) {
    for (int k = 1; k <= N / opts->cf; ++k)
      HIPCHK(hipMemcpyAsync(static_cast<char*>(lambda_all) + (size_t)(N - k * opts->cf) * state, lambda_N, state,
                            hipMemcpyDeviceToDevice, st));
  }
  if (D.shadow) {
    // operand-type copies of the initial values: point 0 (lambda_N) and the C-points that were set to it
    const Rows first = {(const void* const*)D.tabW, 0, 1};
    HIPCHK(launch_cast_rows(1, E.Td(), first, D.shadow, E.Td(), Slots{0, 1}, E.bf16, st));
    D.shadow_valid[0] = 1;
    if (!serial_run(opts) && opts->init_guess == 0) {
      const size_t sbytes = (size_t)E.Td() * E.esz;
      for (int k = 1; k <= N / opts->cf; ++k) {
        HIPCHK(hipMemcpyAsync(static_cast<char*>(D.shadow) + (size_t)k * opts->cf * sbytes, D.shadow, sbytes,
                              hipMemcpyDeviceToDevice, st));
        D.shadow_valid[(size_t)k * opts->cf] = 1;
      }
    }
  }
  D.resnorm = resnorm;
  if (dtheta) HIPCHK(upload_pointers(P.tabDT, (const void* const*)dtheta, N, st));
  D.tabDT = dtheta ? P.tabDT : nullptr;
  D.dE_all = dmemory ? P.dE_all : nullptr;
  D.want_grads = dtheta || dmemory;
  STCHK(D.run(opts->iters));
  if (dtheta || dmemory) {
    // Layer n takes lambda_{n+1} (point N-1-n of the reversed grid).  The closing F-relaxation (a serial
    // run: every step) has already emitted the layers whose lambda_{n+1} it read; one batched pass covers
    // the others: with emission the layers n = 0, cf, 2 cf, .. (lambda_{n+1} is the last F-point of an
    // interval), otherwise all of them.
    const bool emitted = D.emitted;
    const int stride = emitted ? opts->cf : 1;
    const int count = emitted ? (D.serial() ? 0 : N / opts->cf) : N;
    Rows LamNext = {(const void* const*)D.tabW, N - 1, -stride};
    Params DT = {(const void* const*)P.tabDT, 0, stride};
    const Params THs = {(const void* const*)D.tabTh, 0, stride}, THTs = {(const void* const*)D.tabThT, 0, stride};
    const Rows Zs = {(const void* const*)D.tabZ, 0, stride};
    if (count > 0)
      STCHK(gradient_groups(E, D.E2, count, LamNext, THs, THTs, Zs, Slots{0, stride}, dtheta ? &DT : nullptr,
                            dmemory ? P.dE_all : nullptr, opts->h));
    // dL/dE = sum over layers of the per-layer terms, in layer order
    if (dmemory)
      HIPCHK(launch_sum_slots(P.dE_all, N, (long)E.Tm * E.d, static_cast<float*>(dmemory), 1.0f, st));
  }
  return MGRIT_OK;
}
}  // namespace

extern "C" {

int mgrit_forward(const mgrit_model_desc* desc, const mgrit_opts* opts, const void* Z0,
                  const void* const* theta, const void* memory, void* Z_all, float* resnorm, void* workspace,
                  size_t workspace_bytes, void* stream) {
  return forward_impl(desc, opts, Z0, theta, memory, Z_all, resnorm, workspace, workspace_bytes, nullptr, 0, 0,
                      stream);
}

int mgrit_forward_linearising(const mgrit_model_desc* desc, const mgrit_opts* opts, const void* Z0,
                              const void* const* theta, const void* memory, void* Z_all, float* resnorm,
                              void* workspace, size_t workspace_bytes, void* adjoint_workspace,
                              size_t adjoint_workspace_bytes, int with_gradients, void* stream) {
  if (!adjoint_workspace) return MGRIT_INVALID_ARG;
  return forward_impl(desc, opts, Z0, theta, memory, Z_all, resnorm, workspace, workspace_bytes, adjoint_workspace,
                      adjoint_workspace_bytes, with_gradients ? 2 : 1, stream);
}

int mgrit_adjoint(const mgrit_model_desc* desc, const mgrit_opts* opts, const void* Z_all,
                  const void* const* theta, const void* memory, const void* lambda_N, void* lambda_all,
                  void* dmemory, void* const* dtheta, float* resnorm, void* workspace, size_t workspace_bytes,
                  void* stream) {
  return adjoint_impl(desc, opts, Z_all, theta, memory, lambda_N, lambda_all, dmemory, dtheta, resnorm, workspace,
                      workspace_bytes, false, stream);
}

int mgrit_adjoint_linearised(const mgrit_model_desc* desc, const mgrit_opts* opts, const void* Z_all,
                             const void* const* theta, const void* memory, const void* lambda_N,
                             void* lambda_all, void* dmemory, void* const* dtheta, float* resnorm,
                             void* workspace, size_t workspace_bytes, void* stream) {
  return adjoint_impl(desc, opts, Z_all, theta, memory, lambda_N, lambda_all, dmemory, dtheta, resnorm, workspace,
                      workspace_bytes, true, stream);
}

// ---- stacked encoder-decoder grid (paper section 3.1, eq. "fp_transformer") --------------------
namespace {
struct StackedPlan {
  Engine Ee, Ee2, Ed, Ed2;          // encoder / decoder engines of the two lanes
  bool two_lanes = false;
  Driver D;
  void* thT_blocks = nullptr;
  void** tabDT = nullptr;
  size_t enc_block = 0, dec_block = 0;
  size_t bytes = 0;
};

mgrit_model_desc encoder_of(const mgrit_model_desc* dec) {
  mgrit_model_desc m = *dec;
  m.arch = MGRIT_ARCH_ENCODER;
  m.seq = dec->mem_seq;
  m.mem_seq = 0;
  return m;
}

int validate_stacked(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc) {
  STCHK(validate_desc(desc));
  STCHK(validate_opts(opts));
  if (desc->arch != MGRIT_ARCH_CROSS) return MGRIT_INVALID_ARG;
  const mgrit_model_desc me = encoder_of(desc);
  STCHK(validate_desc(&me));
  if (n_enc < 1 || n_enc >= opts->N) return MGRIT_INVALID_ARG;
  return MGRIT_OK;
}

// mode: 0 forward, 1 adjoint, 2 adjoint followed by the parameter-gradient pass
// share_ws, share_mode: as in make_plan (a forward plan that fills the caches of the adjoint plan in share_ws)
int make_stacked_plan(StackedPlan& P, const mgrit_model_desc* md, const mgrit_opts* op, int n_enc, int mode,
                      void* ws, hipStream_t st, void* share_ws = nullptr, int share_mode = 0) {
  const bool adjoint = mode != 0;
  Bump b(ws);
  const mgrit_model_desc me = encoder_of(md);
  P.Ee.init(&me, st);
  P.Ed.init(md, st);
  P.Ed.per_group_mem = true;
  P.enc_block = P.Ee.lay.block_bytes;
  P.dec_block = P.Ed.lay.block_bytes;
  const int N = op->N, n_dec = N - n_enc;
  const bool serial = serial_run(op);
  const int M0 = serial ? 1 : N / op->cf;
  int gc = max_groups(md, M0);
  const int widest = adjoint ? (N > M0 ? N : M0) : M0;
  if (gc > widest) gc = widest;
  P.Ee.keep_z = P.Ed.keep_z = mode == 2;
  P.Ee.recompute = P.Ed.recompute = adjoint && !g_adjoint_cache;
  if (adjoint) { P.Ee.carve_adjoint(b, gc, n_enc); P.Ed.carve_adjoint(b, gc, n_dec); }
  else { P.Ee.carve_forward(b, gc); P.Ed.carve_forward(b, gc); }
  if (!adjoint && share_ws) {
    // the adjoint plan's first carvings repeated on copies of the engines, in its order and with its chunk
    // size (the encoder's cache, memory copy and work buffers come before the decoder's cache)
    Bump shared(share_ws);
    const int widest_a = N > M0 ? N : M0;
    int gca = max_groups(md, M0);
    if (gca > widest_a) gca = widest_a;
    Engine te = P.Ee, td = P.Ed;
    te.keep_z = td.keep_z = share_mode == 2;
    te.recompute = td.recompute = false;
    te.carve_adjoint(shared, gca, n_enc);
    td.carve_adjoint(shared, gca, n_dec);
    P.Ee.take_cache_from(te);
    P.Ed.take_cache_from(td);
    P.D.fill_cache = true;
  }
  P.two_lanes = widest >= 2 && make_lane(P.Ee2, P.Ee, b, adjoint, ws == nullptr);
  if (P.two_lanes && !make_lane(P.Ed2, P.Ed, b, adjoint, ws == nullptr)) return MGRIT_HIP_ERROR;
  Driver& D = P.D;
  D.E = &P.Ee; D.E2 = P.two_lanes ? &P.Ee2 : nullptr;
  D.Ed = &P.Ed; D.Ed2 = P.two_lanes ? &P.Ed2 : nullptr;
  D.n_enc = n_enc; D.x_elems = P.Ee.Td(); D.y_elems = P.Ed.Td();
  D.adjoint = adjoint; D.N = N; D.cf = op->cf; D.L = serial ? 1 : op->levels; D.relax = op->relax; D.h = op->h;
  D.tabW = b.take<void*>(N + 1);
  D.tabTh = b.take<void*>(N);
  if (adjoint) {
    D.tabZ = b.take<void*>(N + 1);
    D.tabThT = b.take<void*>(N);
    P.thT_blocks = b.take_bytes((size_t)n_enc * P.enc_block + (size_t)n_dec * P.dec_block);
  }
  if (mode == 2) {
    P.tabDT = b.take<void*>(N);
    for (Engine* L : {&P.Ee, &P.Ed, P.two_lanes ? &P.Ee2 : nullptr, P.two_lanes ? &P.Ed2 : nullptr}) {
      if (!L) continue;
      L->carve_grad_work(b);
      if (ws && launch_fill_table(L->tabTB, static_cast<char*>(L->tB), L->tB_stride() * (long)L->esz, L->Gc, st) !=
                    hipSuccess)
        return MGRIT_HIP_ERROR;
    }
  }
  D.tabG.assign(D.L, nullptr);
  if (!serial) {
    D.tabR = b.take<void*>(M0);
    D.max_partial = M0 * resnorm_partials_per_group();
    D.partial = b.take<double>(D.max_partial);
    const size_t state = (size_t)D.state_elems() * sizeof(float);
    char* Rbuf = static_cast<char*>(b.take_bytes(M0 * state));
    std::vector<char*> Gbuf(D.L, nullptr);
    for (int l = 1; l < D.L; ++l) {
      const int Nl = N / Driver::ipow(op->cf, l);
      D.tabG[l] = b.take<void*>(Nl + 1);
      Gbuf[l] = static_cast<char*>(b.take_bytes((size_t)(Nl + 1) * state));
    }
    if (ws) {
      if (launch_fill_table(D.tabR, Rbuf, (long)state, M0, st) != hipSuccess) return MGRIT_HIP_ERROR;
      for (int l = 1; l < D.L; ++l) {
        const int Nl = N / Driver::ipow(op->cf, l);
        if (launch_fill_table(D.tabG[l], Gbuf[l], (long)state, Nl + 1, st) != hipSuccess) return MGRIT_HIP_ERROR;
      }
    }
  }
  P.bytes = (b.off + 255) / 256 * 256;
  return MGRIT_OK;
}
}  // namespace

size_t mgrit_stacked_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc, int adjoint) {
  if (validate_stacked(desc, opts, n_enc) != MGRIT_OK || adjoint < 0 || adjoint > 2) return 0;
  StackedPlan P;
  if (make_stacked_plan(P, desc, opts, n_enc, adjoint, nullptr, nullptr) != MGRIT_OK) return 0;
  return P.bytes;
}

}  // extern "C"

namespace {
int forward_stacked_impl(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc, const void* Z0,
                         const void* const* theta, void* Z_all, float* resnorm, void* workspace,
                         size_t workspace_bytes, void* share_ws, size_t share_bytes, int share_mode, void* stream) {
  std::lock_guard<std::recursive_mutex> call_lock(g_call_mutex);
  STCHK(validate_stacked(desc, opts, n_enc));
  if (!Z0 || !Z_all || !workspace) return MGRIT_INVALID_ARG;
  STCHK(check_ptr_array(theta, opts->N));
  const size_t need = mgrit_stacked_workspace_bytes(desc, opts, n_enc, 0);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (workspace_bytes < need) return MGRIT_WORKSPACE_TOO_SMALL;
  if (share_ws) {
    if (!g_adjoint_cache) return MGRIT_INVALID_ARG;
    const size_t need_adj = mgrit_stacked_workspace_bytes(desc, opts, n_enc, share_mode);
    if (need_adj == 0) return MGRIT_INVALID_ARG;
    if (share_bytes < need_adj) return MGRIT_WORKSPACE_TOO_SMALL;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);

  StackedPlan P;
  STCHK(make_stacked_plan(P, desc, opts, n_enc, 0, workspace, st, share_ws, share_mode));
  Driver& D = P.D;
  const int N = opts->N;
  const size_t state = (size_t)D.state_elems() * sizeof(float);
  HIPCHK(launch_fill_table(D.tabW, static_cast<char*>(Z_all), (long)state, N + 1, st));
  HIPCHK(upload_pointers(D.tabTh, theta, N, st));
  if (Z0 != Z_all) HIPCHK(hipMemcpyAsync(Z_all, Z0, state, hipMemcpyDeviceToDevice, st));
  if (!serial_run(opts) && opts->init_guess == 0) {
    for (int k = 1; k <= N / opts->cf; ++k)
      HIPCHK(hipMemcpyAsync(static_cast<char*>(Z_all) + (size_t)k * opts->cf * state, Z0, state,
                            hipMemcpyDeviceToDevice, st));
  }
  D.resnorm = resnorm;
  return D.run(opts->iters);
}

int adjoint_stacked_impl(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc, const void* Z_all,
                         const void* const* theta, const void* lambda_N, void* lambda_all, void* const* dtheta,
                         float* resnorm, void* workspace, size_t workspace_bytes, bool prefilled, void* stream) {
  std::lock_guard<std::recursive_mutex> call_lock(g_call_mutex);
  if (prefilled && !g_adjoint_cache) return MGRIT_INVALID_ARG;
  STCHK(validate_stacked(desc, opts, n_enc));
  if (!Z_all || !lambda_N || !lambda_all || !workspace) return MGRIT_INVALID_ARG;
  STCHK(check_ptr_array(theta, opts->N));
  if (dtheta) STCHK(check_ptr_array((const void* const*)dtheta, opts->N));
  const int mode = dtheta ? 2 : 1;
  const size_t need = mgrit_stacked_workspace_bytes(desc, opts, n_enc, mode);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (workspace_bytes < need) return MGRIT_WORKSPACE_TOO_SMALL;
  hipStream_t st = static_cast<hipStream_t>(stream);

  StackedPlan P;
  STCHK(make_stacked_plan(P, desc, opts, n_enc, mode, workspace, st));
  Driver& D = P.D;
  const int N = opts->N, n_dec = N - n_enc;
  const size_t state = (size_t)D.state_elems() * sizeof(float);
  HIPCHK(launch_fill_table(D.tabW, static_cast<char*>(lambda_all) + (size_t)N * state, -(long)state, N + 1, st));
  HIPCHK(launch_fill_table(D.tabZ, static_cast<char*>(const_cast<void*>(Z_all)), (long)state, N + 1, st));
  HIPCHK(upload_pointers(D.tabTh, theta, N, st));
  char* tblocks = static_cast<char*>(P.thT_blocks);
  HIPCHK(launch_fill_table(D.tabThT, tblocks, (long)P.enc_block, n_enc, st));
  HIPCHK(launch_fill_table(D.tabThT + n_enc, tblocks + (size_t)n_enc * P.enc_block, (long)P.dec_block, n_dec, st));
  const Params TH = {(const void* const*)D.tabTh, 0, 1};
  const Params THT = {(const void* const*)D.tabThT, 0, 1};
  STCHK(transpose_blocks(P.Ee, n_enc, TH, THT));
  STCHK(transpose_blocks(P.Ed, n_dec, shift(TH, n_enc), shift(THT, n_enc)));
  // linearisation cache, batched over layers: encoder layers at the X rows of Z_n, decoder layers at
  // the Y rows with the X rows of the same state as memory
  const Rows Zrows = {(const void* const*)D.tabZ, 0, 1};
  const Rows ZdecX = shift(Zrows, n_enc), ZdecY = Driver::part(ZdecX, D.x_elems);
  if (prefilled) {
    // the forward solve has left every layer but the last of each interval (n = cf-1, 2cf-1, ..): the
    // encoder layers among those, then the decoder layers
    const int cf = opts->cf, left = serial_run(opts) ? 0 : N / cf;
    int left_e = n_enc >= cf ? (n_enc - cf) / cf + 1 : 0;           // layers cf-1 + k cf below n_enc
    if (left_e > left) left_e = left;
    if (left_e > 0)
      STCHK(forward_groups(P.Ee, D.E2, left_e, Rows{(const void* const*)D.tabZ, cf - 1, cf}, NO_ROWS, NO_ROWS,
                           Params{(const void* const*)D.tabTh, cf - 1, cf}, 0.f, 1, Slots{cf - 1, cf}));
    if (left - left_e > 0) {
      const int n0 = cf - 1 + left_e * cf;                           // first of them in the decoder
      const Rows ZX = {(const void* const*)D.tabZ, n0, cf};
      STCHK(forward_groups(P.Ed, D.Ed2, left - left_e, Driver::part(ZX, D.x_elems), NO_ROWS, NO_ROWS,
                           Params{(const void* const*)D.tabTh, n0, cf}, 0.f, 1, Slots{n0 - n_enc, cf}, ZX));
    }
  } else if (!P.Ee.recompute) {
    STCHK(forward_groups(P.Ee, D.E2, n_enc, Zrows, NO_ROWS, NO_ROWS, TH, 0.f, 1, Slots{0, 1}));
    STCHK(forward_groups(P.Ed, D.Ed2, n_dec, ZdecY, NO_ROWS, NO_ROWS, shift(TH, n_enc), 0.f, 1, Slots{0, 1}, ZdecX));
  }
  char* lamN_row = static_cast<char*>(lambda_all) + (size_t)N * state;
  if (lambda_N != lamN_row) HIPCHK(hipMemcpyAsync(lamN_row, lambda_N, state, hipMemcpyDeviceToDevice, st));
  if (!serial_run(opts) && opts->init_guess == 0) {
    for (int k = 1; k <= N / opts->cf; ++k)
      HIPCHK(hipMemcpyAsync(static_cast<char*>(lambda_all) + (size_t)(N - k * opts->cf) * state, lambda_N, state,
                            hipMemcpyDeviceToDevice, st));
  }
  D.resnorm = resnorm;
  if (dtheta) HIPCHK(upload_pointers(P.tabDT, (const void* const*)dtheta, N, st));
  D.tabDT = dtheta ? P.tabDT : nullptr;
  D.want_grads = dtheta != nullptr;
  STCHK(D.run(opts->iters));
  if (dtheta) {
    // Layer n takes lambda_{n+1}: point N-1-n of the reversed grid.  After the closing F-relaxation has
    // emitted the layers whose lambda_{n+1} it read, the layers n = 0, cf, 2 cf, .. are left (all of them
    // without emission; none after a serial run): the encoder layers among them, then the decoder layers.
    const bool emitted = D.emitted;
    const int stride = emitted ? opts->cf : 1;
    const int count = emitted ? (D.serial() ? 0 : N / opts->cf) : N;
    int count_e = (n_enc + stride - 1) / stride;           // groups g with g * stride < n_enc
    if (count_e > count) count_e = count;
    const Rows LamNext = {(const void* const*)D.tabW, N - 1, -stride};
    const Params DT = {(const void* const*)P.tabDT, 0, stride};
    const Params THs = {(const void* const*)D.tabTh, 0, stride}, THTs = {(const void* const*)D.tabThT, 0, stride};
    const Rows Zs = {(const void* const*)D.tabZ, 0, stride};
    if (count_e > 0)
      STCHK(gradient_groups(P.Ee, D.E2, count_e, LamNext, THs, THTs, Zs, Slots{0, stride}, &DT, nullptr, opts->h));
    if (count - count_e > 0) {
      const Params DTd = shift(DT, count_e);
      const Rows Zx = shift(Zs, count_e);
      StackedDec sd = {Zx, NO_ROWS, NO_ROWS, NO_ROWS};
      STCHK(gradient_groups(P.Ed, D.Ed2, count - count_e, Driver::part(shift(LamNext, count_e), D.x_elems),
                            shift(THs, count_e), shift(THTs, count_e), Driver::part(Zx, D.x_elems),
                            Slots{count_e * stride - n_enc, stride}, &DTd, nullptr, opts->h, &sd));
    }
  }
  return MGRIT_OK;
}
}  // namespace

extern "C" {

int mgrit_forward_stacked(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc, const void* Z0,
                          const void* const* theta, void* Z_all, float* resnorm, void* workspace,
                          size_t workspace_bytes, void* stream) {
  return forward_stacked_impl(desc, opts, n_enc, Z0, theta, Z_all, resnorm, workspace, workspace_bytes, nullptr, 0,
                              0, stream);
}

int mgrit_forward_stacked_linearising(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc,
                                      const void* Z0, const void* const* theta, void* Z_all, float* resnorm,
                                      void* workspace, size_t workspace_bytes, void* adjoint_workspace,
                                      size_t adjoint_workspace_bytes, int with_gradients, void* stream) {
  if (!adjoint_workspace) return MGRIT_INVALID_ARG;
  return forward_stacked_impl(desc, opts, n_enc, Z0, theta, Z_all, resnorm, workspace, workspace_bytes,
                              adjoint_workspace, adjoint_workspace_bytes, with_gradients ? 2 : 1, stream);
}

int mgrit_adjoint_stacked(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc, const void* Z_all,
                          const void* const* theta, const void* lambda_N, void* lambda_all, void* const* dtheta,
                          float* resnorm, void* workspace, size_t workspace_bytes, void* stream) {
  return adjoint_stacked_impl(desc, opts, n_enc, Z_all, theta, lambda_N, lambda_all, dtheta, resnorm, workspace,
                              workspace_bytes, false, stream);
}

int mgrit_adjoint_stacked_linearised(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc,
                                     const void* Z_all, const void* const* theta, const void* lambda_N,
                                     void* lambda_all, void* const* dtheta, float* resnorm, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  return adjoint_stacked_impl(desc, opts, n_enc, Z_all, theta, lambda_N, lambda_all, dtheta, resnorm, workspace,
                              workspace_bytes, true, stream);
}

// ---- buffer layers: serial open / close segments around the MGRIT middle ----------------------
namespace {
int validate_buffer(const mgrit_buffer_opts* b) {
  if (!b || b->n_open < 0 || b->n_close < 0 || !isfinite(b->h_buffer)) return MGRIT_INVALID_ARG;
  return MGRIT_OK;
}
mgrit_opts serial_opts(int n, float h) {
  mgrit_opts o;
  memset(&o, 0, sizeof(o));
  o.N = n; o.h = h; o.cf = 1; o.levels = 1; o.iters = 1; o.relax = MGRIT_RELAX_FCF; o.init_guess = 0;
  return o;
}
}  // namespace

size_t mgrit_buffered_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                      const mgrit_buffer_opts* buf, int adjoint) {
  if (validate_buffer(buf) != MGRIT_OK) return 0;
  size_t need = mgrit_workspace_bytes(desc, opts, adjoint);
  if (need == 0) return 0;
  for (int n : {buf->n_open, buf->n_close}) {
    if (n == 0) continue;
    const mgrit_opts so = serial_opts(n, buf->h_buffer);
    const size_t w = mgrit_workspace_bytes(desc, &so, adjoint);
    if (w == 0) return 0;
    if (w > need) need = w;
  }
  return need;
}

// Segments of a buffered run: the open layers (serial), the MGRIT middle, the close layers (serial).  The
// linearising pair gives each segment's adjoint plan a region of its own in one workspace, in this order.
struct BufferedRegions {
  size_t off[3] = {0, 0, 0}, bytes[3] = {0, 0, 0}, total = 0;
};
static int buffered_regions(const mgrit_model_desc* desc, const mgrit_opts* opts, const mgrit_buffer_opts* buf,
                            int mode, BufferedRegions& R) {
  const mgrit_opts so_open = serial_opts(buf->n_open, buf->h_buffer), so_close = serial_opts(buf->n_close, buf->h_buffer);
  const mgrit_opts* seg[3] = {buf->n_open > 0 ? &so_open : nullptr, opts, buf->n_close > 0 ? &so_close : nullptr};
  size_t off = 0;
  for (int i = 0; i < 3; ++i) {
    R.off[i] = off;
    if (!seg[i]) continue;
    R.bytes[i] = mgrit_workspace_bytes(desc, seg[i], mode);
    if (R.bytes[i] == 0) return MGRIT_INVALID_ARG;
    off += (R.bytes[i] + 255) / 256 * 256;
  }
  R.total = off;
  return MGRIT_OK;
}

size_t mgrit_buffered_linearised_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                                 const mgrit_buffer_opts* buf, int with_gradients) {
  if (validate_desc(desc) != MGRIT_OK || validate_opts(opts) != MGRIT_OK || validate_buffer(buf) != MGRIT_OK) return 0;
  BufferedRegions R;
  if (buffered_regions(desc, opts, buf, with_gradients ? 2 : 1, R) != MGRIT_OK) return 0;
  return R.total;
}

// share_ws: the adjoint workspace of the linearising pair (regions as above), or null
static int forward_buffered_impl(const mgrit_model_desc* desc, const mgrit_opts* opts, const mgrit_buffer_opts* buf,
                                 const void* Z0, const void* const* theta, const void* memory, void* Z_all,
                                 float* resnorm, void* workspace, size_t workspace_bytes, void* share_ws,
                                 size_t share_bytes, int share_mode, void* stream) {
  std::lock_guard<std::recursive_mutex> call_lock(g_call_mutex);
  STCHK(validate_desc(desc));
  STCHK(validate_opts(opts));
  STCHK(validate_buffer(buf));
  if (!Z0 || !Z_all || !theta) return MGRIT_INVALID_ARG;
  const size_t need = mgrit_buffered_workspace_bytes(desc, opts, buf, 0);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (!workspace || workspace_bytes < need) return workspace ? MGRIT_WORKSPACE_TOO_SMALL : MGRIT_INVALID_ARG;
  BufferedRegions R;
  if (share_ws) {
    if (!g_adjoint_cache) return MGRIT_INVALID_ARG;
    STCHK(buffered_regions(desc, opts, buf, share_mode, R));
    if (share_bytes < R.total) return MGRIT_WORKSPACE_TOO_SMALL;
  }
  char* sw = static_cast<char*>(share_ws);
  const size_t state = (size_t)desc->batch * desc->seq * desc->d_model * sizeof(float);
  char* Z = static_cast<char*>(Z_all);
  const int no = buf->n_open, nc = buf->n_close, N = opts->N;
  STCHK(check_ptr_array(theta, no + N + nc));
  const void* z_in = Z0;
  if (no > 0) {
    const mgrit_opts so = serial_opts(no, buf->h_buffer);
    STCHK(forward_impl(desc, &so, z_in, theta, memory, Z, nullptr, workspace, workspace_bytes,
                       sw ? sw + R.off[0] : nullptr, R.bytes[0], share_mode, stream));
    z_in = Z + (size_t)no * state;
  }
  STCHK(forward_impl(desc, opts, z_in, theta + no, memory, Z + (size_t)no * state, resnorm, workspace,
                     workspace_bytes, sw ? sw + R.off[1] : nullptr, R.bytes[1], share_mode, stream));
  if (nc > 0) {
    const mgrit_opts so = serial_opts(nc, buf->h_buffer);
    char* row = Z + (size_t)(no + N) * state;
    STCHK(forward_impl(desc, &so, row, theta + no + N, memory, row, nullptr, workspace, workspace_bytes,
                       sw ? sw + R.off[2] : nullptr, R.bytes[2], share_mode, stream));
  }
  return MGRIT_OK;
}

// prefilled: `workspace` is the region workspace that forward_buffered_impl filled
static int adjoint_buffered_impl(const mgrit_model_desc* desc, const mgrit_opts* opts, const mgrit_buffer_opts* buf,
                                 const void* Z_all, const void* const* theta, const void* memory,
                                 const void* lambda_N, void* lambda_all, void* dmemory, void* const* dtheta,
                                 float* resnorm, void* workspace, size_t workspace_bytes, bool prefilled,
                                 void* stream) {
  std::lock_guard<std::recursive_mutex> call_lock(g_call_mutex);
  STCHK(validate_desc(desc));
  STCHK(validate_opts(opts));
  STCHK(validate_buffer(buf));
  if (!Z_all || !lambda_N || !lambda_all || !theta) return MGRIT_INVALID_ARG;
  // the memory gradient would have to be accumulated over the three segments: not offered here
  if (dmemory) return MGRIT_UNSUPPORTED;
  const int mode = dtheta ? 2 : 1;
  BufferedRegions R;                                   // all three segments share the workspace unless prefilled
  size_t need = mgrit_buffered_workspace_bytes(desc, opts, buf, mode);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (prefilled) {
    if (!g_adjoint_cache) return MGRIT_INVALID_ARG;
    STCHK(buffered_regions(desc, opts, buf, mode, R));
    need = R.total;
  }
  if (!workspace || workspace_bytes < need) return workspace ? MGRIT_WORKSPACE_TOO_SMALL : MGRIT_INVALID_ARG;
  char* ws = static_cast<char*>(workspace);
  auto region = [&](int i) { return prefilled ? static_cast<void*>(ws + R.off[i]) : workspace; };
  auto region_bytes = [&](int i) { return prefilled ? R.bytes[i] : workspace_bytes; };
  const size_t state = (size_t)desc->batch * desc->seq * desc->d_model * sizeof(float);
  const char* Z = static_cast<const char*>(Z_all);
  char* Lm = static_cast<char*>(lambda_all);
  const int no = buf->n_open, nc = buf->n_close, N = opts->N;
  STCHK(check_ptr_array(theta, no + N + nc));
  if (dtheta) STCHK(check_ptr_array((const void* const*)dtheta, no + N + nc));
  const void* lam_in = lambda_N;
  if (nc > 0) {
    const mgrit_opts so = serial_opts(nc, buf->h_buffer);
    const size_t off = (size_t)(no + N) * state;
    STCHK(adjoint_impl(desc, &so, Z + off, theta + no + N, memory, lam_in, Lm + off, nullptr,
                       dtheta ? dtheta + no + N : nullptr, nullptr, region(2), region_bytes(2), prefilled, stream));
    lam_in = Lm + off;
  }
  STCHK(adjoint_impl(desc, opts, Z + (size_t)no * state, theta + no, memory, lam_in, Lm + (size_t)no * state,
                     nullptr, dtheta ? dtheta + no : nullptr, resnorm, region(1), region_bytes(1), prefilled, stream));
  if (no > 0) {
    const mgrit_opts so = serial_opts(no, buf->h_buffer);
    STCHK(adjoint_impl(desc, &so, Z, theta, memory, Lm + (size_t)no * state, Lm, nullptr, dtheta, nullptr,
                       region(0), region_bytes(0), prefilled, stream));
  }
  return MGRIT_OK;
}

int mgrit_forward_buffered(const mgrit_model_desc* desc, const mgrit_opts* opts, const mgrit_buffer_opts* buf,
                           const void* Z0, const void* const* theta, const void* memory, void* Z_all,
                           float* resnorm, void* workspace, size_t workspace_bytes, void* stream) {
  return forward_buffered_impl(desc, opts, buf, Z0, theta, memory, Z_all, resnorm, workspace, workspace_bytes,
                               nullptr, 0, 0, stream);
}

int mgrit_forward_buffered_linearising(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                       const mgrit_buffer_opts* buf, const void* Z0, const void* const* theta,
                                       const void* memory, void* Z_all, float* resnorm, void* workspace,
                                       size_t workspace_bytes, void* adjoint_workspace,
                                       size_t adjoint_workspace_bytes, int with_gradients, void* stream) {
  if (!adjoint_workspace) return MGRIT_INVALID_ARG;
  return forward_buffered_impl(desc, opts, buf, Z0, theta, memory, Z_all, resnorm, workspace, workspace_bytes,
                               adjoint_workspace, adjoint_workspace_bytes, with_gradients ? 2 : 1, stream);
}

int mgrit_adjoint_buffered(const mgrit_model_desc* desc, const mgrit_opts* opts, const mgrit_buffer_opts* buf,
                           const void* Z_all, const void* const* theta, const void* memory, const void* lambda_N,
                           void* lambda_all, void* dmemory, void* const* dtheta, float* resnorm, void* workspace,
                           size_t workspace_bytes, void* stream) {
  return adjoint_buffered_impl(desc, opts, buf, Z_all, theta, memory, lambda_N, lambda_all, dmemory, dtheta, resnorm,
                               workspace, workspace_bytes, false, stream);
}

int mgrit_adjoint_buffered_linearised(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                      const mgrit_buffer_opts* buf, const void* Z_all, const void* const* theta,
                                      const void* memory, const void* lambda_N, void* lambda_all, void* dmemory,
                                      void* const* dtheta, float* resnorm, void* workspace, size_t workspace_bytes,
                                      void* stream) {
  return adjoint_buffered_impl(desc, opts, buf, Z_all, theta, memory, lambda_N, lambda_all, dmemory, dtheta, resnorm,
                               workspace, workspace_bytes, true, stream);
}

int layer_step_batched(const mgrit_model_desc* desc, int adjoint, int n_groups, const void* const* in,
                       void* const* out, const void* const* theta, const void* const* lin_state,
                       const void* const* rhs, const void* memory, float hstep, void* workspace,
                       size_t workspace_bytes, void* stream) {
  return layer_step_on(desc, adjoint, n_groups, in, out, theta, lin_state, rhs, memory, hstep, workspace,
                       workspace_bytes, stream, true);
}

size_t mgrit_layer_step_static_bytes(const mgrit_model_desc* desc, int adjoint, int n_groups) {
  return layer_step_bytes(desc, adjoint, n_groups, false);
}

int layer_step_batched_static(const mgrit_model_desc* desc, int adjoint, int n_groups, const void* const* in,
                              void* const* out, const void* const* theta, const void* const* lin_state,
                              const void* const* rhs, const void* memory, float hstep, void* stream) {
  STCHK(validate_desc(desc));
  if (n_groups < 1) return MGRIT_INVALID_ARG;
  const size_t need = layer_step_bytes(desc, adjoint, n_groups, false);
  if (need == 0) return MGRIT_INVALID_ARG;
  if (need > (size_t)MGRIT_STATIC_SCRATCH_BYTES) return MGRIT_WORKSPACE_TOO_SMALL;
  void* ws = nullptr;
  STCHK(static_scratch(&ws));
  return layer_step_on(desc, adjoint, n_groups, in, out, theta, lin_state, rhs, memory, hstep, ws,
                       (size_t)MGRIT_STATIC_SCRATCH_BYTES, stream, false);
}

const char* mgrit_status_string(int status) {
  switch (status) {
    case MGRIT_OK: return "ok";
    case MGRIT_INVALID_ARG: return "invalid argument";
    case MGRIT_UNSUPPORTED: return "unsupported configuration";
    case MGRIT_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MGRIT_HIP_ERROR: return "HIP error";
  }
  return "unknown status";
}

int mgrit_last_hip_error(void) { return g_last_hip_error; }

void mgrit_set_max_groups_per_launch(int n) { g_max_groups = n > 0 ? n : 0; }
int mgrit_default_groups_per_launch(const mgrit_model_desc* desc, int sweep) {
  if (validate_desc(desc) != MGRIT_OK) return 0;
  return default_groups(desc, sweep);
}

void mgrit_set_lanes(int n) { g_lanes = n >= 2 ? 2 : 1; }
void mgrit_set_adjoint_cache(int on) { g_adjoint_cache = on ? 1 : 0; }

// test / tuning hooks (not part of the documented interface)
void mgrit_debug_force_simple_kernels(int gemm, int attn) {
  gemm_force_simple(gemm);
  attn_force_simple(attn);
}

void mgrit_debug_gemm_tile_config(int cfg) { gemm_set_tile_config(cfg); }
void mgrit_debug_attention_wide_blocks(int mask) { attn_set_wide_blocks(mask); }
void mgrit_debug_pipeline_coarse_solve(int on) { g_pipeline = on ? 1 : 0; }
void mgrit_debug_pipeline_chunk(int n) { g_pipe_chunk = n > 0 ? n : 0; }

}  // extern "C"
