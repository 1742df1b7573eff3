// Host-side launchers of the kernels (all enqueue on the given stream, none synchronises).
#pragma once
#include "common.h"

namespace mg {

// ---- gemm.hip ----------------------------------------------------------------
hipError_t launch_gemm(const GemmArgs& a, int epi, bool is_bf16, hipStream_t st);
void gemm_force_simple(int on);
void gemm_set_tile_config(int cfg);
double gemm_model_cost(int n_groups, int M, int N, int K);
void attn_set_wide_blocks(int mask);

// ---- rowwise.hip -------------------------------------------------------------
struct LnFwdArgs {
  int n_groups, T, d;
  Rows X;                                   // LN input = X rows (optional) + packed addend (optional)
  const float* xp; long xp_slot_stride; Slots xp_slots;   // packed fp32 addend
  Params P; long gamma_off, beta_off;
  void* out; long out_slot_stride; Slots out_slots;       // packed, operand type
  float eps;
  // optional (linearisation cache): the normalised row xhat = (x - mean) * rstd, packed operand type with
  // the same row layout as `out`, and rstd, one float per row ([slot][T])
  void* xhat; long xhat_slot_stride; Slots xhat_slots;
  float* rstd;
};
hipError_t launch_ln_fwd(const LnFwdArgs& a, bool is_bf16, hipStream_t st);

struct LnBwdArgs {
  int n_groups, T, d;
  const void* dy; long dy_slot_stride; Slots dy_slots;    // packed operand type: cotangent of LN output
  Rows X;                                                 // LN input = X rows (optional) + addend (optional)
  const float* xp; long xp_slot_stride; Slots xp_slots;   // packed fp32 addend
  Params P; long gamma_off;
  const float* add; long add_slot_stride; Slots add_slots;   // optional packed fp32 added to the VJP
  float* out_f32; long of_slot_stride; Slots of_slots;       // optional: v = add + vjp
  Rows C;                                                     // cotangent rows c (required if out_op or OUT)
  void* out_op; long oo_slot_stride; Slots oo_slots;         // optional packed operand type: c + v
  Rows OUT; Rows RHS; float hstep;                           // optional: OUT = c + hstep*v (+ RHS)
  float rhs_sign;                                            // with RHS: OUT = RHS + rhs_sign * (c + hstep*v), +1 or -1
  float eps;
  // optional: the LN input given as cached xhat (packed operand type) and rstd ([slot][T]) instead of X / xp
  const void* xhat; long xhat_slot_stride; Slots xhat_slots;
  const float* rstd;
  // optional: c as a packed operand-type copy, used for out_op in place of the fp32 rows C
  const void* cop; long cop_slot_stride; Slots cop_slots;
  // optional (with OUT): the same values as OUT once more as a packed operand-type copy
  void* out_cast; long oc_slot_stride; Slots oc_slots;
};
hipError_t launch_ln_bwd(const LnBwdArgs& a, bool is_bf16, hipStream_t st);

// packed operand-type copy of fp32 rows
hipError_t launch_cast_rows(int n_groups, long elems, Rows X, void* out, long out_slot_stride, Slots out_slots,
                            bool is_bf16, hipStream_t st);
// packed operand-type copy of one fp32 array
hipError_t launch_cast_flat(const float* in, void* out, long elems, bool is_bf16, hipStream_t st);
// dst[g] = a[g] - b[g]  on fp32 rows
hipError_t launch_sub_rows(int n_groups, long elems, Rows A, Rows B, Rows D, hipStream_t st);
hipError_t launch_add_rows(int n_groups, long elems, Rows A, Rows B, Rows D, hipStream_t st);   // D = A (+ B)
// partial[block] = sum over the block's elements of (a-b)^2 in double; then out[0] = sqrt(sum partial)
hipError_t launch_resnorm(int n_groups, long elems, Rows A, Rows B, double* partial, int max_partial,
                          float* out, hipStream_t st);
// tab[i] = base + i*stride_bytes, i < n
hipError_t launch_fill_table(void** tab, char* base, long stride_bytes, int n, hipStream_t st);
// tab[i] = ptrs[i]: pointers travel as kernel arguments (safe for any host memory, capturable)
hipError_t upload_pointers(void** tab, const void* const* host_ptrs, int n, hipStream_t st);
// out_g[c, r] = in_g[r, c] for every group; in/out found at byte offset `off` of the blocks
hipError_t launch_transpose(int n_groups, Params in, Params out, long off, int rows, int cols, int elem_bytes,
                            hipStream_t st);

// ---- grads.hip ---------------------------------------------------------------
// dst_g[c, r] = src_g[r, c] (or GELU of it) on packed operand-type buffers, src [rows, cols].
// With `partial` (n_groups * transpose_row_blocks(rows) * cols floats of scratch) also
// sum_out_g[c] (fp32, at byte offset sum_off of the group's output block) = sum_scale * sum over rows of src_g[r, c].
int transpose_row_blocks(int rows);
hipError_t launch_transpose_slots(int n_groups, const void* src, long src_slot_stride, Slots src_slots, int rows,
                                  int cols, void* dst, long dst_slot_stride, Slots dst_slots, bool gelu,
                                  bool is_bf16, float* partial, Params sum_out, long sum_off, float sum_scale,
                                  hipStream_t st);
// LayerNorm gain / shift gradients: sums over tokens of dy * xhat and dy, scaled
struct LnParamArgs {
  int n_groups, T, d;
  const void* dy; long dy_slot_stride; Slots dy_slots;    // packed operand type: cotangent of the LN output
  Rows X;                                                 // LN input = X rows (optional) + addend (optional)
  const float* xp; long xp_slot_stride; Slots xp_slots;
  Params out; long gamma_off, beta_off;                   // fp32 outputs inside the group's output block
  float scale, eps;
};
// out[i] = scale * sum over s < n of in[s * elems + i]   (fixed order)
hipError_t launch_sum_slots(const float* in, int n, long elems, float* out, float scale, hipStream_t st);
int ln_param_partial_rows();          // partial: n_groups * ln_param_partial_rows() * 2 * d floats
hipError_t launch_ln_param_grad(const LnParamArgs& a, float* partial, bool is_bf16, hipStream_t st);

// ---- attention.hip -----------------------------------------------------------
struct AttnArgs {
  int n_groups, B, H, dh, Sq, Sk, causal;
  const void* q; long q_row_stride, q_slot_stride; Slots q_slots;    // operand type; head h at column h*dh
  const void* k; long k_row_stride, k_slot_stride; Slots k_slots;
  const void* v; long v_row_stride, v_slot_stride;                   // same slots as k
  void* o; long o_row_stride, o_slot_stride; Slots o_slots;          // forward output / backward input
  float* lse; long lse_slot_stride; Slots lse_slots;                 // [B,H,Sq] per slot (fwd: optional out)
  // backward only
  const void* dO; long do_row_stride, do_slot_stride; Slots do_slots;
  void* dq; void* dk; void* dv; long dqkv_row_stride, dqkv_slot_stride; Slots dqkv_slots;
  long dkv_row_stride, dkv_slot_stride;                              // dk, dv if laid out unlike dq (0: same)
  float* D; long D_slot_stride; Slots D_slots;                       // [B,H,Sq] scratch: rowsum(dO*O)
};
hipError_t launch_attn_fwd(const AttnArgs& a, bool is_bf16, hipStream_t st);
hipError_t launch_attn_bwd(const AttnArgs& a, bool is_bf16, hipStream_t st);
void attn_force_simple(int on);

}  // namespace mg
