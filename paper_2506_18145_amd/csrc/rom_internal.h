// Internal declarations shared by the librom translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rom.h"

namespace rom {

typedef unsigned short bf16_t;  // raw bf16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(static_cast<unsigned int>(v) << 16);
}
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float hw_f32x2_t __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 pair (lo in bits 0..15), round-to-nearest-even: one v_cvt_pk_bf16_f32
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {
  const hw_f32x2_t f = {lo, hi};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(f, hw_bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return static_cast<bf16_t>(pack_bf16x2(f, 0.0f) & 0xFFFFu);
}
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

__device__ __forceinline__ float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ float fast_rcp(float v) { return __builtin_amdgcn_rcpf(v); }
// SiLU(v) = v / (1 + exp(-v))
__device__ __forceinline__ float silu_f32(float v) {
  return v * fast_rcp(1.0f + fast_exp2(-1.44269504088896341f * v));
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------- routing (Eq. (9))
// logits may be NULL.  tok_of_pos[p] = perm[p] / K.  block_counts: i32 [route_blocks(S), E].
// norm_w (f32 [d_model]) != NULL: route on the RMS-normalised input and write rstd (f32 [N]).
int64_t route_blocks(int64_t n_slots);
hipError_t launch_route_topk(int dtype, const void *x, const void *w_router, const float *b_router,
                             int64_t n_tokens, int d_model, int n_experts, int top_k, int gate_mode,
                             int32_t *expert_idx, float *gate, float *logits, const float *norm_w,
                             float norm_eps, float *rstd, hipStream_t s);
hipError_t launch_permutation(const int32_t *expert_idx, int64_t n_slots, int n_experts, int top_k,
                              int32_t *block_counts, int32_t *counts, int32_t *offsets,
                              int32_t *perm, int32_t *inv_perm, int32_t *tok_of_pos, hipStream_t s);

// K > 1: for every rank r < K, the N tokens grouped by their r-th expert (stable): rank_offsets
// i32 [K][E + 1] (each rank's offsets start at 0), tok_of_rank_pos i32 [K][N] = token at that
// rank's sorted position; block_counts: scratch of rank_grouping_block_counts_bytes
size_t rank_grouping_block_counts_bytes(int64_t n_tokens, int n_experts, int top_k);
hipError_t launch_rank_grouping(const int32_t *expert_idx, int64_t n_tokens, int n_experts, int top_k,
                                int32_t *block_counts, int32_t *rank_offsets, int32_t *tok_of_rank_pos,
                                hipStream_t s);

// load-balance statistics (Eq. (16)); partial: f32 scratch of balance_scratch_bytes(E)
size_t balance_scratch_bytes(int n_experts);
hipError_t launch_balance_stats(const float *logits, const int32_t *counts, int64_t n_tokens,
                                int n_experts, int top_k, float alpha, float *partial, float *frac,
                                float *mean_prob, float *loss, hipStream_t s);

// ---------------------------------------------------------------- grouped GEMM
// C[c_row(p), :] = epilogue( A[a_row(p), :] . W[e(p)]^T ),  p = sorted position in [0, M)
// e(p) from offsets (device, i32 [n_groups+1]); offsets == NULL means one group of M rows.
struct GemmArgs {
  int dtype;                 // ROM_DTYPE_*: type of A and W
  const void *A;             // [*, lda]
  int64_t lda;
  const int32_t *a_rows;     // row of A for position p, NULL = p
  int64_t a_span;            // number of elements of A that may be addressed (rows * lda)
  const void *W;             // [n_groups, N, K] row-major
  const int32_t *offsets;    // NULL = single group; group e is the rows [offsets[e], offsets[e + 1]) (device, i32 [n_groups+1])
  int n_groups;
  int64_t M;                 // total rows (positions)
  int N, K;                  // out features, in features
  void *C;                   // [*, ldc]
  int64_t ldc;
  const int32_t *c_rows;     // row of C for position p, NULL = p
  int c_is_f32;              // 1: C is float regardless of dtype; 0: C has type T
  const float *bias;         // [N] or NULL: added before softplus
  int softplus;              // apply softplus after bias
  const float *row_scale;    // indexed by c_row (NULL = 1): multiplies the row
  const void *residual;      // type T, laid out like C (row c_row, pitch ldc), or NULL: added after the row scale
  int swiglu;                // 1: W's rows are blocks of 8 gate + 8 up features; C [*, N/2] = SiLU(gate) * up
                             // (after the row scale); MFMA kernels only, see grouped_gemm_on_mfma
  int w_kmajor;              // 1: W is [n_groups, K, N] row-major (contraction-major); only where
                             // grouped_gemm_takes_kmajor says so
  int no_xcd_remap;          // set by the launcher: logical tile = workgroup id (no contiguous run per XCD)
  int k_splits;              // > 1: slice the inner dimension; slice s writes its partial sums (fp32, plain
                             // epilogue only) to C + s * c_split_stride; the consumer adds the slices up
  int64_t c_split_stride;    // elements between the outputs of consecutive slices
  int k_per_split;           // filled in by launch_grouped_gemm
};
hipError_t launch_grouped_gemm(const GemmArgs &a, hipStream_t s);
bool grouped_gemm_on_mfma(const GemmArgs &a);
bool grouped_gemm_takes_kmajor(const GemmArgs &a);

// ---------------------------------------------------------------- sequence kernels
// sum over the K slots of a token: dst[n, :] = act(row_scale[n] * sum_k src[inv_perm[n*K+k], :] + bias)
// (row_scale f32 [n_tokens] or NULL, bias f32 [n_cols] or NULL)
hipError_t launch_slot_sum(int src_is_f32, int dst_is_f32, const void *src, int64_t ld_src, void *dst,
                           int64_t ld_dst, const int32_t *inv_perm, int64_t n_tokens, int top_k,
                           int n_cols, const float *bias, int softplus, const float *row_scale,
                           hipStream_t s);
// xdbl (f32 [*, R + 32], token order or sorted) -> dt_low (T [N, R]) and bc (f32 [N, 32])
hipError_t launch_split_xdbl(int dtype, const float *xdbl, int n_slices, int64_t slice_stride,
                             const int32_t *inv_perm, int top_k, int64_t n_tokens, int dt_rank,
                             void *dt_low, float *bc, hipStream_t s);
// number of inner-dimension slices the x projection is cut into (small batches only)
int xproj_k_splits(int64_t rows, int n_groups, int d_inner);
// a sequence of at most this many steps is one run of one conv thread: its state may be updated in place
constexpr int kConvInPlaceMaxLen = 32;
hipError_t launch_conv_silu(int dtype, const void *xz, int64_t ld_xz, const float *conv_w,
                            const float *conv_b, const float *state_in, float *state_out, void *u,
                            int64_t B, int64_t L, int d_inner, hipStream_t s);
// chunk_q / chunk_p: f32 scratch of scan_chunk_state_bytes() each (chunk end states and decays)
size_t scan_chunk_state_bytes(int64_t B, int64_t L, int d_inner);
hipError_t launch_scan_gate(int dtype, const void *u, const void *dt, const float *bc, const void *z,
                            int64_t ld_z, const float *A_log, const float *D, const float *h_in,
                            float *h_out, void *g, int64_t B, int64_t L, int d_inner, float *chunk_q,
                            float *chunk_p, hipStream_t s);
// out[n, :] = (residual[n, :] if given) + sum_k gate[n*K+k] * op[inv_perm[n*K+k], :]
hipError_t launch_combine(int dtype, const void *op, const int32_t *inv_perm, const float *gate,
                          void *out, int64_t n_tokens, int top_k, int d_model, const void *residual,
                          hipStream_t s);

// ---------------------------------------------------------------- backward pass (rom_bwd.hip)
// scratch of the adjoint scan: state checkpoints, chunk carries and per-unit parameter-gradient partials
size_t scan_bwd_ckpt_bytes(int64_t B, int64_t L, int d_inner);
size_t scan_bwd_part_bytes(int64_t n_tok, int d_inner);
// adjoint of scan + gate + softplus: dg is d loss / d (W_out^T d_out) per token, gate (f32 [N] or NULL = 1) the
// weight it is multiplied by; writes d_pre (w.r.t. the softplus argument), d_u (scan part), d_z (pitch ld_dz), all of
// the activation type, d_bc f32 [N, 32], and the parameter gradients d_A_log [d_inner, 16], d_D, d_dt_bias [d_inner]
hipError_t launch_scan_backward(int dtype, const void *u, const void *dt, const float *bc, const void *z, int64_t ld_z,
                                const void *dg, const float *gate, const float *A_log, const float *D, int64_t B,
                                int64_t L, int d_inner, float *ckpt, float *d_bc_part, void *d_pre, void *d_u, void *d_z,
                                int64_t ld_dz, float *d_bc, float *d_A_log, float *d_D, float *d_dt_bias,
                                hipStream_t s);
// d_gate[r] = a[r / a_div, :] . b[b_rows ? b_rows[r] : r, :] over n_cols columns
hipError_t launch_gate_backward(int dtype, const void *a, const void *b, const int32_t *b_rows, int a_div,
                                int64_t n_rows, int n_cols, float *d_gate, hipStream_t s);
size_t router_bwd_partial_bytes(int64_t n_tok, int d_model, int n_experts);
hipError_t launch_router_backward(int dtype, const float *logits, const int32_t *expert_idx, const float *d_gate,
                                  const void *x, int64_t n_tok, int d_model, int n_experts, int top_k, int gate_mode,
                                  float *d_logits, float *partial, float *d_w_router, float *d_b_router, hipStream_t s);
hipError_t launch_dx_finish(int dtype, const void *dx_in, const float *d_logits, const void *w_router, int64_t n_tok,
                            int d_model, int n_experts, void *d_x, hipStream_t s);
size_t conv_bwd_partial_bytes(int64_t B, int64_t L, int d_inner);
hipError_t launch_conv_backward(int dtype, const void *xz, int64_t ld_xz, const float *conv_w, const float *conv_b,
                                const void *du_a, const void *du_b, int64_t B, int64_t L, int d_inner, void *d_xpre,
                                int64_t ld_dx, float *partial, float *d_conv_w, float *d_conv_b, hipStream_t s);
// dst[m][c][r] = src[m][r][c] for n_mats matrices
hipError_t launch_transpose(int dtype, const void *src, void *dst, int n_mats, int rows, int cols, hipStream_t s);
hipError_t launch_pack_dxdbl(int dtype, const float *d_dt_low, const float *d_bc, int64_t n_tok, int dt_rank,
                             void *d_xdbl, hipStream_t s);
// dst[r, :] = scale[scale_idx ? scale_idx[r] : r] * src[src_idx ? src_idx[r] : r, :]
// RMS norm of the pre-norm block: xn = x / sqrt(mean(x^2) + eps) * norm_w (type T), rstd f32 [n_rows]
hipError_t launch_rmsnorm_forward(int dtype, const void *x, const float *norm_w, float eps, int64_t n_rows, int d_model,
                                  void *xn, float *rstd, hipStream_t s);
// its adjoint plus the skip: d_x = d_skip + d(RMSNorm)^T d_xn (d_skip NULL: none); d_norm_w = column sums of d_xn x rstd
// (part: f32 [rmsnorm_wgrad_parts(n_rows), d_model], summed in part order)
int rmsnorm_wgrad_parts(int64_t n_rows);
hipError_t launch_rmsnorm_backward(int dtype, const void *x, const float *norm_w, const float *rstd, const void *d_xn,
                                   const void *d_skip, int64_t n_rows, int d_model, void *d_x, float *part,
                                   float *d_norm_w, hipStream_t s);
hipError_t launch_scale_rows(int dtype, const void *src, const float *scale, const int32_t *src_idx,
                             const int32_t *scale_idx, int64_t n_rows, int n_cols, void *dst, hipStream_t s);
// C[e][m][n] (f32) = sum over positions p in [offsets[e], offsets[e+1]) of scale[ra(p)] * A[ra(p)][m] * B[rb(p)][n]
// (rows_a / rows_b NULL: the position itself; offsets NULL: one group over [0, n_pos); row_scale NULL: 1)
hipError_t launch_wgrad(int dtype, const void *A, int64_t lda, int M, const void *Bm, int64_t ldb, int N,
                        const int32_t *rows_a, const int32_t *rows_b, const float *row_scale, const int32_t *offsets,
                        int n_groups, int64_t n_pos, float *C, hipStream_t s);

// ---------------------------------------------------------------- RoM on Mamba2 (rom_mamba2.hip; bf16 only)
// Mamba2's recurrence per head of 64 channels with the D skip and the SiLU(z) gate:
//   xbc bf16 [B*L, ld_xbc] holds x (head h at columns x_col + 64 h), B (b_col .. + d_state) and C (c_col ..)
//   after conv + SiLU; dt_raw bf16 [B*L, ld_dt], column dt_col + h, before bias and softplus; z bf16
//   [B*L, ld_z], head h at columns 64 h; dt_bias, A_log, D f32 [n_heads]; yz bf16 [B*L, ld_y] =
//   (y + D x) * SiLU(z); h_in / h_out f32 [B, n_heads, d_state, 64] or NULL: the state before the first
//   and after the last step (they may be the same buffer only for L <= 64: one chunk, one segment);
//   carry: f32 scratch of ssd_carry_bytes()
bool ssd_supported(int d_state, int headdim);
size_t ssd_carry_bytes(int64_t B, int64_t L, int n_heads, int d_state);
hipError_t launch_ssd_scan(const void *xbc, int64_t ld_xbc, int x_col, int b_col, int c_col, const void *dt_raw,
                           int64_t ld_dt, int dt_col, const void *z, int64_t ld_z, const float *dt_bias,
                           const float *A_log, const float *D, const float *h_in, float *h_out, int64_t B, int64_t L,
                           int n_heads, int d_state, float *carry, void *yz, int64_t ld_y, hipStream_t s);
// out[n, :] = in[n, :] / sqrt(mean(in[n, :]^2) + eps) * w  (bf16 rows of n_cols, n_cols % 8 == 0; out may be in)
hipError_t launch_rms_rows(const void *in, const float *w, float eps, int64_t n_rows, int n_cols, void *out,
                           hipStream_t s);

// ---------------------------------------------------------------- RoM on Gated DeltaNet (rom_gdn.hip; bf16 only)
// The gated delta rule per head (d_v = 64 value channels, d_k = 64 or 128), q and k L2-normalised inside,
// followed by the per-head RMS norm and the SiLU(z) gate:
//   qkv bf16 [B*L, ld_qkv] after conv + SiLU: q of head h at q_col + d_k h, k at k_col + d_k h, v at v_col + 64 h;
//   proj bf16 [B*L, ld_p]: z of head h at columns 64 h, the beta logit at b_col + h, the decay logit at a_col + h;
//   dt_bias, A_log f32 [n_heads]; norm_w f32 [64]; s_in / s_out f32 [B, n_heads, d_k, 64] or NULL;
//   y bf16 [B*L, ld_y]; carry: f32 scratch of gdn_carry_bytes() (segment carries of long, few sequences)
bool gdn_supported(int d_k, int d_v);
size_t gdn_carry_bytes(int64_t B, int64_t L, int n_heads, int d_k);
hipError_t launch_gdn_scan(const void *qkv, int64_t ld_qkv, int q_col, int k_col, int v_col, const void *proj, int64_t ld_p,
                           int b_col, int a_col, const float *dt_bias, const float *A_log, const float *norm_w, float eps,
                           int64_t B, int64_t L, int n_heads, int d_k, const float *s_in, float *s_out, float *carry,
                           void *y, int64_t ld_y, hipStream_t s);

// timing probes (bench.py --probe): out is f32 scratch of n_blocks * 256 floats
hipError_t launch_probe_issue(int op, int chains, int n_blocks, int iters, float *out, hipStream_t s);
hipError_t launch_probe_scan(int parts, int lds, int n_blocks, int tiles, float *out, hipStream_t s);

// ---------------------------------------------------------------- FFN-MoE (Eq. (14), (15))
// a[p, 8b + t] = SiLU(h[p, 16b + t]) * h[p, 16b + 8 + t], t < 8: h's columns are blocks of 8 gate + 8 up
// features (h T [n_rows, 2*d_ff], a T [n_rows, d_ff]; d_ff % 8 == 0)
hipError_t launch_swiglu(int dtype, const void *h, void *a, int64_t n_rows, int d_ff, hipStream_t s);
// its adjoint: d_h (packed column order, T [n_rows, 2 d_ff]) from h and d_a (T [n_rows, d_ff])
hipError_t launch_swiglu_backward(int dtype, const void *h, const void *d_a, void *d_h, int64_t n_rows, int d_ff,
                                  hipStream_t s);
// dst = a + b over n_elems elements of type T (a multiple of 16 bytes; 16-byte aligned)
hipError_t launch_add(int dtype, const void *a, const void *b, void *dst, int64_t n_elems, hipStream_t s);
// tok_of_pos[p] = perm[p] / K; rstd_sorted (may be NULL) [p] = 1 / sqrt(mean(x[tok_of_pos[p]]^2) + eps)
hipError_t launch_ffn_prep(int dtype, const int32_t *perm, int top_k, int64_t n_slots, const void *x,
                           int d_model, float eps, int32_t *tok_of_pos, float *rstd_sorted, hipStream_t s);

}  // namespace rom
