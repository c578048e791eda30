// C ABI of librom: argument validation, workspace planning and the launch sequences of the
// RoM layer forward pass (Eq. (9)-(13)) and its single-token recurrent step, of the pre-norm
// residual block and stacks of blocks around it, of the FFN-MoE layer that shares the layer's
// routing decision (appendix Eq. (14), (15)) and of the load-balance statistics (Eq. (16)).
#include <string.h>

#include <mutex>

#include "rom_internal.h"

// Scratch of rom_step_static: one copy per GPU the library is loaded on, held until the process
// ends.  Host code never uses this name as an address: the per-device address comes from
// hipGetSymbolAddress (static_scratch_for_current_device below).
constexpr size_t kStaticScratchBytes = static_cast<size_t>(32) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace rom {
namespace {

constexpr size_t kAlign = 256;
constexpr size_t kNone = static_cast<size_t>(-1);

struct Plan {                 // byte offsets inside the workspace
  size_t total;
  size_t expert_idx, gate, counts, offsets, perm, inv_perm, tok_of_pos, block_counts, logits;
  size_t balance_part;        // scratch of rom_balance_stats: placed so that it depends on N, K, E only
  size_t xz, xz_sorted, u, xdbl, dt_low, bc, dt, dt_raw, g, op_sorted, conv_tmp;
  size_t scan_q, scan_p;      // chunk end states / decays of a time-chunked scan
  size_t rstd;                // f32 [N]: 1 / rms of every token of a pre-norm block's input
  int xproj_slices;           // inner-dimension slices the xdbl buffer has room for
  // K == 2 on long inputs: the routed dt projection runs as two passes over the tokens, pass r on
  // every token's r-th expert, the second accumulating into the token-order output and activating
  // (no per-slot staging buffer, no slot sum)
  bool rank_passes;
  size_t rank_offsets, rank_tok, rank_blocks;   // i32 [K][E + 1], i32 [K][N], scratch of the per-rank grouping
};

// Rank passes need the accumulate-then-activate form of the dt projection, which only the
// streaming small-K kernel has (bf16, dt_rank 32 / 64 / 128); short inputs keep the per-slot path
// (its single launches suit the decode step better than two short ones).  Only K == 2: the output
// between two passes is stored in the activation type, so with two passes exactly one addend is
// rounded before the sum - one rounding fewer than per-slot outputs - while every further pass
// would round the growing running sum again (measured at K = 4: 1.7 times the per-slot path's
// error, over the tolerance on dt).
// Only the dt projection: the in projection was run the same way and measured slower than the
// per-slot path (d_model 2048, 16 experts, 16K tokens: 1.29 ms against 1.19): its second pass reads
// the first one's 256 MiB back in the epilogue, through the L1 miss queue and with nothing to
// overlap, which costs more than the slot sum's streaming read; the x projection gained nothing
// (its passes are two more short launches).  The dt projection's accumulating read happens in a
// kernel that is store-bound anyway: 0.30 -> 0.18 ms.
bool use_rank_passes(const rom_dims *d, int64_t n_tok) {
  if (d->top_k != 2 || n_tok < 2048 || d->dtype != ROM_DTYPE_BF16 || d->n_experts_xdt <= 1) return false;
  return d->dt_rank == 32 || d->dt_rank == 64 || d->dt_rank == 128;
}

int check_dims(const rom_dims *d) {
  if (!d) return ROM_E_INVAL;
  if (d->dtype != ROM_DTYPE_F32 && d->dtype != ROM_DTYPE_BF16) return ROM_E_INVAL;
  if (d->gate_mode != 0 && d->gate_mode != 1) return ROM_E_INVAL;
  if (d->d_model <= 0 || d->d_inner <= 0 || d->dt_rank <= 0 || d->n_experts <= 0) return ROM_E_INVAL;
  if (d->top_k < 1 || d->top_k > d->n_experts) return ROM_E_INVAL;
  if (d->n_experts_xdt != 1 && d->n_experts_xdt != d->n_experts) return ROM_E_INVAL;
  if (d->d_state != 16 || d->d_conv != 4) return ROM_E_UNSUPPORTED;
  if (d->n_experts > 64 || d->top_k > 8) return ROM_E_UNSUPPORTED;
  if (d->d_inner % 16 != 0 || d->d_model % 8 != 0) return ROM_E_UNSUPPORTED;
  return ROM_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_weights(const rom_dims *d, const rom_weights *w) {
  if (!w) return ROM_E_INVAL;
  const void *req[] = {w->w_router, w->w_in, w->conv_w, w->w_x, w->w_dt, w->dt_bias, w->A_log, w->D, w->w_out};
  for (const void *p : req)
    if (!p || !aligned16(p)) return ROM_E_INVAL;
  if ((w->b_router && !aligned16(w->b_router)) || (w->conv_b && !aligned16(w->conv_b))) return ROM_E_INVAL;
  (void)d;
  return ROM_OK;
}

// slices of the x projection's inner dimension for a launch over `rows` rows
int xproj_slices_for(const rom_dims *d, int64_t rows) {
  const bool routed_xdt = d->n_experts_xdt > 1;
  int n = xproj_k_splits(rows, routed_xdt ? d->n_experts : 1, d->d_inner);
  const int64_t per = ceil_div(ceil_div(d->d_inner, n), 64) * 64;   // whole 64-wide slabs
  return static_cast<int>(ceil_div(d->d_inner, per));
}

Plan make_plan(const rom_dims *d, int64_t n_seq, int64_t seq_len) {
  const int64_t n_tok = n_seq * seq_len;
  Plan p;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  };
  const size_t N = static_cast<size_t>(n_tok), K = d->top_k, S = N * K, E = d->n_experts;
  const size_t b = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;
  const size_t De = d->d_inner, Dm = d->d_model, R = d->dt_rank;
  const bool multi = K > 1;
  const bool routed_xdt = d->n_experts_xdt > 1;
  p.rank_passes = use_rank_passes(d, n_tok);
  p.xproj_slices = xproj_slices_for(d, n_tok * (routed_xdt ? d->top_k : 1));
  p.expert_idx = take(S * 4);
  p.gate = take(S * 4);
  p.counts = take(E * 4);
  p.offsets = take((E + 1) * 4);
  p.perm = take(S * 4);
  p.inv_perm = take(S * 4);
  p.tok_of_pos = take(S * 4);
  p.block_counts = take(static_cast<size_t>(route_blocks(static_cast<int64_t>(S))) * E * 4);
  p.logits = take(N * E * 4);
  p.balance_part = take(balance_scratch_bytes(d->n_experts));
  p.xz = take(N * 2 * De * b);
  p.xz_sorted = multi ? take(S * 2 * De * b) : kNone;
  p.u = take(N * De * b);
  p.xdbl = take((routed_xdt ? S : N) * (R + 32) * 4 * p.xproj_slices);
  p.dt_low = take(N * R * b);
  p.bc = take(N * 32 * 4);
  p.dt = take(N * De * b);
  p.dt_raw = (multi && routed_xdt && !p.rank_passes) ? take(S * De * b) : kNone;   // per-slot dt pre-activations, in T like every expert output
  p.g = take(N * De * b);
  p.op_sorted = multi ? take(S * Dm * b) : kNone;
  // the conv writes its end state beside the old one only when a sequence is cut into runs
  p.conv_tmp = take(seq_len > kConvInPlaceMaxLen ? static_cast<size_t>(n_seq) * De * 3 * 4 : 0);
  const size_t chunk_bytes = scan_chunk_state_bytes(n_seq, seq_len, d->d_inner);
  p.scan_q = take(chunk_bytes);
  p.scan_p = take(chunk_bytes);
  p.rstd = take(N * 4);
  p.rank_offsets = p.rank_passes ? take(K * (E + 1) * 4) : kNone;
  p.rank_tok = p.rank_passes ? take(S * 4) : kNone;
  p.rank_blocks = p.rank_passes ? take(rank_grouping_block_counts_bytes(n_tok, d->n_experts, d->top_k)) : kNone;
  p.total = off;
  return p;
}

// ---------------------------------------------------------------- stage timing
// One event per stage boundary of a call: the stages run back to back on one stream, so a
// stage's begin is the end of the stage before it (event 0 is recorded before the first stage).
constexpr int kProfEvents = ROM_STAGE_COUNT + 1;
struct Profiler {
  int max_calls = 0, n_calls = 0;
  unsigned stage_mask = ~0u;         // bit i: stage i is timed
  hipEvent_t *ev = nullptr;          // [max_calls][kProfEvents]
  int *end_of = nullptr;             // [max_calls][ROM_STAGE_COUNT]: event index of the stage's end, -1 = stage did not run
  int *begin_of = nullptr;           // same, for its begin
} g_prof;

struct StageMark {
  int call = -1, next = 0, last = -1;
  bool on = false;
  StageMark() {
    if (g_prof.ev && g_prof.n_calls < g_prof.max_calls) {
      call = g_prof.n_calls++;
      on = true;
    }
  }
  void begin(int stage, hipStream_t s) {
    if (!on || last >= 0 || !((g_prof.stage_mask >> stage) & 1u)) return;
    last = call * kProfEvents + next++;
    (void)hipEventRecord(g_prof.ev[last], s);
  }
  void end(int stage, hipStream_t s) {
    if (!on) return;
    if (!((g_prof.stage_mask >> stage) & 1u)) {     // not timed: the next timed stage records its own begin
      last = -1;
      return;
    }
    const int e = call * kProfEvents + next++;
    (void)hipEventRecord(g_prof.ev[e], s);
    g_prof.begin_of[call * ROM_STAGE_COUNT + stage] = last;
    g_prof.end_of[call * ROM_STAGE_COUNT + stage] = e;
    last = e;
  }
};

#define ROM_TRY(expr)                      \
  do {                                     \
    if ((expr) != hipSuccess) return ROM_E_HIP; \
  } while (0)

__global__ void add_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) dst[i] += src[i];
}

__global__ void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// dst[r, d] = src[r, d] * scale[d]  (rows of length n_cols; dst may be src)
template <typename T>
__global__ void fold_cols_kernel(const T *src, const float *__restrict__ scale, T *dst, int64_t n_rows,
                                 int n_cols) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= n_rows * n_cols) return;
  dst[i] = from_f32<T>(to_f32(src[i]) * scale[i % n_cols]);
}

// dst[e, 16b + t, d] = src[e, 8b + t, d] * scale[d], dst[e, 16b + 8 + t, d] = src[e, d_ff + 8b + t, d] * scale[d]
// (t < 8; scale may be NULL): gate and up rows of a SwiGLU expert interleaved in blocks of eight
template <typename T>
__global__ void pack_gate_up_kernel(const T *__restrict__ src, const float *__restrict__ scale, T *__restrict__ dst,
                                    int n_experts, int d_ff, int d_model) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int64_t per_expert = static_cast<int64_t>(2) * d_ff * d_model;
  if (i >= n_experts * per_expert) return;
  const int64_t e = i / per_expert, rem = i % per_expert;
  const int r = static_cast<int>(rem / d_model), d = static_cast<int>(rem % d_model);
  const int b = r / 16, t = r % 16;
  const int src_row = t < 8 ? 8 * b + t : d_ff + 8 * b + (t - 8);
  const float v = to_f32(src[e * per_expert + static_cast<int64_t>(src_row) * d_model + d]);
  dst[i] = from_f32<T>(scale ? v * scale[d] : v);
}

// What turns the layer into the pre-norm, skip-connected block: RMSNorm in front (its scale is
// folded into w_in by rom_fold_norm; the router applies it itself), the block input added behind.
struct BlockOpts {
  const float *norm_w;   // f32 [d_model]
  float eps;
};

int route_into(const rom_dims *d, const rom_weights *w, const void *x, int64_t n_tok,
               int32_t *expert_idx, float *gate, int32_t *counts, int32_t *offsets, int32_t *perm,
               int32_t *inv_perm, int32_t *tok_of_pos, int32_t *block_counts, float *logits,
               const BlockOpts *blk, float *rstd, hipStream_t s, StageMark *mark, int32_t *rank_offsets = nullptr,
               int32_t *rank_tok = nullptr, int32_t *rank_blocks = nullptr) {
  if (mark) mark->begin(ROM_STAGE_ROUTE, s);
  ROM_TRY(launch_route_topk(d->dtype, x, w->w_router, w->b_router, n_tok, d->d_model, d->n_experts,
                            d->top_k, d->gate_mode, expert_idx, gate, logits, blk ? blk->norm_w : nullptr,
                            blk ? blk->eps : 0.0f, rstd, s));
  if (mark) mark->end(ROM_STAGE_ROUTE, s);
  if (mark) mark->begin(ROM_STAGE_PERMUTE, s);
  ROM_TRY(launch_permutation(expert_idx, n_tok * d->top_k, d->n_experts, d->top_k, block_counts,
                             counts, offsets, perm, inv_perm, tok_of_pos, s));
  if (rank_offsets)
    ROM_TRY(launch_rank_grouping(expert_idx, n_tok, d->n_experts, d->top_k, rank_blocks, rank_offsets, rank_tok, s));
  if (mark) mark->end(ROM_STAGE_PERMUTE, s);
  return ROM_OK;
}

int forward_impl(const rom_dims *d, const rom_weights *w, const void *x, int64_t B, int64_t L,
                 const float *conv_in, const float *ssm_in, void *out, float *conv_out,
                 float *ssm_out, void *ws, size_t ws_bytes, hipStream_t s, const BlockOpts *blk = nullptr,
                 const void *route_x = nullptr, const BlockOpts *route_blk = nullptr) {
  // route_x / route_blk: the router alone reads route_x under route_blk's norm (the block's backward:
  // the decision of the forward block, which normalises x for itself, while everything else runs on
  // the materialised norm x)
  int rc = check_dims(d);
  if (rc != ROM_OK) return rc;
  rc = check_weights(d, w);
  if (rc != ROM_OK) return rc;
  if (blk && (!blk->norm_w || !aligned16(blk->norm_w) || !(blk->eps >= 0.0f))) return ROM_E_INVAL;
  if (B < 0 || L < 0) return ROM_E_INVAL;
  if (B == 0 || L == 0) return ROM_OK;
  if (!x || !out || !ws || x == out) return ROM_E_INVAL;
  if (!aligned16(x) || !aligned16(out) || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return ROM_E_INVAL;
  if (B * L * d->top_k > (1ll << 30) || B > 65535) return ROM_E_UNSUPPORTED;
  const int64_t N = B * L;
  Plan p = make_plan(d, B, L);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;

  char *base = static_cast<char *>(ws);
  auto at = [&](size_t off) { return base + off; };
  const int K = d->top_k, E = d->n_experts, De = d->d_inner, Dm = d->d_model, R = d->dt_rank;
  const bool multi = K > 1, routed_xdt = d->n_experts_xdt > 1;
  const int64_t S = N * K;
  float *gate = reinterpret_cast<float *>(at(p.gate));
  int32_t *offsets = reinterpret_cast<int32_t *>(at(p.offsets));
  int32_t *inv_perm = reinterpret_cast<int32_t *>(at(p.inv_perm));
  int32_t *tok_of_pos = reinterpret_cast<int32_t *>(at(p.tok_of_pos));
  const size_t eb = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;
  const float *rstd = blk ? reinterpret_cast<const float *>(at(p.rstd)) : nullptr;

  StageMark mark;
  rc = route_into(d, w, route_x ? route_x : x, N, reinterpret_cast<int32_t *>(at(p.expert_idx)), gate,
                  reinterpret_cast<int32_t *>(at(p.counts)), offsets, reinterpret_cast<int32_t *>(at(p.perm)),
                  inv_perm, tok_of_pos, reinterpret_cast<int32_t *>(at(p.block_counts)),
                  reinterpret_cast<float *>(at(p.logits)), route_blk ? route_blk : blk,
                  reinterpret_cast<float *>(at(p.rstd)), s, &mark,
                  p.rank_passes ? reinterpret_cast<int32_t *>(at(p.rank_offsets)) : nullptr,
                  p.rank_passes ? reinterpret_cast<int32_t *>(at(p.rank_tok)) : nullptr,
                  p.rank_passes ? reinterpret_cast<int32_t *>(at(p.rank_blocks)) : nullptr);
  if (rc != ROM_OK) return rc;

  // the routed GEMMs: expert e's rows are the sorted positions [offsets[e], offsets[e + 1])
  auto routed = [&](GemmArgs &ga) {
    ga.n_groups = E;
    ga.M = S;
    ga.offsets = offsets;
  };
  // pass r of a projection run rank by rank: the N tokens grouped by their r-th expert; rows are
  // gathered from and scattered to token order through the same map
  const bool passes = p.rank_passes;
  auto rank_pass = [&](GemmArgs &ga, int r) {
    ga.n_groups = E;
    ga.M = N;
    ga.offsets = reinterpret_cast<const int32_t *>(at(p.rank_offsets)) + static_cast<size_t>(r) * (E + 1);
    ga.a_rows = reinterpret_cast<const int32_t *>(at(p.rank_tok)) + static_cast<size_t>(r) * N;
    ga.c_rows = ga.a_rows;
  };

  // in / gate projection, Eq. (10)/(11): gather token rows, scatter back to token order (K == 1)
  mark.begin(ROM_STAGE_IN_PROJ, s);
  GemmArgs ga;
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.A = x; ga.lda = Dm; ga.a_rows = tok_of_pos; ga.a_span = N * Dm;
  ga.W = w->w_in; ga.N = 2 * De; ga.K = Dm;
  routed(ga);
  ga.C = multi ? at(p.xz_sorted) : at(p.xz); ga.ldc = 2 * De; ga.c_rows = multi ? nullptr : tok_of_pos;
  // pre-norm block: x @ (W . norm_w)^T scaled by the token's 1/rms is RMSNorm(x) @ W^T
  if (!multi) ga.row_scale = rstd;
  ROM_TRY(launch_grouped_gemm(ga, s));
  if (multi)
    ROM_TRY(launch_slot_sum(eb == 4, eb == 4, at(p.xz_sorted), 2 * De, at(p.xz), 2 * De, inv_perm, N, K, 2 * De,
                            nullptr, 0, rstd, s));
  mark.end(ROM_STAGE_IN_PROJ, s);

  // short conv + SiLU, Eq. (2)
  mark.begin(ROM_STAGE_CONV, s);
  {
    // conv_out may alias conv_in (rom_step): a sequence of up to kConvInPlaceMaxLen steps is one
    // run of one thread, which reads the old state before it writes the new one; longer sequences
    // are cut into runs for different blocks, so the new state goes beside the old one and is
    // copied over
    float *ctmp = reinterpret_cast<float *>(at(p.conv_tmp));
    float *cdst = conv_out;
    const bool beside = conv_out && L > kConvInPlaceMaxLen;
    if (beside) cdst = ctmp;
    ROM_TRY(launch_conv_silu(d->dtype, at(p.xz), 2 * De, w->conv_w, w->conv_b, conv_in, cdst, at(p.u), B, L, De, s));
    if (beside) {
      const int64_t n = B * De * 3;
      hipLaunchKernelGGL(copy_f32_kernel, dim3(static_cast<unsigned>(ceil_div(n, 256))), dim3(256), 0, s, ctmp,
                         conv_out, n);
      ROM_TRY(hipGetLastError());
    }
  }
  mark.end(ROM_STAGE_CONV, s);

  // x projection -> dt_low | B | C
  mark.begin(ROM_STAGE_X_PROJ, s);
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.lda = De; ga.a_span = N * De;
  ga.W = w->w_x; ga.N = R + 32; ga.K = De;
  ga.ldc = R + 32; ga.c_is_f32 = 1;
  ga.k_splits = p.xproj_slices;
  ga.c_split_stride = (routed_xdt ? S : N) * (R + 32);
  float *xdbl = reinterpret_cast<float *>(at(p.xdbl));
  ga.A = at(p.u); ga.C = xdbl;
  if (routed_xdt) {
    ga.a_rows = tok_of_pos;
    routed(ga);
    ga.c_rows = multi ? nullptr : tok_of_pos;
  } else {
    ga.n_groups = 1; ga.M = N;
  }
  ROM_TRY(launch_grouped_gemm(ga, s));
  {
    const bool by_pos = routed_xdt && multi;      // xdbl rows in sorted-slot order, else in token order
    ROM_TRY(launch_split_xdbl(d->dtype, xdbl, ga.k_splits, ga.c_split_stride, by_pos ? inv_perm : nullptr, K, N, R,
                              at(p.dt_low), reinterpret_cast<float *>(at(p.bc)), s));
  }
  mark.end(ROM_STAGE_X_PROJ, s);

  // dt projection + bias + softplus
  mark.begin(ROM_STAGE_DT_PROJ, s);
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.A = at(p.dt_low); ga.lda = R; ga.a_span = N * R;
  ga.W = w->w_dt; ga.N = De; ga.K = R; ga.ldc = De;
  if (passes) {
    // dt[n] = softplus(sum_r W_dt[e_r(n)] dt_low[n] + bias): the sums accumulate in dt (without the
    // bias, so that what is stored in T between the passes is small), the last pass activates
    ga.C = at(p.dt);
    for (int r = 0; r < K; ++r) {
      rank_pass(ga, r);
      ga.residual = r > 0 ? at(p.dt) : nullptr;
      if (r == K - 1) { ga.bias = w->dt_bias; ga.softplus = 1; }
      ROM_TRY(launch_grouped_gemm(ga, s));
    }
  } else if (routed_xdt && multi) {
    ga.a_rows = tok_of_pos;
    routed(ga);
    ga.C = at(p.dt_raw);     // one expert's output per slot, stored in T as in_proj's; summed in fp32 below
    ROM_TRY(launch_grouped_gemm(ga, s));
    ROM_TRY(launch_slot_sum(eb == 4, eb == 4, at(p.dt_raw), De, at(p.dt), De, inv_perm, N, K, De, w->dt_bias, 1,
                            nullptr, s));
  } else {
    ga.C = at(p.dt);
    if (routed_xdt) {
      ga.a_rows = tok_of_pos; ga.c_rows = tok_of_pos;
      routed(ga);
    } else {
      ga.n_groups = 1; ga.M = N;
    }
    ga.bias = w->dt_bias; ga.softplus = 1;
    ROM_TRY(launch_grouped_gemm(ga, s));
  }
  mark.end(ROM_STAGE_DT_PROJ, s);

  // selective scan + D skip + SiLU(z) gate, Eq. (5), (6)
  mark.begin(ROM_STAGE_SCAN, s);
  ROM_TRY(launch_scan_gate(d->dtype, at(p.u), at(p.dt), reinterpret_cast<const float *>(at(p.bc)),
                           at(p.xz) + static_cast<size_t>(De) * eb, 2 * De, w->A_log, w->D, ssm_in, ssm_out, at(p.g), B,
                           L, De, reinterpret_cast<float *>(at(p.scan_q)), reinterpret_cast<float *>(at(p.scan_p)), s));
  mark.end(ROM_STAGE_SCAN, s);

  // out projection, Eq. (13), and the gate-weighted combine, Eq. (12)
  mark.begin(ROM_STAGE_OUT_PROJ, s);
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.A = at(p.g); ga.lda = De; ga.a_rows = tok_of_pos; ga.a_span = N * De;
  ga.W = w->w_out; ga.N = Dm; ga.K = De;
  routed(ga);
  if (multi) {
    ga.C = at(p.op_sorted); ga.ldc = Dm;
    ROM_TRY(launch_grouped_gemm(ga, s));
    mark.end(ROM_STAGE_OUT_PROJ, s);
    mark.begin(ROM_STAGE_COMBINE, s);
    ROM_TRY(launch_combine(d->dtype, at(p.op_sorted), inv_perm, gate, out, N, K, Dm, blk ? x : nullptr, s));
    mark.end(ROM_STAGE_COMBINE, s);
  } else {
    ga.C = out; ga.ldc = Dm; ga.c_rows = tok_of_pos; ga.row_scale = gate;   // gate[n*1 + 0]
    if (blk) ga.residual = x;                                               // skip connection
    ROM_TRY(launch_grouped_gemm(ga, s));
    mark.end(ROM_STAGE_OUT_PROJ, s);
  }
  return ROM_OK;
}

// ---------------------------------------------------------------- FFN-MoE (Eq. (14), (15))
struct FfnPlan {
  size_t total, tok_of_pos, rstd, h, a, op_sorted;
};

int check_ffn(const rom_dims *d, int32_t d_ff) {
  const int rc = check_dims(d);
  if (rc != ROM_OK) return rc;
  if (d_ff <= 0) return ROM_E_INVAL;
  if (d_ff % 16 != 0) return ROM_E_UNSUPPORTED;
  return ROM_OK;
}

FfnPlan make_ffn_plan(const rom_dims *d, int32_t d_ff, int64_t n_tok) {
  FfnPlan p;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  };
  const size_t S = static_cast<size_t>(n_tok) * d->top_k, b = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;
  p.tok_of_pos = take(S * 4);
  p.rstd = take(S * 4);
  // gate | up pre-activations: only the plain FMA kernel (fp32, or operands beyond the MFMA
  // kernels' 32-bit element offsets) writes them out; the MFMA kernels apply SwiGLU themselves
  const bool fused = d->dtype == ROM_DTYPE_BF16 && static_cast<int64_t>(n_tok) * d->d_model < (1ll << 32) &&
                     static_cast<int64_t>(2) * d_ff * d->d_model < (1ll << 32);
  p.h = fused ? kNone : take(S * 2 * d_ff * b);
  p.a = take(S * d_ff * b);
  p.op_sorted = d->top_k > 1 ? take(S * d->d_model * b) : kNone;
  p.total = off;
  return p;
}

// ---------------------------------------------------------------- backward pass
struct BwdPlan {              // byte offsets behind the forward plan
  size_t total, fwd_out, wt_out, wt_dt, wt_x, wt_in, dg_raw, d_gate, d_logits, d_pre, d_u_scan, d_xz, ckpt, bc_part,
      d_bc, d_dt_low, d_xdbl, d_u_x, dx_in, conv_part, router_part;
  // top-K: per-position (sorted slot) staging of the routed input gradients, summed over a token's K
  // slots afterwards like the forward's per-slot outputs: T [S, d_model] (gate-scaled d_out, then
  // d x), T [S, d_inner] (d g, then d u), f32 [S, dt_rank] (d dt_low)
  size_t pos_dm, pos_de, pos_r;
};

BwdPlan make_bwd_plan(const rom_dims *d, int64_t n_seq, int64_t seq_len) {
  BwdPlan p;
  size_t off = make_plan(d, n_seq, seq_len).total;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  };
  const size_t N = static_cast<size_t>(n_seq) * seq_len, E = d->n_experts, Ex = d->n_experts_xdt;
  const size_t b = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;
  const size_t De = d->d_inner, Dm = d->d_model, R = d->dt_rank;
  const size_t K = d->top_k, S = N * K;
  p.fwd_out = take(N * Dm * b);
  p.wt_out = take(E * Dm * De * b);
  p.wt_dt = take(Ex * De * R * b);
  p.wt_x = take(Ex * (R + 32) * De * b);
  p.wt_in = take(E * 2 * De * Dm * b);
  p.dg_raw = take(N * De * b);
  p.d_gate = take(S * 4);
  p.d_logits = take(N * E * 4);
  p.d_pre = take(N * De * b);
  p.d_u_scan = take(N * De * b);
  p.d_xz = take(N * 2 * De * b);
  p.ckpt = take(scan_bwd_ckpt_bytes(n_seq, seq_len, d->d_inner));
  p.bc_part = take(scan_bwd_part_bytes(static_cast<int64_t>(N), d->d_inner));
  p.d_bc = take(N * 32 * 4);
  p.d_dt_low = take(N * R * 4);
  p.d_xdbl = take(N * (R + 32) * b);
  p.d_u_x = take(N * De * b);
  p.dx_in = take(N * Dm * b);
  p.conv_part = take(conv_bwd_partial_bytes(n_seq, seq_len, d->d_inner));
  p.router_part = take(router_bwd_partial_bytes(static_cast<int64_t>(N), d->d_model, d->n_experts));
  p.pos_dm = K > 1 ? take(S * Dm * b) : kNone;
  p.pos_de = K > 1 ? take(S * De * b) : kNone;
  p.pos_r = (K > 1 && Ex > 1) ? take(S * R * 4) : kNone;
  p.total = off;
  return p;
}

// device address of `scratch` on the current device, looked up once per device
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch_for_current_device(void **out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ROM_E_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return ROM_E_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return ROM_OK;
}

// ---------------------------------------------------------------- the frame of the Mamba2 / Gated DeltaNet variants
// What RoM on the two "streamlined" layers shares (Sec. 5.2): router and grouping, ONE routed input
// projection whose rows come back in token order, a conv + SiLU over a column range of it, the layer's
// own sequence kernels, and the routed, gate-weighted output projection.
struct VariantFrame {
  int dtype, gate_mode, n_experts, top_k, d_model;
  int d_proj;                  // columns of the input projection
  int conv_col, d_conv_ch;     // the conv reads columns [conv_col, conv_col + d_conv_ch) of it
  int d_y;                     // columns of the output projection's input
  const void *w_router;
  const float *b_router;
  const void *w_in;
  const float *conv_w, *conv_b;
  const void *w_out;
  // byte offsets inside the workspace
  size_t expert_idx, gate, counts, offsets, perm, inv_perm, tok_of_pos, block_counts, logits;
  size_t proj, proj_sorted, conv_dst, y, op_sorted, conv_tmp;
  // pre-norm residual block (out = x + layer(RMSNorm(x))): the norm's scale (w_in is then the folded weight) or NULL
  const float *pre_norm_w;
  float pre_norm_eps;
  size_t rstd;                 // f32 [N]
};

// argument checks both variants share (after their own dims / weights checks)
int check_variant_call(const void *x, const void *out, const void *ws, int64_t B, int64_t L, int top_k, float eps,
                       const float *conv_in, const float *ssm_in, const float *conv_out, const float *ssm_out) {
  if (!(eps >= 0.0f)) return ROM_E_INVAL;
  if (!x || !out || !ws || x == out) return ROM_E_INVAL;
  if (!aligned16(x) || !aligned16(out) || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return ROM_E_INVAL;
  if (B * L * top_k > (1ll << 30) || B > 65535) return ROM_E_UNSUPPORTED;
  const float *states[] = {conv_in, ssm_in, conv_out, ssm_out};
  for (const float *ptr : states)
    if (ptr && !aligned16(ptr)) return ROM_E_INVAL;
  // a sequence longer than one conv run / one chunk is worked on by several workgroups: they would
  // read the old state while another writes the new one
  if (L > kConvInPlaceMaxLen && ((conv_in && conv_in == conv_out) || (ssm_in && ssm_in == ssm_out))) return ROM_E_INVAL;
  return ROM_OK;
}

// seq(mark): launches the layer's own kernels between the conv and the output projection (they read the
// projection and the conv output, and leave the output projection's input at f.y); returns a ROM_* code.
template <typename SeqFn>
int run_variant(const VariantFrame &f, const void *x, int64_t B, int64_t L, const float *conv_in, float *conv_out,
                void *out, char *base, hipStream_t s, SeqFn &&seq) {
  auto at = [&](size_t off) { return base + off; };
  const int64_t N = B * L, S = N * f.top_k;
  const bool multi = f.top_k > 1;
  float *gate = reinterpret_cast<float *>(at(f.gate));
  int32_t *offsets = reinterpret_cast<int32_t *>(at(f.offsets));
  int32_t *inv_perm = reinterpret_cast<int32_t *>(at(f.inv_perm));
  int32_t *tok_of_pos = reinterpret_cast<int32_t *>(at(f.tok_of_pos));

  // the router and the grouping are the Mamba layer's
  rom_dims rd;
  memset(&rd, 0, sizeof(rd));
  rd.d_model = f.d_model; rd.d_inner = f.d_y; rd.n_experts = f.n_experts; rd.top_k = f.top_k;
  rd.n_experts_xdt = f.n_experts; rd.dtype = f.dtype; rd.gate_mode = f.gate_mode;
  rom_weights rw;
  memset(&rw, 0, sizeof(rw));
  rw.w_router = f.w_router; rw.b_router = f.b_router;
  StageMark mark;
  BlockOpts blk;
  blk.norm_w = f.pre_norm_w;
  blk.eps = f.pre_norm_eps;
  const bool block = f.pre_norm_w != nullptr;
  float *rstd = block ? reinterpret_cast<float *>(at(f.rstd)) : nullptr;
  int rc = route_into(&rd, &rw, x, N, reinterpret_cast<int32_t *>(at(f.expert_idx)), gate,
                      reinterpret_cast<int32_t *>(at(f.counts)), offsets, reinterpret_cast<int32_t *>(at(f.perm)), inv_perm,
                      tok_of_pos, reinterpret_cast<int32_t *>(at(f.block_counts)), reinterpret_cast<float *>(at(f.logits)),
                      block ? &blk : nullptr, rstd, s, &mark);
  if (rc != ROM_OK) return rc;

  // input projection: one routed GEMM, rows back in token order (K > 1: per-slot rows, then their sum)
  mark.begin(ROM_STAGE_IN_PROJ, s);
  GemmArgs ga;
  memset(&ga, 0, sizeof(ga));
  ga.dtype = f.dtype;
  ga.A = x; ga.lda = f.d_model; ga.a_rows = tok_of_pos; ga.a_span = N * f.d_model;
  ga.W = f.w_in; ga.N = f.d_proj; ga.K = f.d_model;
  ga.n_groups = f.n_experts; ga.M = S; ga.offsets = offsets;
  ga.C = multi ? at(f.proj_sorted) : at(f.proj); ga.ldc = f.d_proj; ga.c_rows = multi ? nullptr : tok_of_pos;
  // pre-norm block: x @ (W . norm_w)^T scaled by the token's 1/rms is RMSNorm(x) @ W^T
  if (!multi) ga.row_scale = rstd;
  ROM_TRY(launch_grouped_gemm(ga, s));
  if (multi)
    ROM_TRY(launch_slot_sum(0, 0, at(f.proj_sorted), f.d_proj, at(f.proj), f.d_proj, inv_perm, N, f.top_k, f.d_proj, nullptr, 0,
                            rstd, s));
  mark.end(ROM_STAGE_IN_PROJ, s);

  // short conv + SiLU, read in place from the projection's output
  mark.begin(ROM_STAGE_CONV, s);
  {
    float *ctmp = reinterpret_cast<float *>(at(f.conv_tmp));
    const bool beside = conv_out && L > kConvInPlaceMaxLen;
    ROM_TRY(launch_conv_silu(f.dtype, at(f.proj) + static_cast<size_t>(f.conv_col) * 2, f.d_proj, f.conv_w, f.conv_b, conv_in,
                             beside ? ctmp : conv_out, at(f.conv_dst), B, L, f.d_conv_ch, s));
    if (beside) {
      const int64_t n = B * f.d_conv_ch * 3;
      hipLaunchKernelGGL(copy_f32_kernel, dim3(static_cast<unsigned>(ceil_div(n, 256))), dim3(256), 0, s, ctmp, conv_out, n);
      ROM_TRY(hipGetLastError());
    }
  }
  mark.end(ROM_STAGE_CONV, s);

  rc = seq(mark);
  if (rc != ROM_OK) return rc;

  // output projection and the gate-weighted combine
  mark.begin(ROM_STAGE_OUT_PROJ, s);
  memset(&ga, 0, sizeof(ga));
  ga.dtype = f.dtype;
  ga.A = at(f.y); ga.lda = f.d_y; ga.a_rows = tok_of_pos; ga.a_span = N * f.d_y;
  ga.W = f.w_out; ga.N = f.d_model; ga.K = f.d_y;
  ga.n_groups = f.n_experts; ga.M = S; ga.offsets = offsets;
  if (multi) {
    ga.C = at(f.op_sorted); ga.ldc = f.d_model;
    ROM_TRY(launch_grouped_gemm(ga, s));
    mark.end(ROM_STAGE_OUT_PROJ, s);
    mark.begin(ROM_STAGE_COMBINE, s);
    ROM_TRY(launch_combine(f.dtype, at(f.op_sorted), inv_perm, gate, out, N, f.top_k, f.d_model, block ? x : nullptr, s));
    mark.end(ROM_STAGE_COMBINE, s);
  } else {
    ga.C = out; ga.ldc = f.d_model; ga.c_rows = tok_of_pos; ga.row_scale = gate;
    if (block) ga.residual = x;                                             // skip connection
    ROM_TRY(launch_grouped_gemm(ga, s));
    mark.end(ROM_STAGE_OUT_PROJ, s);
  }
  return ROM_OK;
}

}  // namespace
}  // namespace rom

using namespace rom;

extern "C" {

size_t rom_workspace_bytes(const rom_dims *dims, int64_t B, int64_t L) {
  if (check_dims(dims) != ROM_OK || B < 0 || L < 0) return 0;
  return make_plan(dims, B > 0 ? B : 1, L > 0 ? L : 1).total;
}

size_t rom_route_workspace_bytes(const rom_dims *dims, int64_t N) {
  if (check_dims(dims) != ROM_OK || N < 0) return 0;
  return make_plan(dims, N > 0 ? N : 1, 1).logits;
}

int rom_workspace_layout(const rom_dims *dims, int64_t B, int64_t L, rom_ws_layout *layout) {
  const int rc = check_dims(dims);
  if (rc != ROM_OK) return rc;
  if (!layout || B < 0 || L < 0) return ROM_E_INVAL;
  Plan p = make_plan(dims, B > 0 ? B : 1, L > 0 ? L : 1);
  layout->total_bytes = rom_workspace_bytes(dims, B, L);
  layout->expert_idx = p.expert_idx;
  layout->gate = p.gate;
  layout->counts = p.counts;
  layout->offsets = p.offsets;
  layout->perm = p.perm;
  layout->inv_perm = p.inv_perm;
  layout->logits = p.logits;
  layout->xz = p.xz;
  layout->u = p.u;
  layout->dt_low = p.dt_low;
  layout->bc = p.bc;
  layout->dt = p.dt;
  layout->g = p.g;
  return ROM_OK;
}

int rom_route(const rom_dims *dims, const rom_weights *w, const void *x, int64_t N,
              int32_t *expert_idx, float *gate, int32_t *counts, int32_t *offsets, int32_t *perm,
              int32_t *inv_perm, float *logits, void *ws, size_t ws_bytes, void *hip_stream) {
  int rc = check_dims(dims);
  if (rc != ROM_OK) return rc;
  if (!w || !w->w_router || !aligned16(w->w_router)) return ROM_E_INVAL;
  if (N < 0) return ROM_E_INVAL;
  if (N == 0) return ROM_OK;
  if (!x || !aligned16(x) || !expert_idx || !gate || !counts || !offsets || !perm || !inv_perm || !ws)
    return ROM_E_INVAL;
  if ((reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return ROM_E_INVAL;
  if (N * dims->top_k > (1ll << 30)) return ROM_E_UNSUPPORTED;
  // only the row map and the per-block histograms live in the workspace: the plan's regions up
  // to the logits (the routing arrays themselves are the caller's)
  Plan p = make_plan(dims, N, 1);
  if (ws_bytes < p.logits) return ROM_E_WORKSPACE;
  char *base = static_cast<char *>(ws);
  return route_into(dims, w, x, N, expert_idx, gate, counts, offsets, perm, inv_perm,
                    reinterpret_cast<int32_t *>(base + p.tok_of_pos),
                    reinterpret_cast<int32_t *>(base + p.block_counts), logits, nullptr, nullptr,
                    static_cast<hipStream_t>(hip_stream), nullptr);
}

int rom_balance_stats(const rom_dims *dims, const float *logits, const int32_t *counts, int64_t N,
                      float alpha, float *frac, float *mean_prob, float *loss, void *ws, size_t ws_bytes,
                      void *hip_stream) {
  int rc = check_dims(dims);
  if (rc != ROM_OK) return rc;
  if (N <= 0 || !logits || !counts || !frac || !mean_prob || !loss || !ws) return ROM_E_INVAL;
  if ((reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return ROM_E_INVAL;
  if (N * dims->top_k > (1ll << 30)) return ROM_E_UNSUPPORTED;
  // the scratch lies in front of every region whose size depends on how N splits into B x L
  Plan p = make_plan(dims, N, 1);
  if (ws_bytes < p.balance_part + balance_scratch_bytes(dims->n_experts)) return ROM_E_WORKSPACE;
  float *partial = reinterpret_cast<float *>(static_cast<char *>(ws) + p.balance_part);
  return launch_balance_stats(logits, counts, N, dims->n_experts, dims->top_k, alpha, partial, frac,
                              mean_prob, loss, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? ROM_OK
             : ROM_E_HIP;
}

int rom_layer_forward(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B, int64_t L,
                      const float *conv_state_in, const float *ssm_state_in, void *out,
                      float *conv_state_out, float *ssm_state_out, void *ws, size_t ws_bytes,
                      void *hip_stream) {
  return forward_impl(dims, w, x, B, L, conv_state_in, ssm_state_in, out, conv_state_out,
                      ssm_state_out, ws, ws_bytes, static_cast<hipStream_t>(hip_stream));
}

int rom_fold_norm(const rom_dims *dims, const void *w_in, const float *norm_weight, void *w_in_folded,
                  void *hip_stream) {
  int rc = check_dims(dims);
  if (rc != ROM_OK) return rc;
  if (!w_in || !norm_weight || !w_in_folded) return ROM_E_INVAL;
  const int64_t rows = static_cast<int64_t>(dims->n_experts) * 2 * dims->d_inner;
  const int64_t n = rows * dims->d_model;
  const dim3 grid(static_cast<unsigned>(ceil_div(n, 256)));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (dims->dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(fold_cols_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(w_in),
                       norm_weight, static_cast<bf16_t *>(w_in_folded), rows, dims->d_model);
  else
    hipLaunchKernelGGL(fold_cols_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(w_in),
                       norm_weight, static_cast<float *>(w_in_folded), rows, dims->d_model);
  return hipGetLastError() == hipSuccess ? ROM_OK : ROM_E_HIP;
}

int rom_fold_norm_rows(int dtype, const void *w, const float *norm_weight, void *w_folded, int64_t n_rows, int32_t d_model,
                       void *hip_stream) {
  if (dtype != ROM_DTYPE_F32 && dtype != ROM_DTYPE_BF16) return ROM_E_INVAL;
  if (!w || !norm_weight || !w_folded || n_rows < 0 || d_model <= 0) return ROM_E_INVAL;
  if (n_rows == 0) return ROM_OK;
  const int64_t n = n_rows * d_model;
  const dim3 grid(static_cast<unsigned>(ceil_div(n, 256)));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(fold_cols_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(w), norm_weight,
                       static_cast<bf16_t *>(w_folded), n_rows, d_model);
  else
    hipLaunchKernelGGL(fold_cols_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(w), norm_weight,
                       static_cast<float *>(w_folded), n_rows, d_model);
  return hipGetLastError() == hipSuccess ? ROM_OK : ROM_E_HIP;
}

int rom_block_forward(const rom_dims *dims, const rom_weights *w, const float *norm_weight, float eps,
                      const void *x, int64_t B, int64_t L, const float *conv_state_in,
                      const float *ssm_state_in, void *out, float *conv_state_out, float *ssm_state_out,
                      void *ws, size_t ws_bytes, void *hip_stream) {
  const BlockOpts blk = {norm_weight, eps};
  return forward_impl(dims, w, x, B, L, conv_state_in, ssm_state_in, out, conv_state_out, ssm_state_out,
                      ws, ws_bytes, static_cast<hipStream_t>(hip_stream), &blk);
}

int rom_block_step(const rom_dims *dims, const rom_weights *w, const float *norm_weight, float eps,
                   const void *x, int64_t B, float *conv_state, float *ssm_state, void *out, void *ws,
                   size_t ws_bytes, void *hip_stream) {
  if (B > 0 && (!conv_state || !ssm_state)) return ROM_E_INVAL;
  const BlockOpts blk = {norm_weight, eps};
  return forward_impl(dims, w, x, B, 1, conv_state, ssm_state, out, conv_state, ssm_state, ws, ws_bytes,
                      static_cast<hipStream_t>(hip_stream), &blk);
}

int rom_stack_forward(const rom_dims *dims, const rom_block *blocks, int n_layers, float eps,
                      const void *x, int64_t B, int64_t L, const float *conv_state_in,
                      const float *ssm_state_in, void *out, float *conv_state_out, float *ssm_state_out,
                      void *tmp, void *ws, size_t ws_bytes, void *hip_stream) {
  int rc = check_dims(dims);
  if (rc != ROM_OK) return rc;
  if (!blocks || n_layers < 1 || B < 0 || L < 0) return ROM_E_INVAL;
  if (n_layers > 1 && (!tmp || tmp == x || tmp == out || !aligned16(tmp))) return ROM_E_INVAL;
  for (int j = 0; j < n_layers; ++j) {   // refuse the whole call before the first layer is launched
    rc = check_weights(dims, &blocks[j].w);
    if (rc != ROM_OK) return rc;
    if (!blocks[j].norm_weight || !aligned16(blocks[j].norm_weight)) return ROM_E_INVAL;
  }
  if (B == 0 || L == 0) return ROM_OK;
  const size_t conv_per = static_cast<size_t>(B) * dims->d_inner * 3, ssm_per = static_cast<size_t>(B) * dims->d_inner * 16;
  const void *src = x;
  for (int j = 0; j < n_layers; ++j) {
    // the layers write out and tmp in turn, the last one out
    void *dst = ((n_layers - 1 - j) & 1) ? tmp : out;
    const BlockOpts blk = {blocks[j].norm_weight, eps};
    rc = forward_impl(dims, &blocks[j].w, src, B, L, conv_state_in ? conv_state_in + j * conv_per : nullptr,
                      ssm_state_in ? ssm_state_in + j * ssm_per : nullptr, dst,
                      conv_state_out ? conv_state_out + j * conv_per : nullptr,
                      ssm_state_out ? ssm_state_out + j * ssm_per : nullptr, ws, ws_bytes,
                      static_cast<hipStream_t>(hip_stream), &blk);
    if (rc != ROM_OK) return rc;
    src = dst;
  }
  return ROM_OK;
}

size_t rom_ffn_workspace_bytes(const rom_dims *dims, int32_t d_ff, int64_t N) {
  if (check_ffn(dims, d_ff) != ROM_OK || N < 0) return 0;
  return make_ffn_plan(dims, d_ff, N > 0 ? N : 1).total;
}

int rom_ffn_pack_gate_up(const rom_dims *dims, int32_t d_ff, const void *w_gate_up, const float *norm_weight,
                         void *w_packed, void *hip_stream) {
  int rc = check_ffn(dims, d_ff);
  if (rc != ROM_OK) return rc;
  if (!w_gate_up || !w_packed || w_gate_up == w_packed) return ROM_E_INVAL;
  const int64_t n = static_cast<int64_t>(dims->n_experts) * 2 * d_ff * dims->d_model;
  const dim3 grid(static_cast<unsigned>(ceil_div(n, 256)));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (dims->dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(pack_gate_up_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(w_gate_up),
                       norm_weight, static_cast<bf16_t *>(w_packed), dims->n_experts, d_ff, dims->d_model);
  else
    hipLaunchKernelGGL(pack_gate_up_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(w_gate_up),
                       norm_weight, static_cast<float *>(w_packed), dims->n_experts, d_ff, dims->d_model);
  return hipGetLastError() == hipSuccess ? ROM_OK : ROM_E_HIP;
}

int rom_ffn_moe_forward(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w, int pre_norm, float eps,
                        int add_skip, const void *x, int64_t N, const int32_t *offsets, const int32_t *perm,
                        const int32_t *inv_perm, const float *gate, void *out, void *ws, size_t ws_bytes,
                        void *hip_stream) {
  int rc = check_ffn(dims, d_ff);
  if (rc != ROM_OK) return rc;
  if (!w || !w->w_gate_up || !w->w_down || !aligned16(w->w_gate_up) || !aligned16(w->w_down)) return ROM_E_INVAL;
  if (N < 0 || (pre_norm && !(eps >= 0.0f))) return ROM_E_INVAL;
  if (N == 0) return ROM_OK;
  if (!x || !out || x == out || !offsets || !perm || !inv_perm || !gate || !ws) return ROM_E_INVAL;
  if (!aligned16(x) || !aligned16(out) || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return ROM_E_INVAL;
  if (N * dims->top_k > (1ll << 30)) return ROM_E_UNSUPPORTED;
  const FfnPlan p = make_ffn_plan(dims, d_ff, N);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char *base = static_cast<char *>(ws);
  const int K = dims->top_k, E = dims->n_experts, Dm = dims->d_model;
  const int64_t S = N * K;
  int32_t *tok_of_pos = reinterpret_cast<int32_t *>(base + p.tok_of_pos);
  float *rstd = pre_norm ? reinterpret_cast<float *>(base + p.rstd) : nullptr;
  ROM_TRY(launch_ffn_prep(dims->dtype, perm, K, S, x, Dm, eps, tok_of_pos, rstd, s));

  // gate | up projection of every slot by its expert, rows kept in sorted order
  GemmArgs ga;
  memset(&ga, 0, sizeof(ga));
  ga.dtype = dims->dtype;
  ga.A = x; ga.lda = Dm; ga.a_rows = tok_of_pos; ga.a_span = N * Dm;
  ga.W = w->w_gate_up; ga.N = 2 * d_ff; ga.K = Dm;
  ga.offsets = offsets; ga.n_groups = E; ga.M = S;
  ga.row_scale = rstd;                      // pre-norm: the weight's columns carry the norm's scale
  ga.C = base + p.a; ga.ldc = d_ff; ga.swiglu = 1;
  if (grouped_gemm_on_mfma(ga)) {           // SiLU(gate) * up formed in the GEMM's epilogue
    ROM_TRY(launch_grouped_gemm(ga, s));
  } else {
    if (p.h == kNone) return ROM_E_UNSUPPORTED;   // cannot happen for 16-byte aligned, in-range operands
    ga.C = base + p.h; ga.ldc = 2 * d_ff; ga.swiglu = 0;
    ROM_TRY(launch_grouped_gemm(ga, s));
    ROM_TRY(launch_swiglu(dims->dtype, base + p.h, base + p.a, S, d_ff, s));
  }

  // down projection, weighted by the router's R_i and brought back to token order
  memset(&ga, 0, sizeof(ga));
  ga.dtype = dims->dtype;
  ga.A = base + p.a; ga.lda = d_ff; ga.a_span = S * d_ff;
  ga.W = w->w_down; ga.N = Dm; ga.K = d_ff;
  ga.offsets = offsets; ga.n_groups = E; ga.M = S;
  if (K > 1) {
    ga.C = base + p.op_sorted; ga.ldc = Dm;
    ROM_TRY(launch_grouped_gemm(ga, s));
    ROM_TRY(launch_combine(dims->dtype, base + p.op_sorted, inv_perm, gate, out, N, K, Dm, add_skip ? x : nullptr, s));
  } else {
    ga.C = out; ga.ldc = Dm; ga.c_rows = tok_of_pos; ga.row_scale = gate;
    if (add_skip) ga.residual = x;
    ROM_TRY(launch_grouped_gemm(ga, s));
  }
  return ROM_OK;
}

namespace {
// workspace of rom_ffn_moe_backward
struct FfnBwdPlan {
  size_t total, tok_of_pos, xn, rstd, h, a, o, dsc, d_a, d_h, wt_down, wt_gu, d_xin, part;
};
FfnBwdPlan make_ffn_bwd_plan(const rom_dims *d, int32_t d_ff, int64_t n_tok) {
  FfnBwdPlan p;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  };
  const size_t N = static_cast<size_t>(n_tok), S = N * d->top_k, b = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;
  const size_t Dm = d->d_model, Df = d_ff, E = d->n_experts;
  p.tok_of_pos = take(S * 4);
  p.xn = take(N * Dm * b);
  p.rstd = take(N * 4);
  p.h = take(S * 2 * Df * b);
  p.a = take(S * Df * b);
  p.o = take(S * Dm * b);            // the experts' outputs per position, later the input gradient per position
  p.dsc = take(S * Dm * b);
  p.d_a = take(S * Df * b);
  p.d_h = take(S * 2 * Df * b);
  p.wt_down = take(E * Df * Dm * b);     // transposed weights, written only where the GEMM cannot read W contraction-major
  p.wt_gu = take(E * 2 * Df * Dm * b);
  p.d_xin = take(N * Dm * b);
  p.part = take(static_cast<size_t>(rmsnorm_wgrad_parts(n_tok)) * Dm * 4);
  p.total = off;
  return p;
}
}  // namespace

size_t rom_ffn_backward_workspace_bytes(const rom_dims *dims, int32_t d_ff, int64_t N) {
  if (check_ffn(dims, d_ff) != ROM_OK || N < 0) return 0;
  return make_ffn_bwd_plan(dims, d_ff, N > 0 ? N : 1).total;
}

namespace {
// what of the FFN-MoE layer's training step a call runs
enum { kFfnForward = 1, kFfnBackward = 2 };
int ffn_train_impl(int what, const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w, const float *norm_weight, float eps,
                   int add_skip, const void *x, int64_t N, const int32_t *offsets, const int32_t *perm,
                   const int32_t *inv_perm, const float *gate, void *out, const void *d_out, void *d_x, float *d_gate,
                   const rom_ffn_grads *gr, void *ws, size_t ws_bytes, void *hip_stream) {
  const bool fwd = (what & kFfnForward) != 0, bwd = (what & kFfnBackward) != 0;
  int rc = check_ffn(dims, d_ff);
  if (rc != ROM_OK) return rc;
  if (!w || !w->w_gate_up || !w->w_down || !aligned16(w->w_gate_up) || !aligned16(w->w_down)) return ROM_E_INVAL;
  const bool pre_norm = norm_weight != nullptr;
  if (N < 0 || (pre_norm && (!(eps >= 0.0f) || !aligned16(norm_weight)))) return ROM_E_INVAL;
  if (N == 0) return ROM_OK;
  if (!x || !offsets || !perm || !inv_perm || !gate || !ws || !aligned16(x) ||
      (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0)
    return ROM_E_INVAL;
  if (!bwd && (!out || out == x || !aligned16(out))) return ROM_E_INVAL;
  if (bwd && (!d_out || !d_x || d_x == x || d_x == d_out || !d_gate || !gr || !aligned16(d_out) || !aligned16(d_x)))
    return ROM_E_INVAL;
  if (bwd && (!gr->d_w_gate_up || !gr->d_w_down || !aligned16(gr->d_w_gate_up) || !aligned16(gr->d_w_down) ||
              (pre_norm && !gr->d_norm_weight)))
    return ROM_E_INVAL;
  if (N * dims->top_k > (1ll << 24) || dims->d_model % 8 != 0) return ROM_E_UNSUPPORTED;
  const FfnBwdPlan p = make_ffn_bwd_plan(dims, d_ff, N);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char *base = static_cast<char *>(ws);
  auto at = [&](size_t off) { return base + off; };
  const int K = dims->top_k, E = dims->n_experts, Dm = dims->d_model, dt = dims->dtype;
  const int64_t S = N * K;
  const bool f32 = dt == ROM_DTYPE_F32;
  int32_t *tok_of_pos = reinterpret_cast<int32_t *>(at(p.tok_of_pos));
  float *rstd = reinterpret_cast<float *>(at(p.rstd));
  if (fwd) ROM_TRY(launch_ffn_prep(dt, perm, K, S, x, Dm, eps, tok_of_pos, nullptr, s));
  const void *xin = x;
  if (pre_norm) {       // the experts' input, materialised in the activation type
    if (fwd) ROM_TRY(launch_rmsnorm_forward(dt, x, norm_weight, eps, N, Dm, at(p.xn), rstd, s));
    xin = at(p.xn);
  }
  // plain grouped GEMM over the sorted positions; W_fwd != NULL: contract over W's row index instead
  // (W_fwd [E][k_in][n_out] read as it is where the kernel can, else through its transpose in wt)
  auto gemm = [&](const void *A, int64_t lda, const int32_t *a_rows, int64_t a_row_count, const void *W, int n_out, int k_in,
                  void *C, const int32_t *c_rows, const void *W_fwd, void *wt) -> int {
    GemmArgs ga;
    memset(&ga, 0, sizeof(ga));
    ga.dtype = dt;
    ga.A = A; ga.lda = lda; ga.a_rows = a_rows; ga.a_span = a_row_count * lda;
    ga.W = W; ga.N = n_out; ga.K = k_in;
    ga.offsets = offsets; ga.n_groups = E; ga.M = S;
    ga.C = C; ga.ldc = n_out; ga.c_rows = c_rows;
    if (W_fwd) {
      GemmArgs gk = ga;
      gk.W = W_fwd; gk.w_kmajor = 1;
      if (grouped_gemm_takes_kmajor(gk)) {
        ga = gk;
      } else {
        ROM_TRY(launch_transpose(dt, W_fwd, wt, E, k_in, n_out, s));
        ga.W = wt;
      }
    }
    ROM_TRY(launch_grouped_gemm(ga, s));
    return ROM_OK;
  };
#define ROM_RC(expr)               \
  do {                             \
    const int rc_ = (expr);        \
    if (rc_ != ROM_OK) return rc_; \
  } while (0)
  // forward (re)computation: h = W_gu x~ (pre-activations kept this time), a = SiLU(gate) * up, o = W_down a
  if (fwd) {
    ROM_RC(gemm(xin, Dm, tok_of_pos, N, w->w_gate_up, 2 * d_ff, Dm, at(p.h), nullptr, nullptr, nullptr));
    ROM_TRY(launch_swiglu(dt, at(p.h), at(p.a), S, d_ff, s));
    ROM_RC(gemm(at(p.a), d_ff, nullptr, S, w->w_down, Dm, d_ff, at(p.o), nullptr, nullptr, nullptr));
  }
  if (!bwd) {           // the training step's forward: the experts' outputs weighted, brought to token order, skip added
    ROM_TRY(launch_combine(dt, at(p.o), inv_perm, gate, out, N, K, Dm, add_skip ? x : nullptr, s));
    return ROM_OK;
  }
  // d gate of a slot: d_out of its token against its expert's output
  ROM_TRY(launch_gate_backward(dt, d_out, at(p.o), inv_perm, K, S, Dm, d_gate, s));
  // gate-weighted d_out per position; d W_down = sum over an expert's positions of (gate d_out)^T a; d a
  ROM_TRY(launch_scale_rows(dt, d_out, gate, tok_of_pos, perm, S, Dm, at(p.dsc), s));
  ROM_TRY(launch_wgrad(dt, at(p.dsc), Dm, Dm, at(p.a), d_ff, d_ff, nullptr, nullptr, nullptr, offsets, E, S,
                       gr->d_w_down, s));
  ROM_RC(gemm(at(p.dsc), Dm, nullptr, S, nullptr, d_ff, Dm, at(p.d_a), nullptr, w->w_down, at(p.wt_down)));
  // through the SwiGLU; d W_gu (packed row order) and the input gradient per position
  ROM_TRY(launch_swiglu_backward(dt, at(p.h), at(p.d_a), at(p.d_h), S, d_ff, s));
  ROM_TRY(launch_wgrad(dt, at(p.d_h), 2 * d_ff, 2 * d_ff, xin, Dm, Dm, nullptr, tok_of_pos, nullptr, offsets, E, S,
                       gr->d_w_gate_up, s));
  // input gradient: per position, then to token order (top-1: scattered by the GEMM; top-K: the K rows of a token added)
  void *d_xin = (pre_norm || add_skip) ? static_cast<void *>(at(p.d_xin)) : d_x;
  if (K == 1) {
    ROM_RC(gemm(at(p.d_h), 2 * d_ff, nullptr, S, nullptr, Dm, 2 * d_ff, d_xin, tok_of_pos, w->w_gate_up, at(p.wt_gu)));
  } else {
    ROM_RC(gemm(at(p.d_h), 2 * d_ff, nullptr, S, nullptr, Dm, 2 * d_ff, at(p.o), nullptr, w->w_gate_up, at(p.wt_gu)));
    ROM_TRY(launch_slot_sum(f32, f32, at(p.o), Dm, d_xin, Dm, inv_perm, N, K, Dm, nullptr, 0, nullptr, s));
  }
#undef ROM_RC
  if (pre_norm) {
    ROM_TRY(launch_rmsnorm_backward(dt, x, norm_weight, rstd, d_xin, add_skip ? d_out : nullptr, N, Dm, d_x,
                                    reinterpret_cast<float *>(at(p.part)), gr->d_norm_weight, s));
  } else if (add_skip) {
    ROM_TRY(launch_add(dt, d_xin, d_out, d_x, N * Dm, s));
  }
  return ROM_OK;
}
}  // namespace

int rom_ffn_moe_backward(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w, const float *norm_weight, float eps,
                         int add_skip, const void *x, int64_t N, const int32_t *offsets, const int32_t *perm,
                         const int32_t *inv_perm, const float *gate, const void *d_out, void *d_x, float *d_gate,
                         const rom_ffn_grads *gr, void *ws, size_t ws_bytes, void *hip_stream) {
  return ffn_train_impl(kFfnForward | kFfnBackward, dims, d_ff, w, norm_weight, eps, add_skip, x, N, offsets, perm, inv_perm,
                        gate, nullptr, d_out, d_x, d_gate, gr, ws, ws_bytes, hip_stream);
}

int rom_ffn_moe_forward_train(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w, const float *norm_weight,
                              float eps, int add_skip, const void *x, int64_t N, const int32_t *offsets,
                              const int32_t *perm, const int32_t *inv_perm, const float *gate, void *out, void *ws,
                              size_t ws_bytes, void *hip_stream) {
  return ffn_train_impl(kFfnForward, dims, d_ff, w, norm_weight, eps, add_skip, x, N, offsets, perm, inv_perm, gate, out,
                        nullptr, nullptr, nullptr, nullptr, ws, ws_bytes, hip_stream);
}

int rom_ffn_moe_backward_saved(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w, const float *norm_weight,
                               float eps, int add_skip, const void *x, int64_t N, const int32_t *offsets,
                               const int32_t *perm, const int32_t *inv_perm, const float *gate, const void *d_out,
                               void *d_x, float *d_gate, const rom_ffn_grads *gr, void *ws, size_t ws_bytes,
                               void *hip_stream) {
  return ffn_train_impl(kFfnBackward, dims, d_ff, w, norm_weight, eps, add_skip, x, N, offsets, perm, inv_perm, gate, nullptr,
                        d_out, d_x, d_gate, gr, ws, ws_bytes, hip_stream);
}

int rom_hybrid_stack_forward(const rom_dims *dims, int32_t d_ff, const rom_block *blocks,
                             const rom_ffn_weights *ffns, int ffn_pre_norm, int n_layers, float eps,
                             const void *x, int64_t B, int64_t L, const float *conv_state_in,
                             const float *ssm_state_in, void *out, float *conv_state_out,
                             float *ssm_state_out, void *tmp, void *ws, size_t ws_bytes, void *ffn_ws,
                             size_t ffn_ws_bytes, void *hip_stream) {
  int rc = check_ffn(dims, d_ff);
  if (rc != ROM_OK) return rc;
  if (!blocks || !ffns || n_layers < 1 || B < 0 || L < 0) return ROM_E_INVAL;
  int n_ops = 0;                        // RoM blocks plus the FFN-MoE blocks behind some of them
  for (int j = 0; j < n_layers; ++j) {  // refuse the whole call before the first layer is launched
    rc = check_weights(dims, &blocks[j].w);
    if (rc != ROM_OK) return rc;
    if (!blocks[j].norm_weight || !aligned16(blocks[j].norm_weight)) return ROM_E_INVAL;
    n_ops += 1;
    if (ffns[j].w_gate_up) {
      if (!ffns[j].w_down || !aligned16(ffns[j].w_gate_up) || !aligned16(ffns[j].w_down)) return ROM_E_INVAL;
      n_ops += 1;
    }
  }
  if (n_ops > 1 && (!tmp || tmp == x || tmp == out || !aligned16(tmp))) return ROM_E_INVAL;
  if (B == 0 || L == 0) return ROM_OK;
  if (!ws || (n_ops > n_layers && (!ffn_ws || ffn_ws == ws))) return ROM_E_INVAL;
  const int64_t N = B * L;
  const Plan p = make_plan(dims, B, L);
  if (n_ops > n_layers && ffn_ws_bytes < make_ffn_plan(dims, d_ff, N).total) return ROM_E_WORKSPACE;
  const size_t conv_per = static_cast<size_t>(B) * dims->d_inner * 3, ssm_per = static_cast<size_t>(B) * dims->d_inner * 16;
  char *base = static_cast<char *>(ws);
  const void *src = x;
  int op = 0;
  auto next_dst = [&]() {               // the blocks write out and tmp in turn, the last one out
    void *dst = ((n_ops - 1 - op) & 1) ? tmp : out;
    ++op;
    return dst;
  };
  for (int j = 0; j < n_layers; ++j) {
    void *dst = next_dst();
    const BlockOpts blk = {blocks[j].norm_weight, eps};
    rc = forward_impl(dims, &blocks[j].w, src, B, L, conv_state_in ? conv_state_in + j * conv_per : nullptr,
                      ssm_state_in ? ssm_state_in + j * ssm_per : nullptr, dst,
                      conv_state_out ? conv_state_out + j * conv_per : nullptr,
                      ssm_state_out ? ssm_state_out + j * ssm_per : nullptr, ws, ws_bytes,
                      static_cast<hipStream_t>(hip_stream), &blk);
    if (rc != ROM_OK) return rc;
    src = dst;
    if (ffns[j].w_gate_up) {
      // the grouping the RoM block has just left in its workspace drives the FFN-MoE block
      dst = next_dst();
      rc = rom_ffn_moe_forward(dims, d_ff, &ffns[j], ffn_pre_norm, eps, 1, src, N,
                               reinterpret_cast<const int32_t *>(base + p.offsets),
                               reinterpret_cast<const int32_t *>(base + p.perm),
                               reinterpret_cast<const int32_t *>(base + p.inv_perm),
                               reinterpret_cast<const float *>(base + p.gate), dst, ffn_ws, ffn_ws_bytes, hip_stream);
      if (rc != ROM_OK) return rc;
      src = dst;
    }
  }
  return ROM_OK;
}

int rom_stack_step(const rom_dims *dims, const rom_block *blocks, int n_layers, float eps, const void *x,
                   int64_t B, float *conv_state, float *ssm_state, void *out, void *tmp, void *ws,
                   size_t ws_bytes, void *hip_stream) {
  if (B > 0 && (!conv_state || !ssm_state)) return ROM_E_INVAL;
  return rom_stack_forward(dims, blocks, n_layers, eps, x, B, 1, conv_state, ssm_state, out, conv_state,
                           ssm_state, tmp, ws, ws_bytes, hip_stream);
}

int rom_step(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B, float *conv_state,
             float *ssm_state, void *out, void *ws, size_t ws_bytes, void *hip_stream) {
  if (B > 0 && (!conv_state || !ssm_state)) return ROM_E_INVAL;
  return forward_impl(dims, w, x, B, 1, conv_state, ssm_state, out, conv_state, ssm_state, ws, ws_bytes,
                      static_cast<hipStream_t>(hip_stream));
}

int rom_step_static(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B, float *conv_state,
                    float *ssm_state, void *out, void *hip_stream) {
  const int rc = check_dims(dims);
  if (rc != ROM_OK) return rc;
  if (B < 0) return ROM_E_INVAL;
  if (B > 0 && (!conv_state || !ssm_state)) return ROM_E_INVAL;
  if (B > 65535) return ROM_E_UNSUPPORTED;
  if (B > 0 && make_plan(dims, B, 1).total > kStaticScratchBytes) return ROM_E_STATIC_LIMIT;
  void *ws = nullptr;
  if (B > 0) {
    const int src = static_scratch_for_current_device(&ws);
    if (src != ROM_OK) return src;
  }
  // nothing in the step's workspace has to start at zero: every region is written before it is read
  return forward_impl(dims, w, x, B, 1, conv_state, ssm_state, out, conv_state, ssm_state, ws, kStaticScratchBytes,
                      static_cast<hipStream_t>(hip_stream));
}

// ---------------------------------------------------------------- RoM on a Mamba2 layer (Sec. 5.2, Table 3)
namespace {
struct Mamba2Plan {           // byte offsets inside the workspace
  size_t total;
  size_t expert_idx, gate, counts, offsets, perm, inv_perm, tok_of_pos, block_counts, logits;
  size_t zxbcdt, zx_sorted, xbc, yz, g, op_sorted, carry, conv_tmp, rstd;
};

int check_mamba2_dims(const rom_mamba2_dims *d) {
  if (!d) return ROM_E_INVAL;
  if (d->dtype != ROM_DTYPE_F32 && d->dtype != ROM_DTYPE_BF16) return ROM_E_INVAL;
  if (d->gate_mode != 0 && d->gate_mode != 1) return ROM_E_INVAL;
  if (d->d_model <= 0 || d->d_inner <= 0 || d->d_state <= 0 || d->headdim <= 0 || d->n_experts <= 0) return ROM_E_INVAL;
  if (d->top_k < 1 || d->top_k > d->n_experts) return ROM_E_INVAL;
  if (d->d_inner % d->headdim != 0) return ROM_E_INVAL;
  if (d->dtype != ROM_DTYPE_BF16 || d->d_conv != 4 || !ssd_supported(d->d_state, d->headdim)) return ROM_E_UNSUPPORTED;
  if (d->n_experts > 64 || d->top_k > 8) return ROM_E_UNSUPPORTED;
  if (d->d_inner % 512 != 0 || d->d_model % 8 != 0) return ROM_E_UNSUPPORTED;
  return ROM_OK;
}

Mamba2Plan make_mamba2_plan(const rom_mamba2_dims *d, int64_t n_seq, int64_t seq_len) {
  Mamba2Plan p;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  };
  const size_t N = static_cast<size_t>(n_seq * seq_len), K = d->top_k, S = N * K, E = d->n_experts;
  const size_t De = d->d_inner, Dm = d->d_model, Ns = d->d_state, H = De / d->headdim;
  const size_t Dp = 2 * De + 2 * Ns + H, Dc = De + 2 * Ns;
  p.expert_idx = take(S * 4);
  p.gate = take(S * 4);
  p.counts = take(E * 4);
  p.offsets = take((E + 1) * 4);
  p.perm = take(S * 4);
  p.inv_perm = take(S * 4);
  p.tok_of_pos = take(S * 4);
  p.block_counts = take(static_cast<size_t>(route_blocks(static_cast<int64_t>(S))) * E * 4);
  p.logits = take(N * E * 4);
  p.zxbcdt = take(N * Dp * 2);
  p.zx_sorted = K > 1 ? take(S * Dp * 2) : kNone;
  p.xbc = take(N * Dc * 2);
  p.yz = take(N * De * 2);
  p.g = take(N * De * 2);
  p.op_sorted = K > 1 ? take(S * Dm * 2) : kNone;
  p.carry = take(ssd_carry_bytes(n_seq, seq_len, static_cast<int>(H), d->d_state));
  // the conv writes its end state beside the old one when a sequence is cut into runs
  p.conv_tmp = take(seq_len > kConvInPlaceMaxLen ? static_cast<size_t>(n_seq) * Dc * 3 * 4 : 0);
  p.rstd = take(N * 4);
  p.total = off;
  return p;
}
}  // namespace

size_t rom_mamba2_workspace_bytes(const rom_mamba2_dims *dims, int64_t B, int64_t L) {
  if (check_mamba2_dims(dims) != ROM_OK || B < 0 || L < 0) return 0;
  return make_mamba2_plan(dims, B > 0 ? B : 1, L > 0 ? L : 1).total;
}

int rom_mamba2_workspace_layout(const rom_mamba2_dims *dims, int64_t B, int64_t L, rom_mamba2_ws_layout *layout) {
  const int rc = check_mamba2_dims(dims);
  if (rc != ROM_OK) return rc;
  if (!layout || B < 0 || L < 0) return ROM_E_INVAL;
  const Mamba2Plan p = make_mamba2_plan(dims, B > 0 ? B : 1, L > 0 ? L : 1);
  layout->total_bytes = p.total;
  layout->expert_idx = p.expert_idx;
  layout->gate = p.gate;
  layout->counts = p.counts;
  layout->offsets = p.offsets;
  layout->perm = p.perm;
  layout->inv_perm = p.inv_perm;
  layout->logits = p.logits;
  layout->zxbcdt = p.zxbcdt;
  layout->xbc = p.xbc;
  layout->yz = p.yz;
  layout->g = p.g;
  return ROM_OK;
}

namespace {
int mamba2_impl(const rom_mamba2_dims *d, const rom_mamba2_weights *w, const float *pre_norm_w, float pre_norm_eps,
                const void *x, int64_t B, int64_t L, float eps, const float *conv_in, const float *ssm_in, void *out,
                float *conv_out, float *ssm_out, void *ws, size_t ws_bytes, void *hip_stream);
}

int rom_mamba2_forward(const rom_mamba2_dims *d, const rom_mamba2_weights *w, const void *x, int64_t B, int64_t L,
                       float eps, const float *conv_in, const float *ssm_in, void *out, float *conv_out, float *ssm_out,
                       void *ws, size_t ws_bytes, void *hip_stream) {
  return mamba2_impl(d, w, nullptr, 0.0f, x, B, L, eps, conv_in, ssm_in, out, conv_out, ssm_out, ws, ws_bytes, hip_stream);
}

int rom_mamba2_block_forward(const rom_mamba2_dims *d, const rom_mamba2_weights *w, const float *norm_weight,
                             float norm_eps, const void *x, int64_t B, int64_t L, float eps, const float *conv_in,
                             const float *ssm_in, void *out, float *conv_out, float *ssm_out, void *ws, size_t ws_bytes,
                             void *hip_stream) {
  if (!norm_weight || !aligned16(norm_weight) || !(norm_eps >= 0.0f) || out == x) return ROM_E_INVAL;
  return mamba2_impl(d, w, norm_weight, norm_eps, x, B, L, eps, conv_in, ssm_in, out, conv_out, ssm_out, ws, ws_bytes,
                     hip_stream);
}

namespace {
int mamba2_impl(const rom_mamba2_dims *d, const rom_mamba2_weights *w, const float *pre_norm_w, float pre_norm_eps,
                const void *x, int64_t B, int64_t L, float eps, const float *conv_in, const float *ssm_in, void *out,
                float *conv_out, float *ssm_out, void *ws, size_t ws_bytes, void *hip_stream) {
  int rc = check_mamba2_dims(d);
  if (rc != ROM_OK) return rc;
  if (!w) return ROM_E_INVAL;
  {
    const void *req[] = {w->w_router, w->w_in, w->conv_w, w->dt_bias, w->A_log, w->D, w->norm_w, w->w_out};
    for (const void *ptr : req)
      if (!ptr || !aligned16(ptr)) return ROM_E_INVAL;
    if ((w->b_router && !aligned16(w->b_router)) || (w->conv_b && !aligned16(w->conv_b))) return ROM_E_INVAL;
  }
  if (B < 0 || L < 0) return ROM_E_INVAL;
  if (B == 0 || L == 0) return ROM_OK;
  rc = check_variant_call(x, out, ws, B, L, d->top_k, eps, conv_in, ssm_in, conv_out, ssm_out);
  if (rc != ROM_OK) return rc;
  const Mamba2Plan p = make_mamba2_plan(d, B, L);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char *base = static_cast<char *>(ws);
  const int De = d->d_inner, Ns = d->d_state, H = De / d->headdim, Dp = 2 * De + 2 * Ns + H, Dc = De + 2 * Ns;

  VariantFrame f;
  f.dtype = d->dtype; f.gate_mode = d->gate_mode; f.n_experts = d->n_experts; f.top_k = d->top_k; f.d_model = d->d_model;
  f.d_proj = Dp; f.conv_col = De; f.d_conv_ch = Dc; f.d_y = De;          // z | x | B | C | dt: the conv runs over x | B | C
  f.w_router = w->w_router; f.b_router = w->b_router; f.w_in = w->w_in; f.conv_w = w->conv_w; f.conv_b = w->conv_b;
  f.w_out = w->w_out;
  f.expert_idx = p.expert_idx; f.gate = p.gate; f.counts = p.counts; f.offsets = p.offsets; f.perm = p.perm;
  f.inv_perm = p.inv_perm; f.tok_of_pos = p.tok_of_pos; f.block_counts = p.block_counts; f.logits = p.logits;
  f.proj = p.zxbcdt; f.proj_sorted = p.zx_sorted; f.conv_dst = p.xbc; f.y = p.g; f.op_sorted = p.op_sorted;
  f.conv_tmp = p.conv_tmp;
  f.pre_norm_w = pre_norm_w; f.pre_norm_eps = pre_norm_eps; f.rstd = p.rstd;
  return run_variant(f, x, B, L, conv_in, conv_out, out, base, s, [&](StageMark &mark) {
    // recurrence, D skip, SiLU(z) gate
    mark.begin(ROM_STAGE_SCAN, s);
    ROM_TRY(launch_ssd_scan(base + p.xbc, Dc, 0, De, De + Ns, base + p.zxbcdt, Dp, 2 * De + 2 * Ns, base + p.zxbcdt, Dp,
                            w->dt_bias, w->A_log, w->D, ssm_in, ssm_out, B, L, H, Ns, reinterpret_cast<float *>(base + p.carry),
                            base + p.yz, De, s));
    mark.end(ROM_STAGE_SCAN, s);
    // RMS norm of the gated rows
    mark.begin(ROM_STAGE_DT_PROJ, s);
    ROM_TRY(launch_rms_rows(base + p.yz, w->norm_w, eps, B * L, De, base + p.g, s));
    mark.end(ROM_STAGE_DT_PROJ, s);
    return static_cast<int>(ROM_OK);
  });
}
}  // namespace

int rom_mamba2_step(const rom_mamba2_dims *d, const rom_mamba2_weights *w, const void *x, int64_t B, float eps,
                    float *conv_state, float *ssm_state, void *out, void *ws, size_t ws_bytes, void *hip_stream) {
  if (B > 0 && (!conv_state || !ssm_state)) return ROM_E_INVAL;
  return rom_mamba2_forward(d, w, x, B, 1, eps, conv_state, ssm_state, out, conv_state, ssm_state, ws, ws_bytes,
                            hip_stream);
}

// ---------------------------------------------------------------- RoM on a Gated DeltaNet layer (Sec. 5.2, Table 3)
namespace {
struct GdnPlan {              // byte offsets inside the workspace
  size_t total;
  size_t expert_idx, gate, counts, offsets, perm, inv_perm, tok_of_pos, block_counts, logits;
  size_t proj, proj_sorted, qkv, y, op_sorted, conv_tmp, carry, rstd;
};

int check_gdn_dims(const rom_gdn_dims *d) {
  if (!d) return ROM_E_INVAL;
  if (d->dtype != ROM_DTYPE_F32 && d->dtype != ROM_DTYPE_BF16) return ROM_E_INVAL;
  if (d->gate_mode != 0 && d->gate_mode != 1) return ROM_E_INVAL;
  if (d->d_model <= 0 || d->n_heads <= 0 || d->d_k <= 0 || d->d_v <= 0 || d->n_experts <= 0) return ROM_E_INVAL;
  if (d->top_k < 1 || d->top_k > d->n_experts) return ROM_E_INVAL;
  if (d->dtype != ROM_DTYPE_BF16 || d->d_conv != 4 || !gdn_supported(d->d_k, d->d_v)) return ROM_E_UNSUPPORTED;
  if (d->n_experts > 64 || d->top_k > 8) return ROM_E_UNSUPPORTED;
  if (d->n_heads % 4 != 0 || d->d_model % 8 != 0 || d->n_heads > 16384) return ROM_E_UNSUPPORTED;
  return ROM_OK;
}

GdnPlan make_gdn_plan(const rom_gdn_dims *d, int64_t n_seq, int64_t seq_len) {
  GdnPlan p;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  };
  const size_t N = static_cast<size_t>(n_seq * seq_len), K = d->top_k, S = N * K, E = d->n_experts;
  const size_t H = d->n_heads, Dk = H * d->d_k, Dv = H * d->d_v, Dm = d->d_model;
  const size_t Dp = 2 * Dv + 2 * Dk + 2 * H, Dc = 2 * Dk + Dv;
  p.expert_idx = take(S * 4);
  p.gate = take(S * 4);
  p.counts = take(E * 4);
  p.offsets = take((E + 1) * 4);
  p.perm = take(S * 4);
  p.inv_perm = take(S * 4);
  p.tok_of_pos = take(S * 4);
  p.block_counts = take(static_cast<size_t>(route_blocks(static_cast<int64_t>(S))) * E * 4);
  p.logits = take(N * E * 4);
  p.proj = take(N * Dp * 2);
  p.proj_sorted = K > 1 ? take(S * Dp * 2) : kNone;
  p.qkv = take(N * Dc * 2);
  p.y = take(N * Dv * 2);
  p.op_sorted = K > 1 ? take(S * Dm * 2) : kNone;
  p.conv_tmp = take(seq_len > kConvInPlaceMaxLen ? static_cast<size_t>(n_seq) * Dc * 3 * 4 : 0);
  p.carry = take(gdn_carry_bytes(n_seq, seq_len, d->n_heads, d->d_k));
  p.rstd = take(N * 4);
  p.total = off;
  return p;
}
}  // namespace

size_t rom_gdn_workspace_bytes(const rom_gdn_dims *dims, int64_t B, int64_t L) {
  if (check_gdn_dims(dims) != ROM_OK || B < 0 || L < 0) return 0;
  return make_gdn_plan(dims, B > 0 ? B : 1, L > 0 ? L : 1).total;
}

int rom_gdn_workspace_layout(const rom_gdn_dims *dims, int64_t B, int64_t L, rom_gdn_ws_layout *layout) {
  const int rc = check_gdn_dims(dims);
  if (rc != ROM_OK) return rc;
  if (!layout || B < 0 || L < 0) return ROM_E_INVAL;
  const GdnPlan p = make_gdn_plan(dims, B > 0 ? B : 1, L > 0 ? L : 1);
  layout->total_bytes = p.total;
  layout->expert_idx = p.expert_idx;
  layout->gate = p.gate;
  layout->counts = p.counts;
  layout->offsets = p.offsets;
  layout->perm = p.perm;
  layout->inv_perm = p.inv_perm;
  layout->logits = p.logits;
  layout->proj = p.proj;
  layout->qkv = p.qkv;
  layout->y = p.y;
  return ROM_OK;
}

namespace {
int gdn_impl(const rom_gdn_dims *d, const rom_gdn_weights *w, const float *pre_norm_w, float pre_norm_eps, const void *x,
             int64_t B, int64_t L, float eps, const float *conv_in, const float *ssm_in, void *out, float *conv_out,
             float *ssm_out, void *ws, size_t ws_bytes, void *hip_stream);
}

int rom_gdn_forward(const rom_gdn_dims *d, const rom_gdn_weights *w, const void *x, int64_t B, int64_t L, float eps,
                    const float *conv_in, const float *ssm_in, void *out, float *conv_out, float *ssm_out, void *ws,
                    size_t ws_bytes, void *hip_stream) {
  return gdn_impl(d, w, nullptr, 0.0f, x, B, L, eps, conv_in, ssm_in, out, conv_out, ssm_out, ws, ws_bytes, hip_stream);
}

int rom_gdn_block_forward(const rom_gdn_dims *d, const rom_gdn_weights *w, const float *norm_weight, float norm_eps,
                          const void *x, int64_t B, int64_t L, float eps, const float *conv_in, const float *ssm_in,
                          void *out, float *conv_out, float *ssm_out, void *ws, size_t ws_bytes, void *hip_stream) {
  if (!norm_weight || !aligned16(norm_weight) || !(norm_eps >= 0.0f) || out == x) return ROM_E_INVAL;
  return gdn_impl(d, w, norm_weight, norm_eps, x, B, L, eps, conv_in, ssm_in, out, conv_out, ssm_out, ws, ws_bytes,
                  hip_stream);
}

namespace {
int gdn_impl(const rom_gdn_dims *d, const rom_gdn_weights *w, const float *pre_norm_w, float pre_norm_eps, const void *x,
             int64_t B, int64_t L, float eps, const float *conv_in, const float *ssm_in, void *out, float *conv_out,
             float *ssm_out, void *ws, size_t ws_bytes, void *hip_stream) {
  int rc = check_gdn_dims(d);
  if (rc != ROM_OK) return rc;
  if (!w) return ROM_E_INVAL;
  {
    const void *req[] = {w->w_router, w->w_in, w->conv_w, w->dt_bias, w->A_log, w->norm_w, w->w_out};
    for (const void *ptr : req)
      if (!ptr || !aligned16(ptr)) return ROM_E_INVAL;
    if ((w->b_router && !aligned16(w->b_router)) || (w->conv_b && !aligned16(w->conv_b))) return ROM_E_INVAL;
  }
  if (B < 0 || L < 0) return ROM_E_INVAL;
  if (B == 0 || L == 0) return ROM_OK;
  rc = check_variant_call(x, out, ws, B, L, d->top_k, eps, conv_in, ssm_in, conv_out, ssm_out);
  if (rc != ROM_OK) return rc;
  const GdnPlan p = make_gdn_plan(d, B, L);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char *base = static_cast<char *>(ws);
  const int H = d->n_heads, Dk = H * d->d_k, Dv = H * d->d_v, Dp = 2 * Dv + 2 * Dk + 2 * H, Dc = 2 * Dk + Dv;

  VariantFrame f;
  f.dtype = d->dtype; f.gate_mode = d->gate_mode; f.n_experts = d->n_experts; f.top_k = d->top_k; f.d_model = d->d_model;
  f.d_proj = Dp; f.conv_col = Dv; f.d_conv_ch = Dc; f.d_y = Dv;          // z | q | k | v | b | a: the conv runs over q | k | v
  f.w_router = w->w_router; f.b_router = w->b_router; f.w_in = w->w_in; f.conv_w = w->conv_w; f.conv_b = w->conv_b;
  f.w_out = w->w_out;
  f.expert_idx = p.expert_idx; f.gate = p.gate; f.counts = p.counts; f.offsets = p.offsets; f.perm = p.perm;
  f.inv_perm = p.inv_perm; f.tok_of_pos = p.tok_of_pos; f.block_counts = p.block_counts; f.logits = p.logits;
  f.proj = p.proj; f.proj_sorted = p.proj_sorted; f.conv_dst = p.qkv; f.y = p.y; f.op_sorted = p.op_sorted;
  f.conv_tmp = p.conv_tmp;
  f.pre_norm_w = pre_norm_w; f.pre_norm_eps = pre_norm_eps; f.rstd = p.rstd;
  return run_variant(f, x, B, L, conv_in, conv_out, out, base, s, [&](StageMark &mark) {
    // delta rule, head norm, SiLU(z) gate
    mark.begin(ROM_STAGE_SCAN, s);
    ROM_TRY(launch_gdn_scan(base + p.qkv, Dc, 0, Dk, 2 * Dk, base + p.proj, Dp, Dv + Dc, Dv + Dc + H, w->dt_bias, w->A_log,
                            w->norm_w, eps, B, L, H, d->d_k, ssm_in, ssm_out, reinterpret_cast<float *>(base + p.carry),
                            base + p.y, Dv, s));
    mark.end(ROM_STAGE_SCAN, s);
    return static_cast<int>(ROM_OK);
  });
}
}  // namespace

int rom_gdn_step(const rom_gdn_dims *d, const rom_gdn_weights *w, const void *x, int64_t B, float eps, float *conv_state,
                 float *ssm_state, void *out, void *ws, size_t ws_bytes, void *hip_stream) {
  if (B > 0 && (!conv_state || !ssm_state)) return ROM_E_INVAL;
  return rom_gdn_forward(d, w, x, B, 1, eps, conv_state, ssm_state, out, conv_state, ssm_state, ws, ws_bytes, hip_stream);
}

size_t rom_backward_workspace_bytes(const rom_dims *dims, int64_t B, int64_t L) {
  if (check_dims(dims) != ROM_OK || B < 0 || L < 0) return 0;
  return make_bwd_plan(dims, B > 0 ? B : 1, L > 0 ? L : 1).total;
}

namespace {
int backward_impl(const rom_dims *d, const rom_weights *w, const void *x, int64_t B, int64_t L, const void *d_out,
                  void *d_x, const rom_grads *gr, void *ws, size_t ws_bytes, void *hip_stream, bool recompute,
                  const float *d_gate_extra = nullptr, const void *route_x = nullptr, const BlockOpts *route_blk = nullptr);
}

int rom_layer_backward(const rom_dims *d, const rom_weights *w, const void *x, int64_t B, int64_t L, const void *d_out,
                       void *d_x, const rom_grads *gr, void *ws, size_t ws_bytes, void *hip_stream) {
  return backward_impl(d, w, x, B, L, d_out, d_x, gr, ws, ws_bytes, hip_stream, true);
}

int rom_layer_backward_saved(const rom_dims *d, const rom_weights *w, const void *x, int64_t B, int64_t L,
                             const void *d_out, void *d_x, const rom_grads *gr, void *ws, size_t ws_bytes,
                             void *hip_stream) {
  return backward_impl(d, w, x, B, L, d_out, d_x, gr, ws, ws_bytes, hip_stream, false);
}

namespace {
// workspace of rom_block_backward: the layer's backward plan, then the normalised input, its gradient,
// 1/rms per token and the partial sums of d_norm_weight
struct BlockBwdPlan {
  size_t total, inner, xn, d_xn, rstd, part;
};
BlockBwdPlan make_block_bwd_plan(const rom_dims *d, int64_t B, int64_t L) {
  BlockBwdPlan p;
  const size_t N = static_cast<size_t>(B) * static_cast<size_t>(L);
  const size_t eb = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return at;
  };
  p.inner = make_bwd_plan(d, B, L).total;
  take(p.inner);
  p.xn = take(N * d->d_model * eb);
  p.d_xn = take(N * d->d_model * eb);
  p.rstd = take(N * 4);
  p.part = take(static_cast<size_t>(rmsnorm_wgrad_parts(static_cast<int64_t>(N))) * d->d_model * 4);
  p.total = off;
  return p;
}
}  // namespace

size_t rom_block_backward_workspace_bytes(const rom_dims *d, int64_t B, int64_t L) {
  if (check_dims(d) != ROM_OK || B < 0 || L < 0) return 0;
  if (rom_backward_workspace_bytes(d, B, L) == 0 && B > 0 && L > 0) return 0;
  return make_block_bwd_plan(d, B, L).total;
}

namespace {
// what of the block's training step a call runs
enum { kBlockForward = 1, kBlockBackward = 2 };
int block_train_impl(int what, const rom_dims *d, const rom_weights *w, const float *norm_weight, float eps, const void *x,
                     int64_t B, int64_t L, void *out, const void *d_out, const float *d_gate_ffn, void *d_x,
                     const rom_grads *gr, float *d_norm_weight, void *ws, size_t ws_bytes, void *hip_stream) {
  const bool fwd = (what & kBlockForward) != 0, bwd = (what & kBlockBackward) != 0;
  int rc = check_dims(d);
  if (rc != ROM_OK) return rc;
  if (!norm_weight || !aligned16(norm_weight) || !(eps >= 0.0f) || (bwd && !d_norm_weight)) return ROM_E_INVAL;
  if (B < 0 || L < 0) return ROM_E_INVAL;
  if (B == 0 || L == 0) return ROM_OK;
  if (!x || !ws || !aligned16(x) || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return ROM_E_INVAL;
  if (bwd && (!d_out || !d_x || d_x == x || d_x == d_out || !aligned16(d_out) || !aligned16(d_x))) return ROM_E_INVAL;
  if (!bwd && (!out || out == x || !aligned16(out))) return ROM_E_INVAL;
  if (d->d_model % 8 != 0) return ROM_E_UNSUPPORTED;
  const BlockBwdPlan p = make_block_bwd_plan(d, B, L);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char *base = static_cast<char *>(ws);
  const int64_t N = B * L;
  float *rstd = reinterpret_cast<float *>(base + p.rstd);
  // the router reads the raw x and normalises it itself, exactly as in rom_block_forward: the backward
  // differentiates the expert choice the forward made (a router fed the rounded norm could pick
  // another expert for a token whose two best logits are nearly equal)
  BlockOpts opts;
  opts.norm_w = norm_weight;
  opts.eps = eps;
  if (!bwd) {
    // the training step's forward: the same arithmetic the backward recomputes (materialised norm, plain
    // weights), activations left in the workspace for rom_block_backward_saved
    if (B * L * d->top_k > (1ll << 24) || B > 65535) return ROM_E_UNSUPPORTED;
    rc = check_weights(d, w);
    if (rc != ROM_OK) return rc;
    ROM_TRY(launch_rmsnorm_forward(d->dtype, x, norm_weight, eps, N, d->d_model, base + p.xn, rstd, s));
    char *layer_out = base + make_bwd_plan(d, B, L).fwd_out;
    rc = forward_impl(d, w, base + p.xn, B, L, nullptr, nullptr, layer_out, nullptr, nullptr, ws, make_plan(d, B, L).total, s,
                      nullptr, x, &opts);
    if (rc != ROM_OK) return rc;
    ROM_TRY(launch_add(d->dtype, x, layer_out, out, N * d->d_model, s));
    return ROM_OK;
  }
  // the layer's backward runs on the materialised norm (the forward block never forms it: its in
  // projection scales rows of x W'^T instead, which differs by the rounding of xn to the type)
  if (fwd) ROM_TRY(launch_rmsnorm_forward(d->dtype, x, norm_weight, eps, N, d->d_model, base + p.xn, rstd, s));
  rc = backward_impl(d, w, base + p.xn, B, L, d_out, base + p.d_xn, gr, ws, p.inner, hip_stream, fwd, d_gate_ffn, x, &opts);
  if (rc != ROM_OK) return rc;
  ROM_TRY(launch_rmsnorm_backward(d->dtype, x, norm_weight, rstd, base + p.d_xn, d_out, N, d->d_model, d_x,
                                  reinterpret_cast<float *>(base + p.part), d_norm_weight, s));
  return ROM_OK;
}
}  // namespace

int rom_block_backward(const rom_dims *d, const rom_weights *w, const float *norm_weight, float eps, const void *x,
                       int64_t B, int64_t L, const void *d_out, const float *d_gate_ffn, void *d_x, const rom_grads *gr,
                       float *d_norm_weight, void *ws, size_t ws_bytes, void *hip_stream) {
  return block_train_impl(kBlockForward | kBlockBackward, d, w, norm_weight, eps, x, B, L, nullptr, d_out, d_gate_ffn, d_x, gr,
                          d_norm_weight, ws, ws_bytes, hip_stream);
}

int rom_block_forward_train(const rom_dims *d, const rom_weights *w, const float *norm_weight, float eps, const void *x,
                            int64_t B, int64_t L, void *out, void *ws, size_t ws_bytes, void *hip_stream) {
  return block_train_impl(kBlockForward, d, w, norm_weight, eps, x, B, L, out, nullptr, nullptr, nullptr, nullptr, nullptr, ws,
                          ws_bytes, hip_stream);
}

int rom_block_backward_saved(const rom_dims *d, const rom_weights *w, const float *norm_weight, float eps, const void *x,
                             int64_t B, int64_t L, const void *d_out, const float *d_gate_ffn, void *d_x,
                             const rom_grads *gr, float *d_norm_weight, void *ws, size_t ws_bytes, void *hip_stream) {
  return block_train_impl(kBlockBackward, d, w, norm_weight, eps, x, B, L, nullptr, d_out, d_gate_ffn, d_x, gr, d_norm_weight, ws,
                          ws_bytes, hip_stream);
}

namespace {
int backward_impl(const rom_dims *d, const rom_weights *w, const void *x, int64_t B, int64_t L, const void *d_out,
                  void *d_x, const rom_grads *gr, void *ws, size_t ws_bytes, void *hip_stream, bool recompute,
                  const float *d_gate_extra, const void *route_x, const BlockOpts *route_blk) {
  int rc = check_dims(d);
  if (rc != ROM_OK) return rc;
  rc = check_weights(d, w);
  if (rc != ROM_OK) return rc;
  if (B < 0 || L < 0) return ROM_E_INVAL;
  if (B == 0 || L == 0) return ROM_OK;
  if (!x || !d_out || !d_x || !gr || !ws || d_x == x || d_x == d_out) return ROM_E_INVAL;
  if (!aligned16(x) || !aligned16(d_out) || !aligned16(d_x) || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0)
    return ROM_E_INVAL;
  const float *need[] = {gr->d_w_router, gr->d_w_in, gr->d_conv_w, gr->d_w_x, gr->d_w_dt, gr->d_dt_bias, gr->d_A_log,
                         gr->d_D, gr->d_w_out};
  for (const float *ptr : need)
    if (!ptr || !aligned16(ptr)) return ROM_E_INVAL;
  if (B * L * d->top_k > (1ll << 24) || B > 65535) return ROM_E_UNSUPPORTED;      // grid limits of the reduction kernels
  const BwdPlan bp = make_bwd_plan(d, B, L);
  if (ws_bytes < bp.total) return ROM_E_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char *base = static_cast<char *>(ws);
  auto at = [&](size_t off) { return base + off; };
  const Plan p = make_plan(d, B, L);
  const int64_t N = B * L;
  const int E = d->n_experts, Ex = d->n_experts_xdt, De = d->d_inner, Dm = d->d_model, R = d->dt_rank, K = d->top_k;
  const size_t eb = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;
  const bool routed_xdt = Ex > 1, multi = K > 1;
  const int64_t S = N * K;

  // activations: the forward pass into the front part of the workspace, unless the caller's own
  // rom_layer_forward call on this workspace has just left them there
  if (recompute) {
    rc = forward_impl(d, w, x, B, L, nullptr, nullptr, at(bp.fwd_out), nullptr, nullptr, ws, p.total, s, nullptr, route_x,
                      route_blk);
    if (rc != ROM_OK) return rc;
  }
  const int32_t *offsets = reinterpret_cast<const int32_t *>(at(p.offsets));
  const int32_t *tok_of_pos = reinterpret_cast<const int32_t *>(at(p.tok_of_pos));
  const int32_t *perm = reinterpret_cast<const int32_t *>(at(p.perm));
  const int32_t *inv_perm = reinterpret_cast<const int32_t *>(at(p.inv_perm));
  const float *gate = reinterpret_cast<const float *>(at(p.gate));                 // [N, K]
  float *d_gate = reinterpret_cast<float *>(at(bp.d_gate));
  float *d_logits = reinterpret_cast<float *>(at(bp.d_logits));

  // transposed weights: d_inp = d_out W contracts over the row index of W (the two big projections
  // are transposed only where the GEMM cannot read them contraction-major, see dgrad)
  ROM_TRY(launch_transpose(d->dtype, w->w_dt, at(bp.wt_dt), Ex, De, R, s));            // -> [Ex][R][De]
  ROM_TRY(launch_transpose(d->dtype, w->w_x, at(bp.wt_x), Ex, R + 32, De, s));         // -> [Ex][De][R+32]

  // Input gradient of a routed projection, d_inp[n] = sum_k W[e_k(n)]^T d_outp[n]: the forward's grouped
  // GEMM on the transposed weights.  top-1: rows gathered from and scattered to token order, C is the
  // result.  top-K: A rows by token (or, a_by_pos, already one per sorted position), one output row per
  // sorted position in `pos`, then the K rows of a token are added (like the forward's per-slot outputs).
  // W_fwd (optional): the forward weight [n_groups][k_in][n_out] that Wt is to be the transpose of.  Where
  // the GEMM takes it contraction-major it is read as it is; otherwise it is transposed into Wt here.
  auto dgrad = [&](const void *A, int64_t lda, bool a_by_pos, const void *Wt, int n_groups, int n_out, int k_in, void *C,
                   int64_t ldc, int c_is_f32, void *pos, const void *W_fwd = nullptr) -> int {
    GemmArgs ga;
    memset(&ga, 0, sizeof(ga));
    ga.dtype = d->dtype;
    ga.A = A; ga.lda = lda; ga.a_span = (a_by_pos ? S : N) * lda;
    ga.W = Wt; ga.N = n_out; ga.K = k_in;
    ga.ldc = ldc; ga.c_is_f32 = c_is_f32;
    if (n_groups <= 1) {
      ga.n_groups = 1; ga.M = N; ga.C = C;
    } else {
      ga.n_groups = n_groups; ga.offsets = offsets; ga.M = S;
      ga.a_rows = a_by_pos ? nullptr : tok_of_pos;
      if (!multi) {
        ga.c_rows = tok_of_pos; ga.C = C;
      } else {
        ga.C = pos;
      }
    }
    if (W_fwd) {
      GemmArgs gk = ga;
      gk.W = W_fwd; gk.w_kmajor = 1;
      if (grouped_gemm_takes_kmajor(gk))
        ga = gk;
      else
        ROM_TRY(launch_transpose(d->dtype, W_fwd, const_cast<void *>(Wt), n_groups < 1 ? 1 : n_groups, k_in, n_out, s));
    }
    ROM_TRY(launch_grouped_gemm(ga, s));
    if (n_groups <= 1 || !multi) return ROM_OK;
    const bool f32 = c_is_f32 || eb == 4;
    ROM_TRY(launch_slot_sum(f32, f32, pos, ldc, C, ldc, inv_perm, N, K, n_out, nullptr, 0, nullptr, s));
    return ROM_OK;
  };
  // Weight gradient d W[e] = sum over the expert's sorted positions of d_outp^T inp; both operands by
  // the position's token unless a_by_pos says that A already has one row per position
  auto wgrad = [&](const void *A, int64_t lda, bool a_by_pos, int M, const void *Bm, int64_t ldb, int Nn, int n_groups,
                   float *C) {
    const bool routed_call = n_groups > 1;
    return launch_wgrad(d->dtype, A, lda, M, Bm, ldb, Nn, (routed_call && !a_by_pos) ? tok_of_pos : nullptr,
                        routed_call ? tok_of_pos : nullptr, nullptr, routed_call ? offsets : nullptr, n_groups,
                        routed_call ? S : N, C, s);
  };
#define ROM_RC(expr)            \
  do {                          \
    const int rc_ = (expr);     \
    if (rc_ != ROM_OK) return rc_; \
  } while (0)

  // Eq. (12)/(13): out = sum_k gate_k * (W_out[e_k] g)
  const void *dsc;            // gate-weighted d_out, one row per sorted position
  const float *scan_gate;     // weight the adjoint scan still has to put on d g
  if (!multi) {
    ROM_RC(dgrad(d_out, Dm, false, at(bp.wt_out), E, De, Dm, at(bp.dg_raw), De, 0, nullptr, w->w_out));   // dg_raw = W_out[e]^T d_out
    ROM_TRY(launch_gate_backward(d->dtype, at(bp.dg_raw), at(p.g), nullptr, 1, N, De, d_gate, s));
    // (the gate weight goes onto d_out once, in the buffer that later receives dx_in, so that the
    // weight-gradient kernel contracts two plain operands)
    ROM_TRY(launch_scale_rows(d->dtype, d_out, gate, nullptr, nullptr, N, Dm, at(bp.dx_in), s));
    ROM_TRY(wgrad(at(bp.dx_in), Dm, false, Dm, at(p.g), De, De, E, gr->d_w_out));
    scan_gate = gate;
  } else {
    // d gate of a slot: d_out of its token against the expert output the forward pass left per position
    ROM_TRY(launch_gate_backward(d->dtype, d_out, at(p.op_sorted), inv_perm, K, S, Dm, d_gate, s));
    ROM_TRY(launch_scale_rows(d->dtype, d_out, gate, tok_of_pos, perm, S, Dm, at(bp.pos_dm), s));
    dsc = at(bp.pos_dm);
    ROM_TRY(wgrad(dsc, Dm, true, Dm, at(p.g), De, De, E, gr->d_w_out));
    ROM_RC(dgrad(dsc, Dm, true, at(bp.wt_out), E, De, Dm, at(bp.dg_raw), De, 0, at(bp.pos_de), w->w_out));   // already gate-weighted
    scan_gate = nullptr;
  }
  // Eq. (5), (6): scan, gate, softplus
  ROM_TRY(launch_scan_backward(d->dtype, at(p.u), at(p.dt), reinterpret_cast<const float *>(at(p.bc)),
                               at(p.xz) + static_cast<size_t>(De) * eb, 2 * De, at(bp.dg_raw), scan_gate, w->A_log, w->D,
                               B, L, De, reinterpret_cast<float *>(at(bp.ckpt)),
                               reinterpret_cast<float *>(at(bp.bc_part)), at(bp.d_pre), at(bp.d_u_scan),
                               at(bp.d_xz) + static_cast<size_t>(De) * eb, 2 * De, reinterpret_cast<float *>(at(bp.d_bc)),
                               gr->d_A_log, gr->d_D, gr->d_dt_bias, s));
  // dt projection
  ROM_RC(dgrad(at(bp.d_pre), De, false, at(bp.wt_dt), routed_xdt ? E : 1, R, De, at(bp.d_dt_low), R, 1,
               multi && routed_xdt ? at(bp.pos_r) : nullptr));
  ROM_TRY(wgrad(at(bp.d_pre), De, false, De, at(p.dt_low), R, R, routed_xdt ? E : 1, gr->d_w_dt));
  // x projection
  ROM_TRY(launch_pack_dxdbl(d->dtype, reinterpret_cast<const float *>(at(bp.d_dt_low)),
                            reinterpret_cast<const float *>(at(bp.d_bc)), N, R, at(bp.d_xdbl), s));
  ROM_RC(dgrad(at(bp.d_xdbl), R + 32, false, at(bp.wt_x), routed_xdt ? E : 1, De, R + 32, at(bp.d_u_x), De, 0,
               multi ? at(bp.pos_de) : nullptr));
  ROM_TRY(wgrad(at(bp.d_xdbl), R + 32, false, R + 32, at(p.u), De, De, routed_xdt ? E : 1, gr->d_w_x));
  // Eq. (2): conv + SiLU; writes the conv half of d_xz
  ROM_TRY(launch_conv_backward(d->dtype, at(p.xz), 2 * De, w->conv_w, w->conv_b, at(bp.d_u_scan), at(bp.d_u_x), B, L, De,
                               at(bp.d_xz), 2 * De, reinterpret_cast<float *>(at(bp.conv_part)), gr->d_conv_w,
                               gr->d_conv_b, s));
  // Eq. (10)/(11): in / gate projection
  ROM_RC(dgrad(at(bp.d_xz), 2 * De, false, at(bp.wt_in), E, Dm, 2 * De, at(bp.dx_in), Dm, 0,
               multi ? at(bp.pos_dm) : nullptr, w->w_in));
  ROM_TRY(wgrad(at(bp.d_xz), 2 * De, false, 2 * De, x, Dm, Dm, E, gr->d_w_in));
#undef ROM_RC
  // Eq. (9): the router through the gate weights (plus what an FFN-MoE layer on this decision sends back, Eq. (15))
  if (d_gate_extra) {
    hipLaunchKernelGGL(add_f32_kernel, dim3(static_cast<unsigned>(ceil_div(S, 256))), dim3(256), 0, s, d_gate_extra, d_gate, S);
    ROM_TRY(hipGetLastError());
  }
  ROM_TRY(launch_router_backward(d->dtype, reinterpret_cast<const float *>(at(p.logits)),
                                 reinterpret_cast<const int32_t *>(at(p.expert_idx)), d_gate, x, N, Dm, E, K,
                                 d->gate_mode, d_logits, reinterpret_cast<float *>(at(bp.router_part)), gr->d_w_router,
                                 gr->d_b_router, s));
  ROM_TRY(launch_dx_finish(d->dtype, at(bp.dx_in), d_logits, w->w_router, N, Dm, E, d_x, s));
  return ROM_OK;
}
}  // namespace

const char *rom_strerror(int code) {
  switch (code) {
    case ROM_OK: return "ok";
    case ROM_E_INVAL: return "invalid argument (NULL or misaligned pointer, bad enum or size)";
    case ROM_E_WORKSPACE: return "workspace too small (see rom_workspace_bytes)";
    case ROM_E_UNSUPPORTED: return "shape not supported by this build (see rom_dims)";
    case ROM_E_HIP: return "a HIP call or kernel launch failed";
    case ROM_E_STATIC_LIMIT: return "the call needs more scratch than the library's static buffer holds (see rom_step_static)";
    default: return "unknown error code";
  }
}

int rom_profile_enable(int max_calls) {
  if (g_prof.ev) {
    for (int i = 0; i < g_prof.max_calls * kProfEvents; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    delete[] g_prof.begin_of;
    delete[] g_prof.end_of;
    g_prof.ev = nullptr;
    g_prof.begin_of = nullptr;
    g_prof.end_of = nullptr;
  }
  g_prof.max_calls = 0;
  g_prof.n_calls = 0;
  if (max_calls <= 0) return ROM_OK;
  const int n = max_calls * kProfEvents;
  g_prof.ev = new hipEvent_t[n];
  g_prof.begin_of = new int[max_calls * ROM_STAGE_COUNT];
  g_prof.end_of = new int[max_calls * ROM_STAGE_COUNT];
  for (int i = 0; i < max_calls * ROM_STAGE_COUNT; ++i) g_prof.begin_of[i] = g_prof.end_of[i] = -1;
  for (int i = 0; i < n; ++i)
    if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) return ROM_E_HIP;
  g_prof.max_calls = max_calls;
  return ROM_OK;
}

int rom_profile_select(unsigned stage_mask) {
  g_prof.stage_mask = stage_mask;
  return ROM_OK;
}

int rom_profile_collect(double *stage_ms, int *n_calls) {
  if (!stage_ms || !n_calls) return ROM_E_INVAL;
  for (int i = 0; i < ROM_STAGE_COUNT; ++i) stage_ms[i] = 0.0;
  *n_calls = g_prof.n_calls;
  for (int c = 0; c < g_prof.n_calls; ++c) {
    for (int i = 0; i < ROM_STAGE_COUNT; ++i) {
      int &b = g_prof.begin_of[c * ROM_STAGE_COUNT + i], &e = g_prof.end_of[c * ROM_STAGE_COUNT + i];
      if (b < 0 || e < 0) continue;
      if (hipEventSynchronize(g_prof.ev[e]) != hipSuccess) return ROM_E_HIP;
      float ms = 0.0f;
      if (hipEventElapsedTime(&ms, g_prof.ev[b], g_prof.ev[e]) != hipSuccess) return ROM_E_HIP;
      stage_ms[i] += ms;
      b = e = -1;
    }
  }
  g_prof.n_calls = 0;
  return ROM_OK;
}

int rom_profile_collect_calls(double *stage_ms, int max_calls, int *n_calls) {
  if (!stage_ms || !n_calls || max_calls < 0) return ROM_E_INVAL;
  const int n = g_prof.n_calls < max_calls ? g_prof.n_calls : max_calls;
  *n_calls = n;
  for (int c = 0; c < g_prof.n_calls; ++c) {
    for (int i = 0; i < ROM_STAGE_COUNT; ++i) {
      int &b = g_prof.begin_of[c * ROM_STAGE_COUNT + i], &e = g_prof.end_of[c * ROM_STAGE_COUNT + i];
      float ms = 0.0f;
      if (b >= 0 && e >= 0) {
        if (hipEventSynchronize(g_prof.ev[e]) != hipSuccess) return ROM_E_HIP;
        if (hipEventElapsedTime(&ms, g_prof.ev[b], g_prof.ev[e]) != hipSuccess) return ROM_E_HIP;
      }
      if (c < n) stage_ms[c * ROM_STAGE_COUNT + i] = ms;
      b = e = -1;
    }
  }
  g_prof.n_calls = 0;
  return ROM_OK;
}

// plain copy of known traffic (n_bytes read, n_bytes written), 16 bytes per thread
__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

int rom_profile_copy(const void *src, void *dst, size_t n_bytes, void *hip_stream) {
  if (!src || !dst || src == dst || n_bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return ROM_E_INVAL;
  if (n_bytes == 0) return ROM_OK;
  const int64_t n = static_cast<int64_t>(n_bytes / 16);
  if (ceil_div(n, 256) > 0x7fffffffll) return ROM_E_UNSUPPORTED;
  hipLaunchKernelGGL(calib_copy_kernel, dim3(static_cast<unsigned>(ceil_div(n, 256))), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n);
  return hipGetLastError() == hipSuccess ? ROM_OK : ROM_E_HIP;
}

int rom_probe(int kind, int p0, int p1, int n_blocks, int iters, void *scratch, size_t scratch_bytes,
              void *hip_stream) {
  if (!scratch || n_blocks < 1 || iters < 1 || scratch_bytes < static_cast<size_t>(n_blocks) * 256 * sizeof(float))
    return ROM_E_INVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  float *out = static_cast<float *>(scratch);
  const hipError_t e = kind == 0 ? launch_probe_issue(p0, p1, n_blocks, iters, out, s)
                                 : launch_probe_scan(p0, p1, n_blocks, iters, out, s);
  if (e == hipErrorInvalidValue) return ROM_E_INVAL;
  return e == hipSuccess ? ROM_OK : ROM_E_HIP;
}

const char *rom_stage_name(int stage) {
  static const char *names[ROM_STAGE_COUNT] = {"route", "permute", "in_proj", "conv", "x_proj",
                                               "dt_proj", "scan_gate", "out_proj", "combine"};
  return (stage >= 0 && stage < ROM_STAGE_COUNT) ? names[stage] : "?";
}

}  // extern "C"
