// C ABI of librom: argument validation, workspace planning and the launch sequence of the
// RoM layer forward pass (Eq. (9)-(13)) and its single-token recurrent step.
#include <string.h>

#include "rom_internal.h"

namespace rom {
namespace {

constexpr size_t kAlign = 256;
constexpr size_t kNone = static_cast<size_t>(-1);

struct Plan {                 // byte offsets inside the workspace
  size_t total;
  size_t expert_idx, gate, counts, offsets, perm, inv_perm, tok_of_pos, block_counts, logits;
  size_t xz, xz_sorted, u, xdbl, dt_low, bc, dt, dt_raw, g, op_sorted, conv_tmp, scan_q, scan_p;
};

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
  p.expert_idx = take(S * 4);
  p.gate = take(S * 4);
  p.counts = take(E * 4);
  p.offsets = take((E + 1) * 4);
  p.perm = take(S * 4);
  p.inv_perm = take(S * 4);
  p.tok_of_pos = take(S * 4);
  p.block_counts = take(static_cast<size_t>(route_blocks(static_cast<int64_t>(S))) * E * 4);
  p.logits = take(N * E * 4);
  p.xz = take(N * 2 * De * b);
  p.xz_sorted = multi ? take(S * 2 * De * b) : kNone;
  p.u = take(N * De * b);
  p.xdbl = take((routed_xdt ? S : N) * (R + 32) * 4 * xproj_k_splits(routed_xdt ? S : N, routed_xdt ? d->n_experts : 1, d->d_inner));
  p.dt_low = take(N * R * b);
  p.bc = take(N * 32 * 4);
  p.dt = take(N * De * b);
  p.dt_raw = (multi && routed_xdt) ? take(S * De * 4) : kNone;
  p.g = take(N * De * b);
  p.op_sorted = multi ? take(S * Dm * b) : kNone;
  p.conv_tmp = take(static_cast<size_t>(n_seq) * De * 3 * 4);
  p.scan_q = take(scan_chunk_state_bytes(n_seq, seq_len, d->d_inner));
  p.scan_p = take(scan_chunk_state_bytes(n_seq, seq_len, d->d_inner));
  p.total = off;
  return p;
}

// ---------------------------------------------------------------- stage timing
struct Profiler {
  int max_calls = 0, n_calls = 0;
  hipEvent_t *ev = nullptr;          // [max_calls][ROM_STAGE_COUNT + 1]
} g_prof;

struct StageMark {
  hipStream_t s;
  int call;
  bool on;
  explicit StageMark(hipStream_t st) : s(st), call(-1), on(false) {
    if (g_prof.ev && g_prof.n_calls < g_prof.max_calls) {
      call = g_prof.n_calls++;
      on = true;
      (void)hipEventRecord(g_prof.ev[call * (ROM_STAGE_COUNT + 1)], s);
    }
  }
  void done(int stage) {   // stages must be marked in increasing order; skipped ones get zero time
    if (on) (void)hipEventRecord(g_prof.ev[call * (ROM_STAGE_COUNT + 1) + stage + 1], s);
  }
};

#define ROM_TRY(expr)                      \
  do {                                     \
    if ((expr) != hipSuccess) return ROM_E_HIP; \
  } while (0)

__global__ void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

int route_into(const rom_dims *d, const rom_weights *w, const void *x, int64_t n_tok,
               int32_t *expert_idx, float *gate, int32_t *counts, int32_t *offsets, int32_t *perm,
               int32_t *inv_perm, int32_t *tok_of_pos, int32_t *block_counts, float *logits,
               hipStream_t s, StageMark *mark) {
  ROM_TRY(launch_route_topk(d->dtype, x, w->w_router, w->b_router, n_tok, d->d_model, d->n_experts,
                            d->top_k, d->gate_mode, expert_idx, gate, logits, s));
  if (mark) mark->done(ROM_STAGE_ROUTE);
  ROM_TRY(launch_permutation(expert_idx, n_tok * d->top_k, d->n_experts, d->top_k, block_counts,
                             counts, offsets, perm, inv_perm, tok_of_pos, s));
  if (mark) mark->done(ROM_STAGE_PERMUTE);
  return ROM_OK;
}

int forward_impl(const rom_dims *d, const rom_weights *w, const void *x, int64_t B, int64_t L,
                 const float *conv_in, const float *ssm_in, void *out, float *conv_out,
                 float *ssm_out, void *ws, size_t ws_bytes, hipStream_t s) {
  int rc = check_dims(d);
  if (rc != ROM_OK) return rc;
  rc = check_weights(d, w);
  if (rc != ROM_OK) return rc;
  if (B < 0 || L < 0) return ROM_E_INVAL;
  if (B == 0 || L == 0) return ROM_OK;
  if (!x || !out || !ws || x == out) return ROM_E_INVAL;
  if (!aligned16(x) || !aligned16(out) || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return ROM_E_INVAL;
  if (B * L * d->top_k > (1ll << 30) || B > 65535) return ROM_E_UNSUPPORTED;
  const int64_t N = B * L;
  Plan p = make_plan(d, B, L);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;

  char *base = static_cast<char *>(ws);
  auto at = [&](size_t off) { return static_cast<void *>(base + off); };
  const int K = d->top_k, E = d->n_experts, De = d->d_inner, Dm = d->d_model, R = d->dt_rank;
  const bool multi = K > 1, routed_xdt = d->n_experts_xdt > 1;
  const int64_t S = N * K;
  int32_t *idx = static_cast<int32_t *>(at(p.expert_idx));
  float *gate = static_cast<float *>(at(p.gate));
  int32_t *offsets = static_cast<int32_t *>(at(p.offsets));
  int32_t *inv_perm = static_cast<int32_t *>(at(p.inv_perm));
  int32_t *tok_of_pos = static_cast<int32_t *>(at(p.tok_of_pos));
  const size_t eb = d->dtype == ROM_DTYPE_BF16 ? 2 : 4;

  StageMark mark(s);
  rc = route_into(d, w, x, N, idx, gate, static_cast<int32_t *>(at(p.counts)), offsets,
                  static_cast<int32_t *>(at(p.perm)), inv_perm, tok_of_pos,
                  static_cast<int32_t *>(at(p.block_counts)), static_cast<float *>(at(p.logits)), s, &mark);
  if (rc != ROM_OK) return rc;

  // in / gate projection, Eq. (10)/(11): gather token rows, scatter back to token order (K == 1)
  GemmArgs ga;
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.A = x; ga.lda = Dm; ga.a_rows = tok_of_pos; ga.a_span = N * Dm;
  ga.W = w->w_in; ga.offsets = offsets; ga.n_groups = E;
  ga.M = S; ga.N = 2 * De; ga.K = Dm;
  ga.C = multi ? at(p.xz_sorted) : at(p.xz); ga.ldc = 2 * De; ga.c_rows = multi ? nullptr : tok_of_pos;
  ROM_TRY(launch_grouped_gemm(ga, s));
  if (multi)
    ROM_TRY(launch_slot_sum(eb == 4, eb == 4, at(p.xz_sorted), 2 * De, at(p.xz), 2 * De, inv_perm, N, K,
                            2 * De, nullptr, 0, s));
  mark.done(ROM_STAGE_IN_PROJ);

  // short conv + SiLU, Eq. (2)
  float *conv_tmp = static_cast<float *>(at(p.conv_tmp));
  ROM_TRY(launch_conv_silu(d->dtype, at(p.xz), 2 * De, w->conv_w, w->conv_b, conv_in,
                           conv_out ? conv_tmp : nullptr, at(p.u), B, L, De, s));
  if (conv_out) {
    const int64_t n = B * De * 3;
    hipLaunchKernelGGL(copy_f32_kernel, dim3(static_cast<unsigned>(ceil_div(n, 256))), dim3(256), 0, s,
                       conv_tmp, conv_out, n);
    ROM_TRY(hipGetLastError());
  }
  mark.done(ROM_STAGE_CONV);

  // x projection -> dt_low | B | C
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.A = at(p.u); ga.lda = De; ga.a_span = N * De;
  ga.W = w->w_x; ga.N = R + 32; ga.K = De;
  ga.C = at(p.xdbl); ga.ldc = R + 32; ga.c_is_f32 = 1;
  const int64_t x_rows = routed_xdt ? S : N;
  ga.k_splits = xproj_k_splits(x_rows, routed_xdt ? E : 1, De);
  {   // the slice length is rounded up to whole 64-wide slabs: use the slice count that results
    const int64_t per = ceil_div(ceil_div(De, ga.k_splits), 64) * 64;
    ga.k_splits = static_cast<int>(ceil_div(De, per));
  }
  ga.c_split_stride = x_rows * (R + 32);
  if (routed_xdt) {
    ga.a_rows = tok_of_pos; ga.offsets = offsets; ga.n_groups = E; ga.M = S;
    ga.c_rows = multi ? nullptr : tok_of_pos;
  } else {
    ga.n_groups = 1; ga.M = N;
  }
  ROM_TRY(launch_grouped_gemm(ga, s));
  ROM_TRY(launch_split_xdbl(d->dtype, static_cast<const float *>(at(p.xdbl)), ga.k_splits, ga.c_split_stride,
                            (routed_xdt && multi) ? inv_perm : nullptr, K, N, R, at(p.dt_low),
                            static_cast<float *>(at(p.bc)), s));
  mark.done(ROM_STAGE_X_PROJ);

  // dt projection + bias + softplus
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.A = at(p.dt_low); ga.lda = R; ga.a_span = N * R;
  ga.W = w->w_dt; ga.N = De; ga.K = R;
  if (routed_xdt && multi) {
    ga.a_rows = tok_of_pos; ga.offsets = offsets; ga.n_groups = E; ga.M = S;
    ga.C = at(p.dt_raw); ga.ldc = De; ga.c_is_f32 = 1;
    ROM_TRY(launch_grouped_gemm(ga, s));
    ROM_TRY(launch_slot_sum(1, eb == 4, at(p.dt_raw), De, at(p.dt), De, inv_perm, N, K, De, w->dt_bias, 1, s));
  } else {
    if (routed_xdt) {
      ga.a_rows = tok_of_pos; ga.offsets = offsets; ga.n_groups = E; ga.M = S; ga.c_rows = tok_of_pos;
    } else {
      ga.n_groups = 1; ga.M = N;
    }
    ga.C = at(p.dt); ga.ldc = De; ga.bias = w->dt_bias; ga.softplus = 1;
    ROM_TRY(launch_grouped_gemm(ga, s));
  }
  mark.done(ROM_STAGE_DT_PROJ);

  // selective scan + D skip + SiLU(z) gate, Eq. (5), (6)
  const char *z = static_cast<const char *>(at(p.xz)) + static_cast<size_t>(De) * eb;
  ROM_TRY(launch_scan_gate(d->dtype, at(p.u), at(p.dt), static_cast<const float *>(at(p.bc)), z, 2 * De,
                           w->A_log, w->D, ssm_in, ssm_out, at(p.g), B, L, De,
                           static_cast<float *>(at(p.scan_q)), static_cast<float *>(at(p.scan_p)), s));
  mark.done(ROM_STAGE_SCAN);

  // out projection, Eq. (13), and the gate-weighted combine, Eq. (12)
  memset(&ga, 0, sizeof(ga));
  ga.dtype = d->dtype;
  ga.A = at(p.g); ga.lda = De; ga.a_rows = tok_of_pos; ga.a_span = N * De;
  ga.W = w->w_out; ga.offsets = offsets; ga.n_groups = E;
  ga.M = S; ga.N = Dm; ga.K = De;
  if (multi) {
    ga.C = at(p.op_sorted); ga.ldc = Dm;
    ROM_TRY(launch_grouped_gemm(ga, s));
    mark.done(ROM_STAGE_OUT_PROJ);
    ROM_TRY(launch_combine(d->dtype, at(p.op_sorted), inv_perm, gate, out, N, K, Dm, s));
    mark.done(ROM_STAGE_COMBINE);
  } else {
    ga.C = out; ga.ldc = Dm; ga.c_rows = tok_of_pos; ga.row_scale = gate;   // gate[n*1 + 0]
    ROM_TRY(launch_grouped_gemm(ga, s));
    mark.done(ROM_STAGE_OUT_PROJ);
    mark.done(ROM_STAGE_COMBINE);
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
  Plan p = make_plan(dims, N, 1);
  if (ws_bytes < p.total) return ROM_E_WORKSPACE;
  char *base = static_cast<char *>(ws);
  return route_into(dims, w, x, N, expert_idx, gate, counts, offsets, perm, inv_perm,
                    reinterpret_cast<int32_t *>(base + p.tok_of_pos),
                    reinterpret_cast<int32_t *>(base + p.block_counts), logits,
                    static_cast<hipStream_t>(hip_stream), nullptr);
}

int rom_layer_forward(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B, int64_t L,
                      const float *conv_state_in, const float *ssm_state_in, void *out,
                      float *conv_state_out, float *ssm_state_out, void *ws, size_t ws_bytes,
                      void *hip_stream) {
  return forward_impl(dims, w, x, B, L, conv_state_in, ssm_state_in, out, conv_state_out,
                      ssm_state_out, ws, ws_bytes, static_cast<hipStream_t>(hip_stream));
}

int rom_step(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B, float *conv_state,
             float *ssm_state, void *out, void *ws, size_t ws_bytes, void *hip_stream) {
  if (B > 0 && (!conv_state || !ssm_state)) return ROM_E_INVAL;
  return forward_impl(dims, w, x, B, 1, conv_state, ssm_state, out, conv_state, ssm_state, ws, ws_bytes,
                      static_cast<hipStream_t>(hip_stream));
}

const char *rom_strerror(int code) {
  switch (code) {
    case ROM_OK: return "ok";
    case ROM_E_INVAL: return "invalid argument (NULL or misaligned pointer, bad enum or size)";
    case ROM_E_WORKSPACE: return "workspace too small (see rom_workspace_bytes)";
    case ROM_E_UNSUPPORTED: return "shape not supported by this build (see rom_dims)";
    case ROM_E_HIP: return "a HIP call or kernel launch failed";
    default: return "unknown error code";
  }
}

int rom_profile_enable(int max_calls) {
  if (g_prof.ev) {
    for (int i = 0; i < g_prof.max_calls * (ROM_STAGE_COUNT + 1); ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    g_prof.ev = nullptr;
  }
  g_prof.max_calls = 0;
  g_prof.n_calls = 0;
  if (max_calls <= 0) return ROM_OK;
  const int n = max_calls * (ROM_STAGE_COUNT + 1);
  g_prof.ev = new hipEvent_t[n];
  for (int i = 0; i < n; ++i)
    if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) return ROM_E_HIP;
  g_prof.max_calls = max_calls;
  return ROM_OK;
}

int rom_profile_collect(double *stage_ms, int *n_calls) {
  if (!stage_ms || !n_calls) return ROM_E_INVAL;
  for (int i = 0; i < ROM_STAGE_COUNT; ++i) stage_ms[i] = 0.0;
  *n_calls = g_prof.n_calls;
  for (int c = 0; c < g_prof.n_calls; ++c) {
    hipEvent_t *ev = g_prof.ev + c * (ROM_STAGE_COUNT + 1);
    if (hipEventSynchronize(ev[ROM_STAGE_COUNT]) != hipSuccess) return ROM_E_HIP;
    for (int i = 0; i < ROM_STAGE_COUNT; ++i) {
      float ms = 0.0f;
      if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) return ROM_E_HIP;
      stage_ms[i] += ms;
    }
  }
  g_prof.n_calls = 0;
  return ROM_OK;
}

const char *rom_stage_name(int stage) {
  static const char *names[ROM_STAGE_COUNT] = {"route", "permute", "in_proj", "conv", "x_proj",
                                               "dt_proj", "scan_gate", "out_proj", "combine"};
  return (stage >= 0 && stage < ROM_STAGE_COUNT) ? names[stage] : "?";
}

}  // extern "C"
