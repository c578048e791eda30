// Router (Eq. (9)) and expert grouping for the RoM layer: logits, top-K on logits, softmax
// gates, then a stable counting sort of the (token, k) slots by expert built from wavefront
// ballots and prefix sums (no atomics, so the permutation is reproducible bit for bit).
#include "rom_internal.h"

#include <atomic>
#include <cstdint>
#include <mutex>
#include <type_traits>

namespace rom {

namespace {

constexpr int kWave = 64;

// Wave-wide reductions that leave the result in every lane: the four steps inside a row of 16
// lanes are DPP operands of the add / max itself (no LDS crossbar, no extra instruction), the two
// steps across rows go through the permute network.  Any lane order gives the same maximum; the
// sum is the same in every lane because every step adds the same two partial sums in both partners.
template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<0xB1>(v);      // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);      // quad_perm [2,3,0,1]
  v += dpp_f<0x141>(v);     // row_half_mirror: quads 0 <-> 1, 2 <-> 3
  v += dpp_f<0x140>(v);     // row_mirror: halves of the row
  v += __shfl_xor(v, 16, kWave);
  v += __shfl_xor(v, 32, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f<0xB1>(v));
  v = fmaxf(v, dpp_f<0x4E>(v));
  v = fmaxf(v, dpp_f<0x141>(v));
  v = fmaxf(v, dpp_f<0x140>(v));
  v = fmaxf(v, __shfl_xor(v, 16, kWave));
  v = fmaxf(v, __shfl_xor(v, 32, kWave));
  return v;
}

template <typename T> struct Vec8;  // 8 consecutive elements
template <> struct Vec8<bf16_t> {
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t *p) { raw = *reinterpret_cast<const uint4 *>(p); }
  __device__ __forceinline__ float get(int i) const {
    unsigned int w = (&raw.x)[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xFFFF0000u) : (w << 16));
  }
};
template <> struct Vec8<float> {
  float4 lo, hi;
  __device__ __forceinline__ void load(const float *p) {
    lo = *reinterpret_cast<const float4 *>(p);
    hi = *reinterpret_cast<const float4 *>(p + 4);
  }
  __device__ __forceinline__ float get(int i) const { return i < 4 ? (&lo.x)[i] : (&hi.x)[i - 4]; }
};

// WPT wavefronts handle TOK consecutive tokens: lanes stride over d_model in chunks of 8, each
// lane keeps TOK x EMAX partial dot products, a fixed butterfly sums them (and, for WPT = 4, the
// four waves of the block hand their sums to wave 0 through LDS, added in wave order).
// Lane e then owns logit e of each token and the wave does K arg-max rounds by ballot.
// WPT = 4 is for launches with few tokens (the recurrent step): one token per wave would leave
// most of the chip idle behind a long chain of dependent loads.
// NORM: the router sees the RMS-normalised input x * rstd * norm_w of a pre-norm block.  The
// per-token sum of squares rides along with the dot products (x is read once either way),
// rstd = 1 / sqrt(mean(x^2) + eps) multiplies the finished sums and is written out for the in
// projection's epilogue.
// ROUNDS > 0 (launches with many tokens, WPT = 1): the block first copies the router weights into
// LDS and every wave then handles ROUNDS consecutive groups of TOK tokens, reading the weights from
// there instead of pulling all E rows through the CU's vector L1 once per token group.  Same
// summation order, same bits.  Measured at 16K tokens x d_model 2048, 8 experts: 33.6 us with the
// weights in global memory (4 tokens per wave), 30.0 with them in LDS (2 tokens x 2 rounds); more
// rounds or tokens per wave (fewer waves) are slower (4 x 4: 51 us, 1 x 8: 45 us), and requesting
// the x rows one slice ahead changes nothing.  What remains is the read of x itself at 2.2 TB/s:
// x was last touched a whole layer call earlier and comes from HBM proper, not the infinity cache.
template <typename T, int EMAX, int TOK, int WPT, bool NORM, int ROUNDS = 0>
__global__ __launch_bounds__(256) void route_topk_kernel(
    const T *__restrict__ x, const T *__restrict__ w_router, const float *__restrict__ b_router,
    int64_t n_tokens, int d_model, int n_experts, int top_k, int gate_mode,
    int32_t *__restrict__ expert_idx, float *__restrict__ gate, float *__restrict__ logits,
    const float *__restrict__ norm_w, float norm_eps, float *__restrict__ rstd_out) {
  static_assert(WPT == 1 || WPT == 4, "one wave or one block per token group");
  static_assert(ROUNDS == 0 || WPT == 1, "weights in LDS: one wave per token group");
  __shared__ float part[WPT == 4 ? 4 * TOK * (EMAX + 1) : 1];   // [wave][token][EMAX sums | sum of squares]
  extern __shared__ __attribute__((aligned(16))) uint4 w_lds[];  // ROUNDS > 0: [n_experts][d_model] of T
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (ROUNDS > 0) {
    const int n_vec = n_experts * d_model / (16 / static_cast<int>(sizeof(T)));
    const uint4 *src = reinterpret_cast<const uint4 *>(w_router);
    for (int i = threadIdx.x; i < n_vec; i += blockDim.x) w_lds[i] = src[i];
    __syncthreads();
  }
  const T *w_src = ROUNDS > 0 ? reinterpret_cast<const T *>(w_lds) : w_router;
#pragma unroll 1
  for (int round = 0; round < (ROUNDS > 0 ? ROUNDS : 1); ++round) {
  const int64_t wave_id = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) / kWave;
  const int64_t group_id = WPT == 4 ? static_cast<int64_t>(blockIdx.x)
                                    : (ROUNDS > 0 ? wave_id * ROUNDS + round : wave_id);
  const int64_t tok0 = group_id * TOK;
  if (tok0 >= n_tokens) return;          // whole block (WPT = 4) or whole wave (its later rounds lie further still)

  float acc[TOK][EMAX];
#pragma unroll
  for (int t = 0; t < TOK; ++t)
#pragma unroll
    for (int e = 0; e < EMAX; ++e) acc[t][e] = 0.0f;
  float ss[TOK];
#pragma unroll
  for (int t = 0; t < TOK; ++t) ss[t] = 0.0f;

  const int first = (WPT == 4 ? wave * kWave + lane : lane) * 8;
  constexpr int kStride = WPT * kWave * 8;
  // the x rows of the next slice of d_model are requested before this slice is multiplied
  Vec8<T> xn[TOK];
  if (first < d_model) {
#pragma unroll
    for (int t = 0; t < TOK; ++t) {
      const int64_t tok = (tok0 + t < n_tokens) ? tok0 + t : n_tokens - 1;
      xn[t].load(x + tok * d_model + first);
    }
  }
  for (int d0 = first; d0 < d_model; d0 += kStride) {
    Vec8<T> xv[TOK];
#pragma unroll
    for (int t = 0; t < TOK; ++t) xv[t] = xn[t];
    if (d0 + kStride < d_model) {
#pragma unroll
      for (int t = 0; t < TOK; ++t) {
        const int64_t tok = (tok0 + t < n_tokens) ? tok0 + t : n_tokens - 1;
        xn[t].load(x + tok * d_model + d0 + kStride);
      }
    }
    float xs[TOK][8];
    if (NORM) {
      Vec8<float> nw;
      nw.load(norm_w + d0);
#pragma unroll
      for (int t = 0; t < TOK; ++t)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float xf = xv[t].get(i);
          ss[t] = fmaf(xf, xf, ss[t]);
          xs[t][i] = xf * nw.get(i);
        }
    } else {
#pragma unroll
      for (int t = 0; t < TOK; ++t)
#pragma unroll
        for (int i = 0; i < 8; ++i) xs[t][i] = xv[t].get(i);
    }
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
      if (e < n_experts) {
        Vec8<T> wv;
        wv.load(w_src + static_cast<int64_t>(e) * d_model + d0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float wf = wv.get(i);
#pragma unroll
          for (int t = 0; t < TOK; ++t) acc[t][e] = fmaf(xs[t][i], wf, acc[t][e]);
        }
      }
    }
  }

  if (WPT == 4) {
#pragma unroll
    for (int t = 0; t < TOK; ++t) {
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        const float s = wave_sum(acc[t][e]);
        if (lane == 0) part[(wave * TOK + t) * (EMAX + 1) + e] = s;
      }
      if (NORM) {
        const float s = wave_sum(ss[t]);
        if (lane == 0) part[(wave * TOK + t) * (EMAX + 1) + EMAX] = s;
      }
    }
    __syncthreads();
    if (wave != 0) return;
  }

#pragma unroll
  for (int t = 0; t < TOK; ++t) {
    const int64_t tok = tok0 + t;
    float rstd = 1.0f;
    if (NORM) {
      float sq;
      if (WPT == 4) {
        sq = part[t * (EMAX + 1) + EMAX];
#pragma unroll
        for (int w = 1; w < 4; ++w) sq += part[(w * TOK + t) * (EMAX + 1) + EMAX];
      } else {
        sq = wave_sum(ss[t]);
      }
      rstd = 1.0f / sqrtf(sq / static_cast<float>(d_model) + norm_eps);
      if (lane == 0 && tok < n_tokens) rstd_out[tok] = rstd;
    }
    // lane e keeps logit e
    float mine = -INFINITY;
    if (WPT == 4) {
      if (lane < n_experts && lane < EMAX) {
        float s = part[t * (EMAX + 1) + lane];
#pragma unroll
        for (int w = 1; w < 4; ++w) s += part[(w * TOK + t) * (EMAX + 1) + lane];
        mine = s * rstd + (b_router ? b_router[lane] : 0.0f);
      }
    } else {
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        const float s = wave_sum(acc[t][e]);
        if (lane == e && e < n_experts) mine = s * rstd + (b_router ? b_router[e] : 0.0f);
      }
    }
    if (tok >= n_tokens) continue;
    if (logits && lane < n_experts) logits[tok * n_experts + lane] = mine;

    const float lmax = wave_max(mine);
    const float p_un = (lane < n_experts) ? __expf(mine - lmax) : 0.0f;
    const float denom = wave_sum(p_un);

    // K rounds of arg-max over the experts not yet picked.  The picked set is kept apart from
    // the values, and a round in which no candidate compares equal to the maximum (NaN logits:
    // the max drops them) or every candidate sits at -inf (a masking bias) takes the lowest
    // candidate, so that every round names a valid expert and the K picks are distinct - the
    // grouping kernels index arrays with them.  A NaN logit still gives a NaN gate and a NaN
    // output row for that token, nothing worse.
    bool picked = false;
    float my_gate = 0.0f;       // lane k ends up with the gate of the k-th pick
    int my_pick = 0;
    float picked_sum = 0.0f;
    for (int k = 0; k < top_k; ++k) {
      const bool cand = lane < n_experts && !picked;
      const float best = wave_max(cand ? mine : -INFINITY);
      unsigned long long hit = __ballot(cand && mine == best);
      if (hit == 0ull) hit = __ballot(cand);
      const int e_sel = __ffsll(static_cast<long long>(hit)) - 1;   // lowest index wins ties
      const float p_sel = __shfl(p_un, e_sel, kWave);
      picked_sum += p_sel;
      if (lane == k) { my_pick = e_sel; my_gate = p_sel; }
      if (lane == e_sel) picked = true;
    }
    if (lane < top_k) {
      const float norm = (gate_mode == 1) ? picked_sum : denom;
      expert_idx[tok * top_k + lane] = my_pick;
      gate[tok * top_k + lane] = my_gate / norm;
    }
  }
  }   // rounds
}

// Router for launches with many bf16 tokens and up to 16 experts: the logits x W_r^T (Eq. (9)) as
// 16 x 16 x 32 MFMA tiles, fp32 accumulation.  The per-lane version above converts and multiplies
// every weight in the vector ALU (E x d_model fused multiply-adds and as many conversions per
// token) and reads x at 2.4 TB/s; here x goes from global memory straight into the A fragments
// (a lane's 16 bytes are 8 consecutive features of one token, the four lanes of a token cover 64
// contiguous bytes) and the only work per 16 tokens x 32 features is one LDS read and one MFMA, so
// the kernel is a stream over x: 16 fragments are requested while the previous 16 are multiplied.
// A wave owns 16 tokens; the router weights sit in LDS, one row per expert with a pitch of
// d_model + 8 elements (the rows a fragment read touches then start in different banks).  With
// EP = 8 the lanes of experts 8..15 read rows 0..7 again: columns past n_experts of the tile are
// never looked at.  The 16 x 16 tile of logits is parked in LDS and one lane per token runs the
// same selection as above over its E values: K rounds of arg-max over the experts not yet picked,
// lowest index on ties, a round without a candidate equal to the maximum (NaN logits) takes the
// lowest candidate.  Measured at 16K tokens x d_model 2048, 8 experts: 22.6 us against 27.4.
// (The same with a workgroup per 16 tokens, its four waves a quarter of d_model each and the
// weights read from global memory - every byte of x requested at once - measured 33.6 us: the
// weight fragments then cost the vector L1 as many requests as x itself.  Two waves per workgroup
// instead of four, so that one workgroup's weight copy overlaps another's stream: 26.0 us.)
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 route_bf16x8_t;
typedef float route_f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int route_u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kRouteMfmaBatch = 16;     // fragments of x requested together (16 x 16 bytes per lane)
constexpr int kRouteMfmaWaves = 4;
constexpr size_t kRouteMfmaLdsMax = 160 * 1024;

constexpr size_t route_mfma_lds_bytes(int ep, int d_model, bool norm) {
  return static_cast<size_t>(norm ? 3 : 1) * ep * (d_model + 8) * 2 + kRouteMfmaWaves * 16 * (17 + 1) * sizeof(float);
}

// NORM (the pre-norm block's router): the logits of x * rstd * norm_w.  norm_w is multiplied into the
// weights while they are copied to LDS, in fp32, and the product is kept as three bf16 pieces (8 + 8 + 8
// bits of the fp32 significand: the sum of the pieces is the product to within its last bit) in three planes; a step then issues three MFMAs on the same
// fragment of x - the matrix pipe has the room.  The sum of squares of a token rides along in the
// vector ALU on the fragments the lanes hold anyway; rstd = 1 / sqrt(mean(x^2) + eps) scales the
// finished sums and is written out for the in projection's epilogue.
template <int EP, bool NORM>
__global__ __launch_bounds__(kRouteMfmaWaves *kWave) void route_mfma_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ w_router, const float *__restrict__ b_router,
    int64_t n_tokens, int d_model, int n_experts, int top_k, int gate_mode,
    int32_t *__restrict__ expert_idx, float *__restrict__ gate, float *__restrict__ logits,
    const float *__restrict__ norm_w, float norm_eps, float *__restrict__ rstd_out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char route_lds[];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int cq = lane & 15, gq = lane >> 4;
  const int pitch = (d_model + 8) * 2;                    // bytes
  constexpr int kPlanes = NORM ? 3 : 1;
  const int plane = EP * pitch;
  float(*tile)[17] = reinterpret_cast<float(*)[17]>(route_lds + static_cast<size_t>(kPlanes) * plane) + wave * 16;
  float *rs = reinterpret_cast<float *>(route_lds + static_cast<size_t>(kPlanes) * plane) + kRouteMfmaWaves * 16 * 17 + wave * 16;

  const int64_t tok0 = (static_cast<int64_t>(blockIdx.x) * kRouteMfmaWaves + wave) * 16;
  // (a wave past the end walks the last token again and stores nothing: no barrier is skipped)
  const int64_t tok_ld = (tok0 + cq < n_tokens) ? tok0 + cq : n_tokens - 1;
  const route_u32x4_t *xp = reinterpret_cast<const route_u32x4_t *>(x + tok_ld * d_model + 8 * gq);
  const unsigned char *wp = route_lds + (cq % EP) * pitch + 16 * gq;
  const int n_steps = d_model / 32;                       // one MFMA each; a step is 4 vectors further along the row

  // the first fragments of x are requested before the weights are copied: the copy hides their latency
  route_u32x4_t cur[kRouteMfmaBatch], nxt[kRouteMfmaBatch];
  const int n_batches = n_steps / kRouteMfmaBatch;
#pragma unroll
  for (int u = 0; u < kRouteMfmaBatch; ++u) {
    nxt[u] = route_u32x4_t{0u, 0u, 0u, 0u};
    if (n_batches > 0) cur[u] = __builtin_nontemporal_load(xp + 4 * u);
  }

  {
    const int chunks = d_model / 8;                       // 16-byte pieces per row
    const uint4 *src = reinterpret_cast<const uint4 *>(w_router);
    for (int i = threadIdx.x; i < EP * chunks; i += blockDim.x) {
      const int n = i / chunks, c = i - n * chunks;
      uint4 v = {0u, 0u, 0u, 0u};
      if (n < n_experts) v = src[static_cast<int64_t>(n) * chunks + c];
      if (!NORM) {
        *reinterpret_cast<uint4 *>(route_lds + n * pitch + c * 16) = v;
      } else {
        const float4 n0 = *reinterpret_cast<const float4 *>(norm_w + c * 8);
        const float4 n1 = *reinterpret_cast<const float4 *>(norm_w + c * 8 + 4);
        const float nw[8] = {n0.x, n0.y, n0.z, n0.w, n1.x, n1.y, n1.z, n1.w};
        const unsigned int *vw = &v.x;
        unsigned int hi[4], mid[4], lo[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float f[2] = {__uint_as_float(vw[q] << 16) * nw[2 * q], __uint_as_float(vw[q] & 0xFFFF0000u) * nw[2 * q + 1]};
          unsigned int piece[3][2];
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const bf16_t a = f32_to_bf16(f[h]);
            const float r1 = f[h] - bf16_to_f32(a);            // exact: what the first 8 bits leave
            const bf16_t b = f32_to_bf16(r1);
            const float r2 = r1 - bf16_to_f32(b);              // exact: what the next 8 bits leave
            piece[0][h] = a; piece[1][h] = b; piece[2][h] = f32_to_bf16(r2);
          }
          hi[q] = piece[0][0] | (piece[0][1] << 16);
          mid[q] = piece[1][0] | (piece[1][1] << 16);
          lo[q] = piece[2][0] | (piece[2][1] << 16);
        }
        unsigned char *dst = route_lds + n * pitch + c * 16;
        *reinterpret_cast<uint4 *>(dst) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        *reinterpret_cast<uint4 *>(dst + plane) = make_uint4(mid[0], mid[1], mid[2], mid[3]);
        *reinterpret_cast<uint4 *>(dst + 2 * plane) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
      }
    }
  }
  __syncthreads();

  route_f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
  float ss = 0.0f;                                        // NORM: this lane's share of the token's sum of squares
  auto step = [&](const route_u32x4_t &xv, int ks) {
#pragma unroll
    for (int pl = kPlanes - 1; pl >= 0; --pl) {           // smallest pieces first
      const route_u32x4_t wv = *reinterpret_cast<const route_u32x4_t *>(wp + pl * plane + ks * 64);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(route_bf16x8_t, xv),
                                                    __builtin_bit_cast(route_bf16x8_t, wv), acc, 0, 0, 0);
    }
    if (NORM) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = __uint_as_float(xv[q] << 16), b = __uint_as_float(xv[q] & 0xFFFF0000u);
        ss = fmaf(a, a, ss);
        ss = fmaf(b, b, ss);
      }
    }
  };
  for (int b = 0; b < n_batches; ++b) {
    if (b + 1 < n_batches) {
#pragma unroll
      for (int u = 0; u < kRouteMfmaBatch; ++u) nxt[u] = __builtin_nontemporal_load(xp + 4 * ((b + 1) * kRouteMfmaBatch + u));
    }
#pragma unroll
    for (int u = 0; u < kRouteMfmaBatch; ++u) step(cur[u], b * kRouteMfmaBatch + u);
#pragma unroll
    for (int u = 0; u < kRouteMfmaBatch; ++u) cur[u] = nxt[u];
  }
  for (int ks = n_batches * kRouteMfmaBatch; ks < n_steps; ++ks) {      // d_model / 32 not a multiple of the batch
    const route_u32x4_t xv = xp[4 * ks];
    step(xv, ks);
  }

  if (NORM) {
    // the four lanes of token cq add their shares; the scale goes to the lanes that hold the token's sums
    ss += __shfl_xor(ss, 16, kWave);
    ss += __shfl_xor(ss, 32, kWave);
    const float rstd = 1.0f / sqrtf(ss / static_cast<float>(d_model) + norm_eps);
    if (gq == 0) {
      rs[cq] = rstd;
      if (tok0 + cq < n_tokens) rstd_out[tok0 + cq] = rstd;
    }
    __syncthreads();
  }
  // lane (cq, gq) holds the logits of expert cq for the tokens 4 gq .. 4 gq + 3 of the tile
  const float bias = (b_router && cq < n_experts) ? b_router[cq] : 0.0f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float v = (NORM ? acc[r] * rs[4 * gq + r] : acc[r]) + bias;
    tile[4 * gq + r][cq] = v;
    const int64_t tok = tok0 + 4 * gq + r;
    if (logits && cq < n_experts && tok < n_tokens) logits[tok * n_experts + cq] = v;
  }
  __syncthreads();

  const int64_t tok = tok0 + lane;
  if (lane >= 16 || tok >= n_tokens) return;
  float v[EP], p[EP];
  float lmax = -INFINITY;
#pragma unroll
  for (int e = 0; e < EP; ++e) {
    v[e] = (e < n_experts) ? tile[lane][e] : -INFINITY;
    lmax = fmaxf(lmax, v[e]);
  }
  float denom = 0.0f;
#pragma unroll
  for (int e = 0; e < EP; ++e) {
    p[e] = (e < n_experts) ? __expf(v[e] - lmax) : 0.0f;
    denom += p[e];
  }
  // first walk of the K rounds: the sum of the picked probabilities (the gate's normaliser when
  // gate_mode = 1); second walk: the same rounds again, now writing
  float picked_sum = 0.0f;
  for (int pass = 0; pass < 2; ++pass) {
    unsigned picked = 0u;
    const float norm = (gate_mode == 1) ? picked_sum : denom;
    for (int k = 0; k < top_k; ++k) {
      float best = -INFINITY;
#pragma unroll
      for (int e = 0; e < EP; ++e)
        if (e < n_experts && !(picked >> e & 1u)) best = fmaxf(best, v[e]);
      int sel = -1, low = -1;
      float p_sel = 0.0f, p_low = 0.0f;
#pragma unroll
      for (int e = EP - 1; e >= 0; --e) {
        const bool cand = e < n_experts && !(picked >> e & 1u);
        if (cand) { low = e; p_low = p[e]; }
        if (cand && v[e] == best) { sel = e; p_sel = p[e]; }
      }
      if (sel < 0) { sel = low; p_sel = p_low; }
      if (sel < 0) sel = 0;                              // (top_k > n_experts is refused by the host)
      picked |= 1u << sel;
      if (pass == 0) {
        picked_sum += p_sel;
      } else {
        expert_idx[tok * top_k + k] = sel;
        gate[tok * top_k + k] = p_sel / norm;
      }
    }
  }
}

// more than 64 KiB of dynamic LDS needs a function attribute, set once per device
template <int EP, bool NORM> hipError_t route_mfma_allow_lds() {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static std::atomic<bool> done[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
  std::lock_guard<std::mutex> lock(mu);
  if (done[dev].load(std::memory_order_relaxed)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&route_mfma_kernel<EP, NORM>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kRouteMfmaLdsMax));
  if (e == hipSuccess) done[dev].store(true, std::memory_order_release);
  return e;
}

// ------------------------------------------------------------------ stable grouping
constexpr int kSortBlock = 256;   // slots per block, one per thread
constexpr int kSortWaves = kSortBlock / kWave;

// per-wave population count of every expert among this wave's slots, via ballots
__device__ __forceinline__ unsigned long long match_expert(int key, int n_experts, int lane,
                                                           int *wave_counts /* LDS [E] or NULL */) {
  unsigned long long mine = 0ull;
  for (int e = 0; e < n_experts; ++e) {
    const unsigned long long m = __ballot(key == e);
    if (key == e) mine = m;
    if (wave_counts && lane == 0) wave_counts[e] = __popcll(m);
  }
  return mine;
}

// The three grouping kernels sort n_items keys; item s has the key expert_idx[s * stride + r] with
// r = blockIdx.y (hist, scatter) or blockIdx.x (offsets).  stride 1, one rank: all N*K slots by
// expert.  stride K, K ranks: for every rank r the N tokens by their r-th expert (the K > 1 path of
// the layer runs a routed projection as K passes over the tokens, one per rank).  Per-rank arrays
// follow one another: block_counts [rank][block][E], offsets [rank][E + 1] (each starting at 0),
// tok_of_pos [rank][n_items].
__global__ __launch_bounds__(kSortBlock) void hist_kernel(const int32_t *__restrict__ expert_idx,
                                                          int64_t n_items, int n_experts, int stride,
                                                          int32_t *__restrict__ block_counts) {
  __shared__ int cnt[kSortWaves][64];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t s = static_cast<int64_t>(blockIdx.x) * kSortBlock + threadIdx.x;
  const int key = (s < n_items) ? expert_idx[s * stride + blockIdx.y] : -1;
  match_expert(key, n_experts, lane, cnt[wave]);
  __syncthreads();
  if (threadIdx.x < n_experts) {
    int total = 0;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) total += cnt[w][threadIdx.x];
    block_counts[(static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * n_experts + threadIdx.x] = total;
  }
}

// One block of up to 16 waves: wave w turns block_counts[:, e] for e = w, w + 16, ... into an
// exclusive prefix over blocks, 64 blocks at a time with a wave-wide scan; thread 0 then builds
// counts / offsets.
constexpr int kOffsetWaves = 16;
__global__ __launch_bounds__(kOffsetWaves *kWave) void offsets_kernel(int32_t *__restrict__ block_counts,
                                                                      int64_t n_blocks, int n_experts,
                                                                      int32_t *__restrict__ counts,
                                                                      int32_t *__restrict__ offsets) {
  __shared__ int total[64];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int n_waves = blockDim.x / kWave;
  block_counts += static_cast<int64_t>(blockIdx.x) * n_blocks * n_experts;      // this rank's arrays
  offsets += blockIdx.x * (n_experts + 1);
  if (counts) counts += blockIdx.x * n_experts;
  for (int e = wave; e < n_experts; e += n_waves) {
    int run = 0;
    for (int64_t b0 = 0; b0 < n_blocks; b0 += kWave) {
      const int64_t b = b0 + lane;
      const int c = b < n_blocks ? block_counts[b * n_experts + e] : 0;
      int incl = c;
#pragma unroll
      for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
      }
      if (b < n_blocks) block_counts[b * n_experts + e] = run + incl - c;
      run += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) {
      total[e] = run;
      if (counts) counts[e] = run;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < n_experts; ++i) { offsets[i] = run; run += total[i]; }
    offsets[n_experts] = run;
  }
}

// perm / inv_perm may be NULL (the per-rank groupings need the row map alone); tok_of_pos[pos] = s / tok_div
__global__ __launch_bounds__(kSortBlock) void scatter_kernel(
    const int32_t *__restrict__ expert_idx, int64_t n_items, int n_experts, int stride, int tok_div,
    const int32_t *__restrict__ block_base, const int32_t *__restrict__ offsets,
    int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm, int32_t *__restrict__ tok_of_pos) {
  __shared__ int cnt[kSortWaves][64];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t s = static_cast<int64_t>(blockIdx.x) * kSortBlock + threadIdx.x;
  const int key = (s < n_items) ? expert_idx[s * stride + blockIdx.y] : -1;
  const unsigned long long same = match_expert(key, n_experts, lane, cnt[wave]);
  __syncthreads();
  if (s >= n_items || key < 0 || key >= n_experts) return;      // (a key outside [0, E) is never written by the router)
  const unsigned long long below = same & ((1ull << lane) - 1ull);
  offsets += blockIdx.y * (n_experts + 1);
  int pos = offsets[key] + block_base[(static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * n_experts + key] +
            __popcll(below);
  for (int w = 0; w < wave; ++w) pos += cnt[w][key];
  if (inv_perm) inv_perm[s] = pos;
  if (perm) perm[pos] = static_cast<int32_t>(s);
  tok_of_pos[static_cast<int64_t>(blockIdx.y) * n_items + pos] = static_cast<int32_t>(s / tok_div);
}

// Whole grouping in one workgroup for small slot counts (decode steps): three passes over the
// slots in rounds of 256, counts and running bases in LDS.
__global__ __launch_bounds__(kSortBlock) void permutation_small_kernel(
    const int32_t *__restrict__ expert_idx, int n_slots, int n_experts, int top_k,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv_perm, int32_t *__restrict__ tok_of_pos) {
  __shared__ int cnt[kSortWaves][64];
  __shared__ int base[64];          // running position of every expert
  __shared__ int total[64];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (threadIdx.x < 64) total[threadIdx.x] = 0;
  __syncthreads();
  for (int s0 = 0; s0 < n_slots; s0 += kSortBlock) {      // histogram
    const int s = s0 + threadIdx.x;
    match_expert(s < n_slots ? expert_idx[s] : -1, n_experts, lane, cnt[wave]);
    __syncthreads();
    if (threadIdx.x < n_experts) {
      int t = 0;
#pragma unroll
      for (int w = 0; w < kSortWaves; ++w) t += cnt[w][threadIdx.x];
      total[threadIdx.x] += t;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    int run = 0;
    for (int e = 0; e < n_experts; ++e) {
      offsets[e] = run;
      base[e] = run;
      counts[e] = total[e];
      run += total[e];
    }
    offsets[n_experts] = run;
  }
  __syncthreads();
  for (int s0 = 0; s0 < n_slots; s0 += kSortBlock) {      // stable scatter
    const int s = s0 + threadIdx.x;
    const int key = s < n_slots ? expert_idx[s] : -1;
    const unsigned long long same = match_expert(key, n_experts, lane, cnt[wave]);
    __syncthreads();
    if (s < n_slots && key >= 0 && key < n_experts) {
      int pos = base[key] + __popcll(same & ((1ull << lane) - 1ull));
      for (int w = 0; w < wave; ++w) pos += cnt[w][key];
      inv_perm[s] = pos;
      perm[pos] = s;
      tok_of_pos[pos] = s / top_k;
    }
    __syncthreads();
    if (threadIdx.x < n_experts) {
      int t = 0;
#pragma unroll
      for (int w = 0; w < kSortWaves; ++w) t += cnt[w][threadIdx.x];
      base[threadIdx.x] += t;
    }
    __syncthreads();
  }
}

// Load-balance statistics, Eq. (16).  A wavefront holds 64 / EP tokens at a time (EP = the expert
// count rounded up to a power of two): lane = token_in_wave * EP + expert.  The softmax maximum
// and denominator are butterflies inside a group of EP lanes, and each lane keeps the running
// sum of its own expert's probability.  Blocks own fixed token ranges and their sums are added
// in block order by the second kernel, so the result is the same on every run.
constexpr int kBalanceBlock = 256;
constexpr int kBalanceMaxBlocks = 256;

__global__ __launch_bounds__(kBalanceBlock) void balance_partial_kernel(
    const float *__restrict__ logits, int64_t n_tokens, int n_experts, int ep,
    float *__restrict__ partial) {
  __shared__ float wave_part[kBalanceBlock / kWave][64];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int e = lane & (ep - 1);
  const int tok_per_wave = kWave / ep;
  const int64_t wave_id = static_cast<int64_t>(blockIdx.x) * (kBalanceBlock / kWave) + wave;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * (kBalanceBlock / kWave) * tok_per_wave;
  float acc = 0.0f;
  // every lane of the wave runs the same number of rounds (the shuffles need all of them)
  for (int64_t t0 = wave_id * tok_per_wave; t0 < n_tokens; t0 += stride) {
    const int64_t tok = t0 + lane / ep;
    const bool live = tok < n_tokens && e < n_experts;
    const float l = live ? logits[tok * n_experts + e] : -INFINITY;
    float m = l;
    for (int o = 1; o < ep; o <<= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
    // a group past the last token holds only -inf: keep exp's argument finite there
    const float p = live ? fast_exp2((l - m) * 1.44269504088896341f) : 0.0f;
    float den = p;
    for (int o = 1; o < ep; o <<= 1) den += __shfl_xor(den, o, kWave);
    if (live) acc += p / den;
  }
  for (int o = ep; o < kWave; o <<= 1) acc += __shfl_xor(acc, o, kWave);
  if (lane < ep) wave_part[wave][lane] = acc;
  __syncthreads();
  if (threadIdx.x < n_experts) {
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < kBalanceBlock / kWave; ++w) t += wave_part[w][threadIdx.x];
    partial[static_cast<int64_t>(blockIdx.x) * n_experts + threadIdx.x] = t;
  }
}

// One block of kFinishWaves wavefronts, lane = expert: wave w adds the block sums b = w, w + 16, ...
// in that order, wave 0 then adds the 16 wave sums in wave order - a fixed tree, so the result
// does not depend on timing, and no lane walks more than 16 dependent loads.
constexpr int kFinishWaves = 16;
__global__ __launch_bounds__(kFinishWaves * kWave) void balance_finish_kernel(
    const float *__restrict__ partial, int n_blocks, const int32_t *__restrict__ counts,
    int64_t n_tokens, int n_experts, int top_k, float alpha, float *__restrict__ frac,
    float *__restrict__ mean_prob, float *__restrict__ loss) {
  __shared__ float wave_part[kFinishWaves][kWave];
  const int e = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  float t = 0.0f;
  if (e < n_experts)
    for (int b = wave; b < n_blocks; b += kFinishWaves) t += partial[static_cast<int64_t>(b) * n_experts + e];
  wave_part[wave][e] = t;
  __syncthreads();
  if (wave != 0) return;
  float prod = 0.0f;
  if (e < n_experts) {
    float total = 0.0f;
#pragma unroll
    for (int w = 0; w < kFinishWaves; ++w) total += wave_part[w][e];
    const float pm = total / static_cast<float>(n_tokens);
    const float f = static_cast<float>(counts[e]) / (static_cast<float>(n_tokens) * static_cast<float>(top_k));
    frac[e] = f;
    mean_prob[e] = pm;
    prod = f * pm;
  }
  const float sum = wave_sum(prod);
  if (e == 0) *loss = alpha * static_cast<float>(n_experts) * sum;
}

template <typename T, bool NORM>
hipError_t route_dispatch(const void *x, const void *w_router, const float *b_router,
                          int64_t n_tokens, int d_model, int n_experts, int top_k, int gate_mode,
                          int32_t *expert_idx, float *gate, float *logits, const float *norm_w,
                          float norm_eps, float *rstd, hipStream_t s) {
  const T *xp = static_cast<const T *>(x);
  const T *wp = static_cast<const T *>(w_router);
  const size_t w_bytes = static_cast<size_t>(n_experts) * d_model * sizeof(T);
  constexpr size_t kRouteLdsMax = 48 * 1024;
  constexpr int kRouteRounds = 2;
#define ROM_ROUTE_LAUNCH(EMAX, TOK, WPT)                                                         \
  do {                                                                                           \
    const int64_t groups = ceil_div(n_tokens, TOK);                                              \
    const int64_t blocks = WPT == 4 ? groups : ceil_div(groups, 4);                              \
    hipLaunchKernelGGL((route_topk_kernel<T, EMAX, TOK, WPT, NORM>),                             \
                       dim3(static_cast<unsigned>(blocks)), dim3(256), 0, s, xp, wp, b_router,   \
                       n_tokens, d_model, n_experts, top_k, gate_mode, expert_idx, gate, logits, \
                       norm_w, norm_eps, rstd);                                                  \
  } while (0)
  // few tokens: one token per block / per wavefront so that the launch still spreads over the chip
  if (n_tokens <= 1024 && n_experts <= 8) ROM_ROUTE_LAUNCH(8, 1, 4);
  else if (n_tokens <= 1024 && n_experts <= 16) ROM_ROUTE_LAUNCH(16, 1, 4);
  else if (n_tokens <= 8192 && n_experts <= 8) ROM_ROUTE_LAUNCH(8, 1, 1);
  else if (n_tokens <= 8192 && n_experts <= 16) ROM_ROUTE_LAUNCH(16, 1, 1);
  // many tokens: router weights in LDS when they fit 48 KiB
#define ROM_ROUTE_LAUNCH_LDS(EMAX, TOK, ROUNDS)                                                   \
  do {                                                                                           \
    const int64_t blocks = ceil_div(ceil_div(n_tokens, TOK), 4 * ROUNDS);                        \
    hipLaunchKernelGGL((route_topk_kernel<T, EMAX, TOK, 1, NORM, ROUNDS>),                       \
                       dim3(static_cast<unsigned>(blocks)), dim3(256), w_bytes, s, xp, wp,       \
                       b_router, n_tokens, d_model, n_experts, top_k, gate_mode, expert_idx,     \
                       gate, logits, norm_w, norm_eps, rstd);                                    \
  } while (0)
  // bf16, up to 16 experts: the logits on the matrix pipe (with the pre-norm folded into the weights
  // three planes of them must fit the LDS)
#define ROM_ROUTE_LAUNCH_MFMA(EP)                                                                 \
  do {                                                                                           \
    const size_t lds = route_mfma_lds_bytes(EP, d_model, NORM);                                  \
    if (lds > 64 * 1024) {                                                                       \
      const hipError_t e = route_mfma_allow_lds<EP, NORM>();                                     \
      if (e != hipSuccess) return e;                                                             \
    }                                                                                            \
    const int64_t blocks = ceil_div(n_tokens, 16 * kRouteMfmaWaves);                             \
    hipLaunchKernelGGL((route_mfma_kernel<EP, NORM>), dim3(static_cast<unsigned>(blocks)),       \
                       dim3(kRouteMfmaWaves *kWave), lds, s, reinterpret_cast<const bf16_t *>(x), \
                       reinterpret_cast<const bf16_t *>(w_router), b_router, n_tokens, d_model,  \
                       n_experts, top_k, gate_mode, expert_idx, gate, logits, norm_w, norm_eps,  \
                       rstd);                                                                    \
  } while (0)
  else if (std::is_same<T, bf16_t>::value && n_experts <= 16 && d_model % 32 == 0 &&
           route_mfma_lds_bytes(n_experts <= 8 ? 8 : 16, d_model, NORM) <= kRouteMfmaLdsMax &&
           (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(w_router) & 15) == 0 &&
           (!NORM || (reinterpret_cast<uintptr_t>(norm_w) & 15) == 0)) {
    if (n_experts <= 8) ROM_ROUTE_LAUNCH_MFMA(8);
    else ROM_ROUTE_LAUNCH_MFMA(16);
  }
#undef ROM_ROUTE_LAUNCH_MFMA
  else if (n_experts <= 8 && w_bytes <= kRouteLdsMax) ROM_ROUTE_LAUNCH_LDS(8, 2, kRouteRounds);
  else if (n_experts <= 16 && w_bytes <= kRouteLdsMax) ROM_ROUTE_LAUNCH_LDS(16, 2, kRouteRounds);
#undef ROM_ROUTE_LAUNCH_LDS
  // (a block per token group with a quarter of d_model per wave, (8, 4, 4), measured no faster
  // here: the launch is bound by refilling L1 with the router weights, not by loads in flight)
  else if (n_experts <= 8) ROM_ROUTE_LAUNCH(8, 4, 1);
  else if (n_experts <= 16) ROM_ROUTE_LAUNCH(16, 2, 1);
  else if (n_experts <= 32) ROM_ROUTE_LAUNCH(32, 1, 1);
  else ROM_ROUTE_LAUNCH(64, 1, 1);
#undef ROM_ROUTE_LAUNCH
  return hipGetLastError();
}

}  // namespace

int64_t route_blocks(int64_t n_slots) { return ceil_div(n_slots, kSortBlock); }

hipError_t launch_route_topk(int dtype, const void *x, const void *w_router, const float *b_router,
                             int64_t n_tokens, int d_model, int n_experts, int top_k, int gate_mode,
                             int32_t *expert_idx, float *gate, float *logits, const float *norm_w,
                             float norm_eps, float *rstd, hipStream_t s) {
#define ROM_ROUTE_ARGS x, w_router, b_router, n_tokens, d_model, n_experts, top_k, gate_mode, expert_idx, gate, \
                       logits, norm_w, norm_eps, rstd, s
  if (norm_w)
    return dtype == ROM_DTYPE_BF16 ? route_dispatch<bf16_t, true>(ROM_ROUTE_ARGS)
                                   : route_dispatch<float, true>(ROM_ROUTE_ARGS);
  return dtype == ROM_DTYPE_BF16 ? route_dispatch<bf16_t, false>(ROM_ROUTE_ARGS)
                                 : route_dispatch<float, false>(ROM_ROUTE_ARGS);
#undef ROM_ROUTE_ARGS
}

size_t balance_scratch_bytes(int n_experts) {
  return static_cast<size_t>(kBalanceMaxBlocks) * static_cast<size_t>(n_experts) * sizeof(float);
}

hipError_t launch_balance_stats(const float *logits, const int32_t *counts, int64_t n_tokens,
                                int n_experts, int top_k, float alpha, float *partial, float *frac,
                                float *mean_prob, float *loss, hipStream_t s) {
  int ep = 1;
  while (ep < n_experts) ep <<= 1;
  const int64_t tok_per_block = (kBalanceBlock / kWave) * (kWave / ep);
  int64_t blocks = ceil_div(n_tokens, tok_per_block);
  if (blocks > kBalanceMaxBlocks) blocks = kBalanceMaxBlocks;
  hipLaunchKernelGGL(balance_partial_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kBalanceBlock), 0,
                     s, logits, n_tokens, n_experts, ep, partial);
  hipLaunchKernelGGL(balance_finish_kernel, dim3(1), dim3(kFinishWaves * kWave), 0, s, partial, static_cast<int>(blocks),
                     counts, n_tokens, n_experts, top_k, alpha, frac, mean_prob, loss);
  return hipGetLastError();
}

hipError_t launch_permutation(const int32_t *expert_idx, int64_t n_slots, int n_experts, int top_k,
                              int32_t *block_counts, int32_t *counts, int32_t *offsets,
                              int32_t *perm, int32_t *inv_perm, int32_t *tok_of_pos, hipStream_t s) {
  if (n_slots <= 2048) {
    hipLaunchKernelGGL(permutation_small_kernel, dim3(1), dim3(kSortBlock), 0, s, expert_idx,
                       static_cast<int>(n_slots), n_experts, top_k, counts, offsets, perm, inv_perm, tok_of_pos);
    return hipGetLastError();
  }
  const int64_t blocks = route_blocks(n_slots);
  hipLaunchKernelGGL(hist_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kSortBlock), 0, s,
                     expert_idx, n_slots, n_experts, 1, block_counts);
  const int offset_waves = n_experts < kOffsetWaves ? n_experts : kOffsetWaves;
  hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(offset_waves * kWave), 0, s, block_counts, blocks, n_experts,
                     counts, offsets);
  hipLaunchKernelGGL(scatter_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kSortBlock), 0, s,
                     expert_idx, n_slots, n_experts, 1, top_k, block_counts, offsets, perm, inv_perm,
                     tok_of_pos);
  return hipGetLastError();
}

size_t rank_grouping_block_counts_bytes(int64_t n_tokens, int n_experts, int top_k) {
  return static_cast<size_t>(top_k) * route_blocks(n_tokens) * n_experts * sizeof(int32_t);
}

hipError_t launch_rank_grouping(const int32_t *expert_idx, int64_t n_tokens, int n_experts, int top_k,
                                int32_t *block_counts, int32_t *rank_offsets, int32_t *tok_of_rank_pos,
                                hipStream_t s) {
  const int64_t blocks = route_blocks(n_tokens);
  const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(top_k));
  hipLaunchKernelGGL(hist_kernel, grid, dim3(kSortBlock), 0, s, expert_idx, n_tokens, n_experts, top_k, block_counts);
  const int offset_waves = n_experts < kOffsetWaves ? n_experts : kOffsetWaves;
  hipLaunchKernelGGL(offsets_kernel, dim3(static_cast<unsigned>(top_k)), dim3(offset_waves * kWave), 0, s, block_counts,
                     blocks, n_experts, static_cast<int32_t *>(nullptr), rank_offsets);
  hipLaunchKernelGGL(scatter_kernel, grid, dim3(kSortBlock), 0, s, expert_idx, n_tokens, n_experts, top_k, 1,
                     block_counts, rank_offsets, static_cast<int32_t *>(nullptr), static_cast<int32_t *>(nullptr),
                     tok_of_rank_pos);
  return hipGetLastError();
}

}  // namespace rom
