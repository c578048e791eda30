// Sequence-mixing and elementwise kernels of the RoM layer:
//   causal depthwise conv + SiLU (Eq. (2)), selective scan with D skip and SiLU(z) gating
//   (Eq. (5), (6)/(13)), the per-token sums over the K selected experts (Eq. (10)/(11)) and the
//   gate-weighted combine (Eq. (12)), plus the small helpers of the FFN-MoE layer (row map,
//   1 / rms per routed row, SwiGLU for fp32).  All of this is bandwidth / plain-ALU work: no MFMA here.
#include "rom_internal.h"

namespace rom {

namespace {

// ------------------------------------------------------------------ small vector helpers
// Global loads of 8 / 16 bytes go through native vector types:
// assigning HIP's uint4 / float4 structs from memory is a memcpy into the register struct, which
// keeps a struct that lives across the tile loop in scratch memory.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4v_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_u4(const void *p) {
  const u32x4_t v = *static_cast<const u32x4_t *>(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 ld_u2(const void *p) {
  const u32x2_t v = *static_cast<const u32x2_t *>(p);
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ float4 ld_f4(const void *p) {
  const f32x4v_t v = *static_cast<const f32x4v_t *>(p);
  return make_float4(v.x, v.y, v.z, v.w);
}
template <typename T> struct Chunk;           // 16 bytes of T
template <> struct Chunk<bf16_t> {
  static constexpr int kElems = 8;
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t *p) { raw = ld_u4(p); }
  __device__ __forceinline__ void store(bf16_t *p) const { *reinterpret_cast<uint4 *>(p) = raw; }
  __device__ __forceinline__ float get(int i) const {
    const unsigned int w = (&raw.x)[i >> 1];
    return __uint_as_float((i & 1) ? (w & 0xFFFF0000u) : (w << 16));
  }
  __device__ __forceinline__ void set_pair(int i, float lo, float hi) {   // elements 2i, 2i+1
    (&raw.x)[i] = pack_bf16x2(lo, hi);
  }
};
template <> struct Chunk<float> {
  static constexpr int kElems = 4;
  float4 raw;
  __device__ __forceinline__ void load(const float *p) { raw = ld_f4(p); }
  __device__ __forceinline__ void store(float *p) const { *reinterpret_cast<float4 *>(p) = raw; }
  __device__ __forceinline__ float get(int i) const { return (&raw.x)[i]; }
  __device__ __forceinline__ void set_pair(int i, float lo, float hi) {
    (&raw.x)[2 * i] = lo;
    (&raw.x)[2 * i + 1] = hi;
  }
};

__device__ __forceinline__ float softplus_f32(float v) {
  // log(1 + exp(v)) without overflow; for v > 20 the correction is below fp32 resolution
  return v > 20.0f ? v : log1pf(__expf(v));
}

// ------------------------------------------------------------------ sum over the K slots
template <typename TS, typename TD>
__global__ __launch_bounds__(256) void slot_sum_kernel(const TS *__restrict__ src, int64_t ld_src,
                                                       TD *__restrict__ dst, int64_t ld_dst,
                                                       const int32_t *__restrict__ inv_perm,
                                                       int64_t n_tokens, int top_k, int n_cols,
                                                       const float *__restrict__ bias, int softplus,
                                                       const float *__restrict__ row_scale) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int pairs = (n_cols + 1) / 2;
  if (idx >= n_tokens * pairs) return;
  const int64_t n = idx / pairs;
  const int c = static_cast<int>(idx % pairs) * 2;
  const bool two = c + 1 < n_cols;            // an odd column count ends on a single column
  float a0 = 0.0f, a1 = 0.0f;
  for (int k = 0; k < top_k; ++k) {
    const int64_t row = inv_perm[n * top_k + k];
    a0 += to_f32(src[row * ld_src + c]);
    if (two) a1 += to_f32(src[row * ld_src + c + 1]);
  }
  if (row_scale) { a0 *= row_scale[n]; a1 *= row_scale[n]; }
  if (bias) { a0 += bias[c]; if (two) a1 += bias[c + 1]; }
  if (softplus) { a0 = softplus_f32(a0); a1 = softplus_f32(a1); }
  dst[n * ld_dst + c] = from_f32<TD>(a0);
  if (two) dst[n * ld_dst + c + 1] = from_f32<TD>(a1);
}

// xdbl rows (f32, R + 32 columns) -> dt_low (T) and bc (f32); sums the K slots when inv_perm is given
template <typename T>
__global__ __launch_bounds__(256) void split_xdbl_kernel(const float *__restrict__ xdbl, int n_slices,
                                                         int64_t slice_stride,
                                                         const int32_t *__restrict__ inv_perm,
                                                         int top_k, int64_t n_tokens, int dt_rank,
                                                         T *__restrict__ dt_low, float *__restrict__ bc) {
  const int n_cols = dt_rank + 32;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n_tokens * n_cols) return;
  const int64_t n = idx / n_cols;
  const int c = static_cast<int>(idx % n_cols);
  float acc = 0.0f;
  for (int sl = 0; sl < n_slices; ++sl) {      // split-K partial sums, fixed order
    const float *src = xdbl + sl * slice_stride;
    if (inv_perm) {
      for (int k = 0; k < top_k; ++k) acc += src[static_cast<int64_t>(inv_perm[n * top_k + k]) * n_cols + c];
    } else {
      acc += src[n * n_cols + c];
    }
  }
  if (c < dt_rank) dt_low[n * dt_rank + c] = from_f32<T>(acc);
  else bc[n * 32 + (c - dt_rank)] = acc;
}

// ------------------------------------------------------------------ conv + SiLU, Eq. (2)
// A thread owns one 16-byte group of channels and walks kConvRun consecutive time steps with the
// last three inputs in registers, so every input row is read once (plus a 3-row halo per run).
constexpr int kConvRun = kConvInPlaceMaxLen;

template <typename T>
__global__ __launch_bounds__(256) void conv_silu_kernel(
    const T *__restrict__ xz, int64_t ld_xz, const float *__restrict__ conv_w,
    const float *__restrict__ conv_b, const float *__restrict__ state_in,
    float *__restrict__ state_out, T *__restrict__ u, int64_t L, int d_inner) {
  constexpr int V = Chunk<T>::kElems;
  const int groups = d_inner / V;
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= groups) return;
  const int c0 = g * V;
  const int64_t b = blockIdx.z;
  const int64_t t0 = static_cast<int64_t>(blockIdx.y) * kConvRun;
  const int64_t t1 = (t0 + kConvRun < L) ? t0 + kConvRun : L;

  float w[V][4], bias[V], h[3][V];
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const float4 wv = *reinterpret_cast<const float4 *>(conv_w + static_cast<int64_t>(c0 + i) * 4);
    w[i][0] = wv.x; w[i][1] = wv.y; w[i][2] = wv.z; w[i][3] = wv.w;
    bias[i] = conv_b ? conv_b[c0 + i] : 0.0f;
  }
  const T *xrow = xz + b * L * ld_xz + c0;
  // history: inputs at t0-3, t0-2, t0-1.  The carried state of the V channels of this thread is
  // 3*V consecutive floats ([channel][3], oldest first): read with 16-byte loads.
  float st[3 * V];
  if (t0 < 3) {
    if (state_in) {
      const float4 *sp = reinterpret_cast<const float4 *>(state_in + (b * d_inner + c0) * 3);
#pragma unroll
      for (int i = 0; i < 3 * V / 4; ++i) {
        const float4 v = sp[i];
        st[4 * i] = v.x; st[4 * i + 1] = v.y; st[4 * i + 2] = v.z; st[4 * i + 3] = v.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 3 * V; ++i) st[i] = 0.0f;
    }
  }
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int64_t t = t0 - 3 + j;
    if (t >= 0) {
      Chunk<T> ch;
      ch.load(xrow + t * ld_xz);
#pragma unroll
      for (int i = 0; i < V; ++i) h[j][i] = ch.get(i);
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i) h[j][i] = st[i * 3 + j];   // t0 == 0 here: t = -3..-1 -> slot j
    }
  }
  T *urow = u + b * L * d_inner + c0;
  for (int64_t t = t0; t < t1; ++t) {
    Chunk<T> ch, out;
    ch.load(xrow + t * ld_xz);
    float r[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const float cur = ch.get(i);
      const float c = bias[i] + w[i][0] * h[0][i] + w[i][1] * h[1][i] + w[i][2] * h[2][i] + w[i][3] * cur;
      h[0][i] = h[1][i]; h[1][i] = h[2][i]; h[2][i] = cur;
      r[i] = silu_f32(c);
    }
#pragma unroll
    for (int i = 0; i < V / 2; ++i) out.set_pair(i, r[2 * i], r[2 * i + 1]);
    out.store(urow + t * d_inner);
  }
  if (state_out && t1 == L) {
    float4 *sp = reinterpret_cast<float4 *>(state_out + (b * d_inner + c0) * 3);
    float so[3 * V];
#pragma unroll
    for (int i = 0; i < V; ++i)
#pragma unroll
      for (int j = 0; j < 3; ++j) so[i * 3 + j] = h[j][i];
#pragma unroll
    for (int i = 0; i < 3 * V / 4; ++i) sp[i] = make_float4(so[4 * i], so[4 * i + 1], so[4 * i + 2], so[4 * i + 3]);
  }
}

// ------------------------------------------------------------------ selective scan, Eq. (5)
// Lane = (channel, state): 16 lanes share a channel, a 256-thread block owns 16 channels of one
// sequence chunk and walks it once; the 16 states of a channel live in registers, one per lane.
// Work is cut into tiles of kScanTile steps and groups of 16 steps:
//   * the block fetches a tile of dt, u, z (16 channels wide) and of B_t, C_t with 8/16-byte
//     loads one tile ahead of use (registers) and parks it in LDS once the tile before it is done
//     with (one tile in LDS: 24 KiB per block, so that six blocks fit a CU);
//     B/C are stored transposed so that lane n reads B_{t,n}, C_{t,n} of four steps at once;
//   * lane n of a channel picks up dt, u, z of step n of a group and hands dt and dt*u round
//     with DPP row broadcasts;
//   * the 16 products C_n*h_n of 16 steps are summed by a transposing butterfly (15 DPP adds per
//     step pair instead of a full reduction per step) that leaves y of step n in lane n, which
//     then applies the D skip and the SiLU(z) gate and writes g over the z it has just read;
//     g leaves LDS in 4-channel packets.
// The kernel is bound by plain ALU issue (about ten issue slots per step and lane, the
// exponential counting for several).  One sequence of 4096 channels is exactly one wavefront per
// SIMD, which issues at a lower rate than several would; launches with fewer workgroups than CUs
// are therefore cut into n_chunks time chunks: a state-only pass (kStateOnly: no C, z, reduction
// or output) runs every chunk but the last from a zero state and leaves its end state q and total
// decay P = exp(A * sum dt); the full pass then starts chunk c from the fold h <- P_k h + q_k over
// the chunks before it.  The recurrence is linear in h, so this is the same arithmetic regrouped.
// Beyond one workgroup per CU the state-only pass costs as much as the better issue rate gains.
constexpr int kScanTile = 64;
constexpr bool kScanDouble = true;
constexpr int kScanGroups = kScanTile / 16;
constexpr int kScanCh = 16;
constexpr int kBcPitch = kScanTile + 4;     // floats; keeps 16-byte alignment of the row reads

template <int CTRL> __device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadRev = 0x1B;       // quad_perm [3,2,1,0]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7 - i inside each 8
constexpr int kDppRowMirror = 0x140;    // lane i <-> 15 - i inside each 16
constexpr int kDppRowBcast0 = 0x150;    // row_newbcast:0 (+j for lane j of the row)

// floats per step row of the dt/u/z/g tiles (16 channels + padding that keeps rows 16-byte aligned
// and spreads the 16 steps a row of lanes reads over the banks).  The tiles hold floats: converting
// once when a tile is parked is cheaper than converting in the issue-bound inner loop.
constexpr int kChPitch = kScanCh + 4;

struct __attribute__((aligned(16))) ScanSmem {     // one tile of inputs
  float dt[kScanTile][kChPitch];
  float u[kScanTile][kChPitch];
  float zg[kScanTile][kChPitch];        // z on the way in; with a single tile in LDS the lane that read z_t puts g_t in its place
  float bc[32][kBcPitch];               // [B_0..B_15, C_0..C_15][step]
};

template <int J> struct StepSeq {
  __device__ static __forceinline__ void run(float dt_r, float dtu_r, float a2, const float *bv,
                                             float &h, float *hs) {
    StepSeq<J - 1>::run(dt_r, dtu_r, a2, bv, h, hs);
    const float dtj = dpp<kDppRowBcast0 + J>(dt_r);
    const float dtuj = dpp<kDppRowBcast0 + J>(dtu_r);
    const float da = fast_exp2(dtj * a2);
    h = fmaf(da, h, dtuj * bv[J]);
    hs[J] = h;
  }
};
template <> struct StepSeq<-1> {
  __device__ static __forceinline__ void run(float, float, float, const float *, float &, float *) {}
};

// p[j] = hs[j] * cv[j]; sum p[j] over the 16 lanes of a row for every j; lane i returns the
// total of p[i].  Contraction is off so that every "x + dpp(x)" stays one DPP add.
__device__ __forceinline__ float transpose_reduce16(const float *hs, const float *cv, int n) {
#pragma clang fp contract(off)
  float a[8], b[4], c[2];
  const bool hi8 = (n & 8) != 0, hi4 = (n & 4) != 0, hi2 = (n & 2) != 0, hi1 = (n & 1) != 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float pl = hs[j] * cv[j], ph = hs[j + 8] * cv[j + 8];
    const float lo = dpp<kDppRowMirror>(pl) + pl;
    const float hi = dpp<kDppRowMirror>(ph) + ph;
    a[j] = hi8 ? hi : lo;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = dpp<kDppHalfMirror>(a[j]) + a[j];
    const float hi = dpp<kDppHalfMirror>(a[j + 4]) + a[j + 4];
    b[j] = hi4 ? hi : lo;
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const float lo = dpp<kDppQuadRev>(b[j]) + b[j];
    const float hi = dpp<kDppQuadRev>(b[j + 2]) + b[j + 2];
    c[j] = hi2 ? hi : lo;
  }
  const float lo = dpp<kDppQuadXor1>(c[0]) + c[0];
  const float hi = dpp<kDppQuadXor1>(c[1]) + c[1];
  return hi1 ? hi : lo;
}

// sum of v over the 16 lanes of a row, in every lane
__device__ __forceinline__ float row_sum16(float v) {
#pragma clang fp contract(off)
  v = dpp<kDppRowMirror>(v) + v;
  v = dpp<kDppHalfMirror>(v) + v;
  v = dpp<kDppQuadRev>(v) + v;
  v = dpp<kDppQuadXor1>(v) + v;
  return v;
}

// N consecutive elements of T held in registers
template <typename T, int N> struct Pack;
__device__ __forceinline__ float bf16_word_get(unsigned int w, int odd) {
  return __uint_as_float(odd ? (w & 0xFFFF0000u) : (w << 16));
}
template <> struct Pack<bf16_t, 8> {
  uint4 raw;
  __device__ __forceinline__ void to_floats(float *f) const {
    f[0] = bf16_word_get(raw.x, 0); f[1] = bf16_word_get(raw.x, 1);
    f[2] = bf16_word_get(raw.y, 0); f[3] = bf16_word_get(raw.y, 1);
    f[4] = bf16_word_get(raw.z, 0); f[5] = bf16_word_get(raw.z, 1);
    f[6] = bf16_word_get(raw.w, 0); f[7] = bf16_word_get(raw.w, 1);
  }
  __device__ __forceinline__ void load(const bf16_t *p) { raw = ld_u4(p); }
  __device__ __forceinline__ void zero() { raw = make_uint4(0, 0, 0, 0); }
  __device__ __forceinline__ void park(float *p) const {      // as floats, 16-byte aligned
    *reinterpret_cast<float4 *>(p) = make_float4(bf16_word_get(raw.x, 0), bf16_word_get(raw.x, 1),
                                                 bf16_word_get(raw.y, 0), bf16_word_get(raw.y, 1));
    *reinterpret_cast<float4 *>(p + 4) = make_float4(bf16_word_get(raw.z, 0), bf16_word_get(raw.z, 1),
                                                     bf16_word_get(raw.w, 0), bf16_word_get(raw.w, 1));
  }
};
template <> struct Pack<bf16_t, 4> {
  uint2 raw;
  __device__ __forceinline__ void load(const bf16_t *p) { raw = ld_u2(p); }
  __device__ __forceinline__ void zero() { raw = make_uint2(0, 0); }
  __device__ __forceinline__ void park(float *p) const {
    *reinterpret_cast<float4 *>(p) = make_float4(bf16_word_get(raw.x, 0), bf16_word_get(raw.x, 1),
                                                 bf16_word_get(raw.y, 0), bf16_word_get(raw.y, 1));
  }
  __device__ __forceinline__ void from_floats(const float4 &v) {
    raw.x = pack_bf16x2(v.x, v.y);
    raw.y = pack_bf16x2(v.z, v.w);
  }
  __device__ __forceinline__ void store(bf16_t *p) const { *reinterpret_cast<uint2 *>(p) = raw; }
};
template <> struct Pack<float, 8> {
  float4 lo, hi;
  __device__ __forceinline__ void to_floats(float *f) const {
    f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w;
    f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
  }
  __device__ __forceinline__ void load(const float *p) {
    lo = ld_f4(p);
    hi = ld_f4(p + 4);
  }
  __device__ __forceinline__ void zero() { lo = make_float4(0.f, 0.f, 0.f, 0.f); hi = lo; }
  __device__ __forceinline__ void park(float *p) const {
    *reinterpret_cast<float4 *>(p) = lo;
    *reinterpret_cast<float4 *>(p + 4) = hi;
  }
};
template <> struct Pack<float, 4> {
  float4 raw;
  __device__ __forceinline__ void load(const float *p) { raw = ld_f4(p); }
  __device__ __forceinline__ void zero() { raw = make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ __forceinline__ void park(float *p) const { *reinterpret_cast<float4 *>(p) = raw; }
  __device__ __forceinline__ void from_floats(const float4 &v) { raw = v; }
  __device__ __forceinline__ void store(float *p) const { *reinterpret_cast<float4 *>(p) = raw; }
};

// One thread's share of a tile: 8 channels of one step of dt (threads 0..127) or u (128..255),
// 4 channels of one step of z, 8 of the 32 B/C values of one step (the state-only pass takes
// neither z nor C).
template <typename T> struct ScanStage {
  Pack<T, 8> du;
  Pack<T, 4> z;
  float4 bc0, bc1;
};

template <typename T, bool kStateOnly, bool kTail>
__device__ __forceinline__ void scan_fetch(ScanStage<T> &r, const T *dt_b, const T *u_b, const T *z_b,
                                           const float *bc_b, int64_t t0, int64_t t_end, int d_inner,
                                           int64_t ld_z, int tid) {
  const int64_t t_du = t0 + ((tid & 127) >> 1);
  if (!kTail || t_du < t_end) r.du.load((tid < 128 ? dt_b : u_b) + t_du * d_inner + (tid & 1) * 8);
  else r.du.zero();
  const int64_t t_z = t0 + (tid >> 2);
  const bool want_bc = !kStateOnly || (tid & 3) < 2;
  if (!kTail || t_z < t_end) {
    if (!kStateOnly) r.z.load(z_b + t_z * ld_z + (tid & 3) * 4);
    if (want_bc) {
      const float *src = bc_b + t_z * 32 + (tid & 3) * 8;
      r.bc0 = ld_f4(src);
      r.bc1 = ld_f4(src + 4);
    }
  } else {
    if (!kStateOnly) r.z.zero();
    r.bc0 = make_float4(0.f, 0.f, 0.f, 0.f);
    r.bc1 = r.bc0;
  }
}

template <typename T, bool kStateOnly>
__device__ __forceinline__ void scan_park(ScanSmem &sm, const ScanStage<T> &r, int tid) {
  r.du.park((tid < 128 ? &sm.dt[0][0] : &sm.u[0][0]) + ((tid & 127) >> 1) * kChPitch + (tid & 1) * 8);
  const int row = tid >> 2, part = tid & 3;
  if (!kStateOnly) r.z.park(&sm.zg[row][part * 4]);
  if (!kStateOnly || part < 2) {
    const int col = part * 8;
    sm.bc[col + 0][row] = r.bc0.x; sm.bc[col + 1][row] = r.bc0.y;
    sm.bc[col + 2][row] = r.bc0.z; sm.bc[col + 3][row] = r.bc0.w;
    sm.bc[col + 4][row] = r.bc1.x; sm.bc[col + 5][row] = r.bc1.y;
    sm.bc[col + 6][row] = r.bc1.z; sm.bc[col + 7][row] = r.bc1.w;
  }
}

// grid: (d_inner / 16, B, chunks handled by this pass).  chunk_q / chunk_p: f32
// [B][n_chunks][d_inner][16], end state from zero and total decay of every chunk but the last.
// NB = 1: one tile in LDS (24 KiB, six blocks per CU); NB = 2: two tiles and two g tiles (58 KiB):
// the next tile is parked while this one is computed and a tile costs one barrier instead of two,
// which pays when the launch has no more than one block per CU anyway.
template <typename T, bool kStateOnly, int NB>
__global__ __launch_bounds__(256) void scan_kernel(
    const T *__restrict__ u, const T *__restrict__ dt, const float *__restrict__ bc,
    const T *__restrict__ z, int64_t ld_z, const float *__restrict__ A_log,
    const float *__restrict__ D, const float *__restrict__ h_in, float *__restrict__ h_out,
    T *__restrict__ g, int64_t L, int d_inner, int64_t chunk_len, int n_chunks,
    float *__restrict__ chunk_q, float *__restrict__ chunk_p) {
  __shared__ ScanSmem tiles[NB];
  __shared__ float g_tiles[NB == 2 ? 2 : 1][NB == 2 ? kScanTile : 1][kChPitch];
  const int tid = threadIdx.x;
  const int n = tid & 15;            // state index = lane inside the DPP row
  const int cl = tid >> 4;           // channel inside the block
  // consecutive workgroups land on different XCDs (round-robin over 8): give each XCD a
  // contiguous run of channel groups so that neighbours in memory share an L2.
  const int n_groups = d_inner / kScanCh;
  int grp = blockIdx.x;
  if (n_groups % 8 == 0) grp = (blockIdx.x % 8) * (n_groups / 8) + blockIdx.x / 8;
  const int c0 = grp * kScanCh;
  const int ch = c0 + cl;
  const int64_t b = blockIdx.y;
  const int chunk = blockIdx.z;
  const int64_t t_begin = chunk * chunk_len;
  const int64_t t_end = (t_begin + chunk_len < L) ? t_begin + chunk_len : L;

  const float a2 = -__expf(A_log[static_cast<int64_t>(ch) * 16 + n]) * 1.44269504088896341f;
  const float d_skip = kStateOnly ? 0.0f : D[ch];
  // chunk_q / chunk_p hold n_chunks slots per sequence: slots 0..n_chunks-2 the chunk summaries,
  // the last slot of chunk_q a copy of the incoming state taken by the state-only pass, so that
  // the full pass of a chunked launch never reads h_in (h_out may alias it, and the last chunk's
  // block writes h_out while blocks of earlier chunks may still be starting)
  float h = 0.0f;
  if (kStateOnly) {
    if (chunk == 0)
      chunk_q[((b * n_chunks + (n_chunks - 1)) * d_inner + ch) * 16 + n] = h_in ? h_in[(b * d_inner + ch) * 16 + n] : 0.0f;
  } else {
    if (n_chunks > 1) h = chunk_q[((b * n_chunks + (n_chunks - 1)) * d_inner + ch) * 16 + n];
    else h = h_in ? h_in[(b * d_inner + ch) * 16 + n] : 0.0f;
    for (int k = 0; k < chunk; ++k) {      // fold the chunks before this one
      const int64_t at = ((b * n_chunks + k) * d_inner + ch) * 16 + n;
      h = fmaf(chunk_p[at], h, chunk_q[at]);
    }
  }
  float dt_sum = 0.0f;

  const T *u_b = u + b * L * d_inner + c0;
  const T *dt_b = dt + b * L * d_inner + c0;
  const T *z_b = kStateOnly ? nullptr : z + b * L * ld_z + c0;
  const float *bc_b = bc + b * L * 32;
  T *g_b = kStateOnly ? nullptr : g + b * L * d_inner + c0;

  ScanStage<T> st;
  const int64_t n_tiles = (t_end - t_begin + kScanTile - 1) / kScanTile;
  if (t_begin + kScanTile <= t_end)
    scan_fetch<T, kStateOnly, false>(st, dt_b, u_b, z_b, bc_b, t_begin, t_end, d_inner, ld_z, tid);
  else
    scan_fetch<T, kStateOnly, true>(st, dt_b, u_b, z_b, bc_b, t_begin, t_end, d_inner, ld_z, tid);
  scan_park<T, kStateOnly>(tiles[0], st, tid);
  __syncthreads();

  for (int64_t ti = 0; ti < n_tiles; ++ti) {
    ScanSmem &sm = tiles[NB == 2 ? (ti & 1) : 0];
    float(*g_tile)[kChPitch] = NB == 2 ? g_tiles[ti & 1] : sm.zg;
    const int64_t t0 = t_begin + ti * kScanTile;
    const bool has_next = ti + 1 < n_tiles;
    if (has_next) {     // next tile's inputs travel while this tile is computed
      if (t0 + 2 * kScanTile <= t_end)
        scan_fetch<T, kStateOnly, false>(st, dt_b, u_b, z_b, bc_b, t0 + kScanTile, t_end, d_inner, ld_z, tid);
      else
        scan_fetch<T, kStateOnly, true>(st, dt_b, u_b, z_b, bc_b, t0 + kScanTile, t_end, d_inner, ld_z, tid);
    }
    // the state-only pass is one long dependency chain with little else to do: unrolled over the
    // groups, the scheduler hoists every exponential of the tile and runs out of registers
#pragma unroll(kStateOnly ? 1 : kScanGroups)
    for (int gi = 0; gi < kScanGroups; ++gi) {
      const int s0 = gi * 16;
      const float dt_r = sm.dt[s0 + n][cl];
      const float u_r = sm.u[s0 + n][cl];
      const float dtu_r = dt_r * u_r;
      float bv[16], hs[16];
#pragma unroll
      for (int j = 0; j < 16; j += 4) {
        const float4 b4 = *reinterpret_cast<const float4 *>(&sm.bc[n][s0 + j]);
        bv[j] = b4.x; bv[j + 1] = b4.y; bv[j + 2] = b4.z; bv[j + 3] = b4.w;
      }
      StepSeq<15>::run(dt_r, dtu_r, a2, bv, h, hs);
      if (kStateOnly) {
        dt_sum += dt_r;
      } else {
        float cv[16];
#pragma unroll
        for (int j = 0; j < 16; j += 4) {
          const float4 c4 = *reinterpret_cast<const float4 *>(&sm.bc[16 + n][s0 + j]);
          cv[j] = c4.x; cv[j + 1] = c4.y; cv[j + 2] = c4.z; cv[j + 3] = c4.w;
        }
        const float z_r = sm.zg[s0 + n][cl];
        const float y = transpose_reduce16(hs, cv, n) + d_skip * u_r;
        g_tile[s0 + n][cl] = y * silu_f32(z_r);
      }
    }
    if (NB == 2 && has_next) scan_park<T, kStateOnly>(tiles[(ti + 1) & 1], st, tid);
    __syncthreads();     // everyone is done reading the tile; g is complete (and the next tile parked)
    if (!kStateOnly) {   // g of this tile: thread -> (step row, 4 channels), the packet it parks z into
      const int r = tid >> 2, q = (tid & 3) * 4;
      const int64_t t = t0 + r;
      if (t < t_end) {
        Pack<T, 4> pk;
        pk.from_floats(*reinterpret_cast<const float4 *>(&g_tile[r][q]));
        pk.store(g_b + t * d_inner + q);
      }
    }
    if (NB == 1 && has_next) {
      scan_park<T, kStateOnly>(sm, st, tid);
      __syncthreads();
    }
  }
  if (kStateOnly) {
    const int64_t at = ((b * n_chunks + chunk) * d_inner + ch) * 16 + n;
    chunk_q[at] = h;
    chunk_p[at] = fast_exp2(a2 * row_sum16(dt_sum));
  } else if (h_out && chunk == n_chunks - 1) {
    h_out[(b * d_inner + ch) * 16 + n] = h;
  }
}

// ------------------------------------------------------------------ selective scan, software-pipelined
// The same lane = (channel, state) layout and LDS tiles as scan_kernel<T, false, 2>, for launches
// with at most one block per CU (one long sequence: one wavefront per SIMD, nobody else to hide a
// stall).  Measured on MI355X, a lone wavefront issues an independent fp32 instruction every 5
// clocks, a DPP one every 5, v_exp_f32 every 9, and waits 8.8 clocks for a dependent FMA: the
// only latency-bound piece of a 16-step group is its chain of 16 dependent FMAs, so the groups of
// a tile run as a three-stage pipeline whose stages are interleaved instruction by instruction -
//   A(g+1): decay exp2(dt*A) and input dt*u*B of the next group (48 independent instructions),
//   B(g):   the 16 dependent FMAs of this group,
//   C(g-1): C.h products, transposing reduction, D skip and SiLU(z) gate of the previous group
// - one FMA of B, then three instructions of A and up to five of C, fenced so that the compiler
// keeps the order.  All of a lane's tile inputs (dt, u, z of its four steps, B and C of all 64)
// are read from LDS into registers at the top of the tile, in the order of use.
struct ScanPipeRegs {
  float dt_r[kScanGroups], u_r[kScanGroups], z_r[kScanGroups], dtu_r[kScanGroups];
  float bv[kScanGroups][16], cv[kScanGroups][16];
  float da[2][16], xx[2][16], hs[2][16];
  float ra[8], rb[4], rc[2], y;
  float h, a2, d_skip;
  bool hi8, hi4, hi2, hi1;
};

// slot J of phase P (P = -1 .. kScanGroups): step J of B(P), step J of A(P + 1), unit J of C(P - 1)
// (PARTS: bit 0 = A, 1 = B, 2 = C; anything but 7 is for timing probes)
template <int P, int J, int PARTS = 7>
__device__ __forceinline__ void scan_pipe_slot(ScanPipeRegs &r, float (*g_tile)[kChPitch], int n, int cl) {
#pragma clang fp contract(off)
  if constexpr ((PARTS & 2) != 0 && P >= 0 && P < kScanGroups) {
    r.h = __builtin_fmaf(r.da[P & 1][J], r.h, r.xx[P & 1][J]);
    r.hs[P & 1][J] = r.h;
  }
  if constexpr ((PARTS & 1) != 0 && P + 1 >= 0 && P + 1 < kScanGroups) {
    constexpr int G = P + 1;
    r.da[G & 1][J] = fast_exp2(dpp<kDppRowBcast0 + J>(r.dt_r[G]) * r.a2);
    r.xx[G & 1][J] = dpp<kDppRowBcast0 + J>(r.dtu_r[G]) * r.bv[G][J];
  }
  if constexpr ((PARTS & 4) != 0 && P - 1 >= 0 && P - 1 < kScanGroups) {
    constexpr int G = P - 1;
    const float *hs = r.hs[G & 1];
    const float *cv = r.cv[G];
    if constexpr (J < 8) {
      const float pl = hs[J] * cv[J], ph = hs[J + 8] * cv[J + 8];
      const float lo = dpp<kDppRowMirror>(pl) + pl;
      const float hi = dpp<kDppRowMirror>(ph) + ph;
      r.ra[J] = r.hi8 ? hi : lo;
    } else if constexpr (J < 12) {
      constexpr int I = J - 8;
      const float lo = dpp<kDppHalfMirror>(r.ra[I]) + r.ra[I];
      const float hi = dpp<kDppHalfMirror>(r.ra[I + 4]) + r.ra[I + 4];
      r.rb[I] = r.hi4 ? hi : lo;
    } else if constexpr (J < 14) {
      constexpr int I = J - 12;
      const float lo = dpp<kDppQuadRev>(r.rb[I]) + r.rb[I];
      const float hi = dpp<kDppQuadRev>(r.rb[I + 2]) + r.rb[I + 2];
      r.rc[I] = r.hi2 ? hi : lo;
    } else if constexpr (J == 14) {
      const float lo = dpp<kDppQuadXor1>(r.rc[0]) + r.rc[0];
      const float hi = dpp<kDppQuadXor1>(r.rc[1]) + r.rc[1];
      r.y = r.hi1 ? hi : lo;
    } else {
      const float y = r.y + r.d_skip * r.u_r[G];
      g_tile[G * 16 + n][cl] = y * silu_f32(r.z_r[G]);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
}
template <int P, int J, int PARTS = 7> struct ScanPipeSlots {
  __device__ static __forceinline__ void run(ScanPipeRegs &r, float (*g_tile)[kChPitch], int n, int cl) {
    ScanPipeSlots<P, J - 1, PARTS>::run(r, g_tile, n, cl);
    scan_pipe_slot<P, J, PARTS>(r, g_tile, n, cl);
  }
};
template <int P, int PARTS> struct ScanPipeSlots<P, -1, PARTS> {
  __device__ static __forceinline__ void run(ScanPipeRegs &, float (*)[kChPitch], int, int) {}
};
template <int P, int PARTS = 7> struct ScanPipePhases {
  __device__ static __forceinline__ void run(ScanPipeRegs &r, float (*g_tile)[kChPitch], int n, int cl) {
    ScanPipePhases<P - 1, PARTS>::run(r, g_tile, n, cl);
    ScanPipeSlots<P, 15, PARTS>::run(r, g_tile, n, cl);
  }
};
template <int PARTS> struct ScanPipePhases<-2, PARTS> {
  __device__ static __forceinline__ void run(ScanPipeRegs &, float (*)[kChPitch], int, int) {}
};

__device__ __forceinline__ void scan_pipe_read16(float *dst, const float *row) {
#pragma unroll
  for (int j = 0; j < 16; j += 4) {
    const float4 v = *reinterpret_cast<const float4 *>(row + j);
    dst[j] = v.x; dst[j + 1] = v.y; dst[j + 2] = v.z; dst[j + 3] = v.w;
  }
}

// grid: (d_inner / 16, B, n_chunks); arguments as scan_kernel<T, false, 2>.
// HELPERS: the block has 512 threads.  Wavefronts 0..3 ("compute") only read their tile inputs
// from LDS, run the phases and leave g in LDS; wavefronts 4..7 ("helpers", one beside each compute
// wavefront on its SIMD) do everything that touches global memory - fetch tile t+2, convert and
// park tile t+1, turn the finished g tile into coalesced stores - so that none of it sits on the
// lone compute wavefront's critical path.  One block barrier per tile, at which the compute side
// says "tile t read, g of tile t complete" and the helper side "tile t+1 parked".
// Without HELPERS (256 threads) every wavefront does both, for launches with two blocks per CU.
template <typename T, bool HELPERS>
__global__ __launch_bounds__(HELPERS ? 512 : 256) void scan_pipe_kernel(
    const T *__restrict__ u, const T *__restrict__ dt, const float *__restrict__ bc,
    const T *__restrict__ z, int64_t ld_z, const float *__restrict__ A_log,
    const float *__restrict__ D, const float *__restrict__ h_in, float *__restrict__ h_out,
    T *__restrict__ g, int64_t L, int d_inner, int64_t chunk_len, int n_chunks,
    float *__restrict__ chunk_q, float *__restrict__ chunk_p) {
  __shared__ ScanSmem tiles[2];
  __shared__ float g_tiles[2][kScanTile][kChPitch];
  const bool computes = !HELPERS || threadIdx.x < 256;
  const bool helps = !HELPERS || threadIdx.x >= 256;
  const int tid = threadIdx.x & 255;
  const int n = tid & 15;            // state index = lane inside the DPP row
  const int cl = tid >> 4;           // channel inside the block
  const int n_groups = d_inner / kScanCh;
  int grp = blockIdx.x;
  if (n_groups % 8 == 0) grp = (blockIdx.x % 8) * (n_groups / 8) + blockIdx.x / 8;
  const int c0 = grp * kScanCh;
  const int ch = c0 + cl;
  const int64_t b = blockIdx.y;
  const int chunk = blockIdx.z;
  const int64_t t_begin = chunk * chunk_len;
  const int64_t t_end = (t_begin + chunk_len < L) ? t_begin + chunk_len : L;
  const int64_t n_tiles = (t_end - t_begin + kScanTile - 1) / kScanTile;

  const T *u_b = u + b * L * d_inner + c0;
  const T *dt_b = dt + b * L * d_inner + c0;
  const T *z_b = z + b * L * ld_z + c0;
  const float *bc_b = bc + b * L * 32;
  T *g_b = g + b * L * d_inner + c0;

  // global -> registers of tile number `tile` (rows past t_end are zero-filled: dt = 0 leaves h alone)
  ScanStage<T> st;
  auto fetch = [&](int64_t tile) __attribute__((always_inline)) {
    const int64_t t0 = t_begin + tile * kScanTile;
    if (t0 + kScanTile <= t_end)
      scan_fetch<T, false, false>(st, dt_b, u_b, z_b, bc_b, t0, t_end, d_inner, ld_z, tid);
    else
      scan_fetch<T, false, true>(st, dt_b, u_b, z_b, bc_b, t0, t_end, d_inner, ld_z, tid);
  };
  // g of tile number `tile`: thread -> (step row, 4 channels)
  auto store_g = [&](int64_t tile) __attribute__((always_inline)) {
    const int row = tid >> 2, q = (tid & 3) * 4;
    const int64_t t = t_begin + tile * kScanTile + row;
    if (t < t_end) {
      Pack<T, 4> pk;
      pk.from_floats(*reinterpret_cast<const float4 *>(&g_tiles[tile & 1][row][q]));
      pk.store(g_b + t * d_inner + q);
    }
  };

  ScanPipeRegs r;
  if (computes) {
    r.a2 = -__expf(A_log[static_cast<int64_t>(ch) * 16 + n]) * 1.44269504088896341f;
    r.d_skip = D[ch];
    r.hi8 = (n & 8) != 0; r.hi4 = (n & 4) != 0; r.hi2 = (n & 2) != 0; r.hi1 = (n & 1) != 0;
    if (n_chunks > 1) r.h = chunk_q[((b * n_chunks + (n_chunks - 1)) * d_inner + ch) * 16 + n];
    else r.h = h_in ? h_in[(b * d_inner + ch) * 16 + n] : 0.0f;
    for (int k = 0; k < chunk; ++k) {      // fold the chunks before this one
      const int64_t at = ((b * n_chunks + k) * d_inner + ch) * 16 + n;
      r.h = fmaf(chunk_p[at], r.h, chunk_q[at]);
    }
  }
  if (helps) {
    fetch(0);
    scan_park<T, false>(tiles[0], st, tid);
    if (n_tiles > 1) fetch(1);
  }
  __syncthreads();

  for (int64_t ti = 0; ti < n_tiles; ++ti) {
    const bool has_next = ti + 1 < n_tiles;
    if (computes) {
      ScanSmem &sm = tiles[ti & 1];
      // this lane's share of the tile, in the order the phases consume it
#pragma unroll
      for (int gi = 0; gi < kScanGroups; ++gi) {
        r.dt_r[gi] = sm.dt[gi * 16 + n][cl];
        r.u_r[gi] = sm.u[gi * 16 + n][cl];
        r.dtu_r[gi] = r.dt_r[gi] * r.u_r[gi];
      }
      scan_pipe_read16(r.bv[0], &sm.bc[n][0]);
      scan_pipe_read16(r.bv[1], &sm.bc[n][16]);
      scan_pipe_read16(r.cv[0], &sm.bc[16 + n][0]);
#pragma unroll
      for (int gi = 2; gi < kScanGroups; ++gi) {
        scan_pipe_read16(r.bv[gi], &sm.bc[n][gi * 16]);
        scan_pipe_read16(r.cv[gi - 1], &sm.bc[16 + n][(gi - 1) * 16]);
      }
      scan_pipe_read16(r.cv[kScanGroups - 1], &sm.bc[16 + n][(kScanGroups - 1) * 16]);
#pragma unroll
      for (int gi = 0; gi < kScanGroups; ++gi) r.z_r[gi] = sm.zg[gi * 16 + n][cl];
      __builtin_amdgcn_sched_barrier(0);
      ScanPipePhases<kScanGroups>::run(r, g_tiles[ti & 1], n, cl);
    }
    if (helps) {
      if (HELPERS && ti > 0) store_g(ti - 1);         // complete since the barrier that ended tile ti - 1
      if (has_next) {
        scan_park<T, false>(tiles[(ti + 1) & 1], st, tid);    // (its last readers passed that same barrier)
        if (ti + 2 < n_tiles) fetch(ti + 2);
      }
    }
    __syncthreads();     // tile ti is read and its g complete; tile ti + 1 is parked
    if (!HELPERS) store_g(ti);
  }
  if (HELPERS && helps && n_tiles > 0) store_g(n_tiles - 1);
  if (computes && h_out && chunk == n_chunks - 1) h_out[(b * d_inner + ch) * 16 + n] = r.h;
}

// ------------------------------------------------------------------ single-step scan (L == 1)
// One recurrence update per (sequence, channel, state): bound by reading and writing the fp32
// state.  A lane owns four consecutive states of one channel (one 16-byte load and store), four
// lanes share a channel and reduce C.h with two DPP adds inside their quad.
template <typename T>
__global__ __launch_bounds__(256) void scan_step_kernel(
    const T *__restrict__ u, const T *__restrict__ dt, const float *__restrict__ bc,
    const T *__restrict__ z, int64_t ld_z, const float *__restrict__ A_log,
    const float *__restrict__ D, const float *__restrict__ h_in, float *__restrict__ h_out,
    T *__restrict__ g, int64_t n_seq, int d_inner) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int q = threadIdx.x & 3;                   // which four states
  const int64_t bc_idx = idx >> 2;                 // (sequence, channel)
  if (bc_idx >= n_seq * d_inner) return;           // whole quads leave together
  const int64_t b = bc_idx / d_inner;
  const int ch = static_cast<int>(bc_idx % d_inner);
  const float4 al = *reinterpret_cast<const float4 *>(A_log + static_cast<int64_t>(ch) * 16 + q * 4);
  const float4 bv = *reinterpret_cast<const float4 *>(bc + b * 32 + q * 4);
  const float4 cv = *reinterpret_cast<const float4 *>(bc + b * 32 + 16 + q * 4);
  const float dt_r = to_f32(dt[bc_idx]);
  const float u_r = to_f32(u[bc_idx]);
  const float dtu = dt_r * u_r;
  float4 h = h_in ? *reinterpret_cast<const float4 *>(h_in + idx * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
  const float k = -1.44269504088896341f * dt_r;
  h.x = fmaf(fast_exp2(k * __expf(al.x)), h.x, dtu * bv.x);
  h.y = fmaf(fast_exp2(k * __expf(al.y)), h.y, dtu * bv.y);
  h.z = fmaf(fast_exp2(k * __expf(al.z)), h.z, dtu * bv.z);
  h.w = fmaf(fast_exp2(k * __expf(al.w)), h.w, dtu * bv.w);
  if (h_out) *reinterpret_cast<float4 *>(h_out + idx * 4) = h;
  float part = h.x * cv.x + h.y * cv.y + h.z * cv.z + h.w * cv.w;
  {
#pragma clang fp contract(off)
    part = dpp<kDppQuadXor1>(part) + part;
    part = dpp<0x4E>(part) + part;                 // quad_perm [2,3,0,1]
  }
  if (q == 0) g[bc_idx] = from_f32<T>((part + D[ch] * u_r) * silu_f32(to_f32(z[b * ld_z + ch])));
}

// ------------------------------------------------------------------ sum over the K slots, wide form
// slot_sum_kernel with eight columns per thread and 16-byte accesses (n_cols, ld_src, ld_dst multiples of 8,
// 16-byte aligned bases): the scalar form above moves two or four bytes per lane and reaches half
// the bandwidth
template <typename TS, typename TD>
__global__ __launch_bounds__(256) void slot_sum8_kernel(const TS *__restrict__ src, int64_t ld_src,
                                                        TD *__restrict__ dst, int64_t ld_dst,
                                                        const int32_t *__restrict__ inv_perm,
                                                        int64_t n_tokens, int top_k, int n_cols,
                                                        const float *__restrict__ bias, int softplus,
                                                        const float *__restrict__ row_scale) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int groups = n_cols / 8;
  if (idx >= n_tokens * groups) return;
  const int64_t n = idx / groups;
  const int c = static_cast<int>(idx % groups) * 8;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.0f;
  for (int k = 0; k < top_k; ++k) {
    const int64_t row = inv_perm[n * top_k + k];
    Pack<TS, 8> v;
    v.load(src + row * ld_src + c);
    float f[8];
    v.to_floats(f);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += f[i];
  }
  if (row_scale) {
    const float rs = row_scale[n];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] *= rs;
  }
  if (bias) {
    const float4 b0 = ld_f4(bias + c), b1 = ld_f4(bias + c + 4);
    acc[0] += b0.x; acc[1] += b0.y; acc[2] += b0.z; acc[3] += b0.w;
    acc[4] += b1.x; acc[5] += b1.y; acc[6] += b1.z; acc[7] += b1.w;
  }
  if (softplus) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = softplus_f32(acc[i]);
  }
  Pack<TD, 4> lo, hi;
  lo.from_floats(make_float4(acc[0], acc[1], acc[2], acc[3]));
  hi.from_floats(make_float4(acc[4], acc[5], acc[6], acc[7]));
  lo.store(dst + n * ld_dst + c);
  hi.store(dst + n * ld_dst + c + 4);
}

// ------------------------------------------------------------------ combine, Eq. (12)
template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const T *__restrict__ op,
                                                      const int32_t *__restrict__ inv_perm,
                                                      const float *__restrict__ gate,
                                                      T *__restrict__ out, int64_t n_tokens,
                                                      int top_k, int d_model,
                                                      const T *__restrict__ residual) {
  constexpr int V = Chunk<T>::kElems;
  const int groups = d_model / V;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n_tokens * groups) return;
  const int64_t n = idx / groups;
  const int c0 = static_cast<int>(idx % groups) * V;
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.0f;
  if (residual) {                 // skip connection: start from the block's input row
    Chunk<T> r;
    r.load(residual + n * d_model + c0);
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = r.get(i);
  }
  for (int k = 0; k < top_k; ++k) {
    const int64_t row = inv_perm[n * top_k + k];
    const float gk = gate[n * top_k + k];
    Chunk<T> ch;
    ch.load(op + row * d_model + c0);
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = fmaf(gk, ch.get(i), acc[i]);
  }
  Chunk<T> o;
#pragma unroll
  for (int i = 0; i < V / 2; ++i) o.set_pair(i, acc[2 * i], acc[2 * i + 1]);
  o.store(out + n * d_model + c0);
}

// ------------------------------------------------------------------ FFN-MoE helpers, Eq. (14), (15)
// a[p, 8b + t] = SiLU(h[p, 16b + t]) * h[p, 16b + 8 + t]: the SwiGLU of one expert's projection row,
// whose columns come in blocks of 8 gate + 8 up features (the packed weight's row order)
template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const T *__restrict__ h, T *__restrict__ a,
                                                     int64_t n_rows, int d_ff) {
  constexpr int V = Chunk<T>::kElems;
  const int groups = d_ff / V;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n_rows * groups) return;
  const int64_t row = idx / groups;
  const int c0 = static_cast<int>(idx % groups) * V;
  Chunk<T> g, u, o;
  const int goff = 16 * (c0 / 8) + (c0 % 8);
  g.load(h + row * 2 * d_ff + goff);
  u.load(h + row * 2 * d_ff + goff + 8);
#pragma unroll
  for (int i = 0; i < V / 2; ++i)
    o.set_pair(i, silu_f32(g.get(2 * i)) * u.get(2 * i), silu_f32(g.get(2 * i + 1)) * u.get(2 * i + 1));
  o.store(a + row * d_ff + c0);
}

// adjoint of the SwiGLU above, in the same packed column order:
// d_h[p, 16b + t] = d_a[p, 8b + t] * up * s (1 + gate (1 - s)),  d_h[p, 16b + 8 + t] = d_a[p, 8b + t] * gate * s,  s = sigmoid(gate)
template <typename T>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T *__restrict__ h, const T *__restrict__ d_a,
                                                         T *__restrict__ d_h, int64_t n_rows, int d_ff) {
  constexpr int V = Chunk<T>::kElems;
  const int groups = d_ff / V;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n_rows * groups) return;
  const int64_t row = idx / groups;
  const int c0 = static_cast<int>(idx % groups) * V;
  Chunk<T> g, u, da, og, ou;
  const int goff = 16 * (c0 / 8) + (c0 % 8);
  g.load(h + row * 2 * d_ff + goff);
  u.load(h + row * 2 * d_ff + goff + 8);
  da.load(d_a + row * d_ff + c0);
  float dg[V], du[V];
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const float gv = g.get(i), sg = 1.0f / (1.0f + __expf(-gv));
    dg[i] = da.get(i) * u.get(i) * sg * (1.0f + gv * (1.0f - sg));
    du[i] = da.get(i) * gv * sg;
  }
#pragma unroll
  for (int i = 0; i < V / 2; ++i) {
    og.set_pair(i, dg[2 * i], dg[2 * i + 1]);
    ou.set_pair(i, du[2 * i], du[2 * i + 1]);
  }
  og.store(d_h + row * 2 * d_ff + goff);
  ou.store(d_h + row * 2 * d_ff + goff + 8);
}

// dst = a + b, 16 bytes per thread
template <typename T>
__global__ __launch_bounds__(256) void add_kernel(const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ dst,
                                                  int64_t n_chunks) {
  constexpr int V = Chunk<T>::kElems;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= n_chunks) return;
  Chunk<T> x, y, o;
  x.load(a + idx * V);
  y.load(b + idx * V);
#pragma unroll
  for (int i = 0; i < V / 2; ++i) o.set_pair(i, x.get(2 * i) + y.get(2 * i), x.get(2 * i + 1) + y.get(2 * i + 1));
  o.store(dst + idx * V);
}

// tok_of_pos[p] = perm[p] / K for the sorted positions of a routing decision made elsewhere
__global__ __launch_bounds__(256) void tok_of_pos_kernel(const int32_t *__restrict__ perm, int top_k,
                                                         int64_t n_slots, int32_t *__restrict__ tok_of_pos) {
  const int64_t p = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (p < n_slots) tok_of_pos[p] = perm[p] / top_k;
}

// one wavefront per sorted position: rstd_sorted[p] = 1 / sqrt(mean(x[tok_of_pos[p], :]^2) + eps)
template <typename T>
__global__ __launch_bounds__(256) void rstd_sorted_kernel(const T *__restrict__ x, int d_model,
                                                          const int32_t *__restrict__ tok_of_pos,
                                                          int64_t n_slots, float eps,
                                                          float *__restrict__ rstd_sorted) {
  constexpr int V = Chunk<T>::kElems;
  const int lane = threadIdx.x & 63;
  const int64_t p = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
  if (p >= n_slots) return;                       // whole wavefront
  const T *row = x + static_cast<int64_t>(tok_of_pos[p]) * d_model;
  float ss = 0.0f;
  for (int c0 = lane * V; c0 < d_model; c0 += 64 * V) {
    Chunk<T> c;
    c.load(row + c0);
#pragma unroll
    for (int i = 0; i < V; ++i) ss = fmaf(c.get(i), c.get(i), ss);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) ss += __shfl_xor(ss, o, 64);
  if (lane == 0) rstd_sorted[p] = 1.0f / sqrtf(ss / static_cast<float>(d_model) + eps);
}

// ------------------------------------------------------------------ timing probes (bench.py --probe)
// What a wavefront can issue, measured rather than assumed: chains of one instruction kind,
// dependent or independent, at a chosen number of wavefronts per SIMD; and the pipelined scan's
// tile with parts switched off and without its memory traffic.  Not on any product path.
template <int CHAINS, int OP>   // OP 0: v_fma_f32, 1: v_exp_f32, 2: v_mov_b32_dpp (row broadcast)
__global__ __launch_bounds__(256) void probe_issue_kernel(float *out, int iters, float a, float b) {
  float acc[CHAINS];
#pragma unroll
  for (int c = 0; c < CHAINS; ++c) acc[c] = threadIdx.x * 1e-3f + c;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int r = 0; r < 64 / CHAINS; ++r) {
#pragma unroll
      for (int c = 0; c < CHAINS; ++c) {
        if (OP == 0) asm volatile("v_fma_f32 %0, %1, %0, %2" : "+v"(acc[c]) : "v"(a), "v"(b));
        if (OP == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(acc[c]));
        if (OP == 2) asm volatile("v_mov_b32_dpp %0, %0 row_newbcast:3 row_mask:0xf bank_mask:0xf" : "+v"(acc[c]));
      }
    }
  }
  float s = 0.0f;
#pragma unroll
  for (int c = 0; c < CHAINS; ++c) s += acc[c];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// PARTS as in scan_pipe_slot; LDS 0: registers only, 1: + the tile's LDS reads, 2: + a barrier and an LDS write per tile
template <int PARTS, int LDS>
__global__ __launch_bounds__(256) void probe_scan_kernel(float *out, int tiles) {
  __shared__ ScanSmem sm;
  __shared__ float g_tile[kScanTile][kChPitch];
  const int tid = threadIdx.x, n = tid & 15, cl = tid >> 4;
  for (int i = tid; i < static_cast<int>(sizeof(ScanSmem) / 4); i += 256) reinterpret_cast<float *>(&sm)[i] = 1e-3f * (i % 97);
  for (int i = tid; i < kScanTile * kChPitch; i += 256) (&g_tile[0][0])[i] = 0.0f;
  __syncthreads();
  ScanPipeRegs r;
  r.a2 = -0.5f - n; r.d_skip = 1.0f; r.h = 0.1f * n; r.y = 0.0f;
  r.hi8 = (n & 8) != 0; r.hi4 = (n & 4) != 0; r.hi2 = (n & 2) != 0; r.hi1 = (n & 1) != 0;
  for (int gi = 0; gi < kScanGroups; ++gi) {
    r.dt_r[gi] = 0.01f * (gi + 1); r.u_r[gi] = 0.5f; r.dtu_r[gi] = 0.005f; r.z_r[gi] = 0.3f;
    for (int j = 0; j < 16; ++j) { r.bv[gi][j] = 0.1f * j; r.cv[gi][j] = 0.2f; }
  }
  for (int j = 0; j < 16; ++j) { r.da[0][j] = r.da[1][j] = 0.99f; r.xx[0][j] = r.xx[1][j] = 0.01f; r.hs[0][j] = r.hs[1][j] = 0.0f; }
  for (int j = 0; j < 8; ++j) r.ra[j] = 0.0f;
  for (int j = 0; j < 4; ++j) r.rb[j] = 0.0f;
  r.rc[0] = r.rc[1] = 0.0f;
  for (int t = 0; t < tiles; ++t) {
    if (LDS >= 1) {
#pragma unroll
      for (int gi = 0; gi < kScanGroups; ++gi) {
        r.dt_r[gi] = sm.dt[gi * 16 + n][cl];
        r.u_r[gi] = sm.u[gi * 16 + n][cl];
        r.dtu_r[gi] = r.dt_r[gi] * r.u_r[gi];
        scan_pipe_read16(r.bv[gi], &sm.bc[n][gi * 16]);
        scan_pipe_read16(r.cv[gi], &sm.bc[16 + n][gi * 16]);
        r.z_r[gi] = sm.zg[gi * 16 + n][cl];
      }
    } else {
#pragma unroll
      for (int gi = 0; gi < kScanGroups; ++gi) r.dt_r[gi] += r.h * 1e-30f;     // keeps the work inside the loop
    }
    __builtin_amdgcn_sched_barrier(0);
    ScanPipePhases<kScanGroups, PARTS>::run(r, g_tile, n, cl);
    if (LDS >= 2) {
      __syncthreads();
      sm.dt[tid >> 2][(tid & 3) * 4] = g_tile[tid >> 2][(tid & 3) * 4] * 1e-9f + 0.01f;
    }
  }
  float s = r.h + r.y;
  for (int j = 0; j < 16; ++j) s += r.da[0][j] + r.da[1][j] + r.xx[0][j] + r.xx[1][j] + r.hs[0][j] + r.hs[1][j];
  for (int j = 0; j < 8; ++j) s += r.ra[j];
  out[blockIdx.x * 256 + tid] = s + g_tile[tid & 63][0];
}

inline dim3 grid1d(int64_t work, int block) { return dim3(static_cast<unsigned>(ceil_div(work, block))); }

}  // namespace

hipError_t launch_slot_sum(int src_is_f32, int dst_is_f32, const void *src, int64_t ld_src, void *dst,
                           int64_t ld_dst, const int32_t *inv_perm, int64_t n_tokens, int top_k,
                           int n_cols, const float *bias, int softplus, const float *row_scale,
                           hipStream_t s) {
  const bool wide = n_cols % 8 == 0 && ld_src % 8 == 0 && ld_dst % 8 == 0 &&
                    reinterpret_cast<uintptr_t>(src) % 16 == 0 && reinterpret_cast<uintptr_t>(dst) % 16 == 0 &&
                    (!bias || reinterpret_cast<uintptr_t>(bias) % 16 == 0);
  const dim3 grid = wide ? grid1d(n_tokens * (n_cols / 8), 256) : grid1d(n_tokens * ((n_cols + 1) / 2), 256);
#define ROM_SS(TS, TD)                                                                            \
  do {                                                                                            \
    if (wide)                                                                                     \
      hipLaunchKernelGGL((slot_sum8_kernel<TS, TD>), grid, dim3(256), 0, s, static_cast<const TS *>(src), \
                         ld_src, static_cast<TD *>(dst), ld_dst, inv_perm, n_tokens, top_k, n_cols, \
                         bias, softplus, row_scale);                                              \
    else                                                                                          \
      hipLaunchKernelGGL((slot_sum_kernel<TS, TD>), grid, dim3(256), 0, s, static_cast<const TS *>(src), \
                         ld_src, static_cast<TD *>(dst), ld_dst, inv_perm, n_tokens, top_k, n_cols, \
                         bias, softplus, row_scale);                                              \
  } while (0)
  if (src_is_f32 && dst_is_f32) ROM_SS(float, float);
  else if (src_is_f32) ROM_SS(float, bf16_t);
  else if (dst_is_f32) ROM_SS(bf16_t, float);
  else ROM_SS(bf16_t, bf16_t);
#undef ROM_SS
  return hipGetLastError();
}

hipError_t launch_swiglu(int dtype, const void *h, void *a, int64_t n_rows, int d_ff, hipStream_t s) {
  const int V = dtype == ROM_DTYPE_BF16 ? 8 : 4;
  const dim3 grid = grid1d(n_rows * (d_ff / V), 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(swiglu_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(h),
                       static_cast<bf16_t *>(a), n_rows, d_ff);
  else
    hipLaunchKernelGGL(swiglu_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(h),
                       static_cast<float *>(a), n_rows, d_ff);
  return hipGetLastError();
}

hipError_t launch_swiglu_backward(int dtype, const void *h, const void *d_a, void *d_h, int64_t n_rows, int d_ff,
                                  hipStream_t s) {
  const int V = dtype == ROM_DTYPE_BF16 ? 8 : 4;
  const dim3 grid = grid1d(n_rows * (d_ff / V), 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(swiglu_bwd_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(h),
                       static_cast<const bf16_t *>(d_a), static_cast<bf16_t *>(d_h), n_rows, d_ff);
  else
    hipLaunchKernelGGL(swiglu_bwd_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(h),
                       static_cast<const float *>(d_a), static_cast<float *>(d_h), n_rows, d_ff);
  return hipGetLastError();
}

hipError_t launch_add(int dtype, const void *a, const void *b, void *dst, int64_t n_elems, hipStream_t s) {
  const int V = dtype == ROM_DTYPE_BF16 ? 8 : 4;
  if (n_elems % V != 0) return hipErrorInvalidValue;
  const dim3 grid = grid1d(n_elems / V, 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(add_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(a),
                       static_cast<const bf16_t *>(b), static_cast<bf16_t *>(dst), n_elems / V);
  else
    hipLaunchKernelGGL(add_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(a),
                       static_cast<const float *>(b), static_cast<float *>(dst), n_elems / V);
  return hipGetLastError();
}

hipError_t launch_ffn_prep(int dtype, const int32_t *perm, int top_k, int64_t n_slots, const void *x,
                           int d_model, float eps, int32_t *tok_of_pos, float *rstd_sorted, hipStream_t s) {
  hipLaunchKernelGGL(tok_of_pos_kernel, grid1d(n_slots, 256), dim3(256), 0, s, perm, top_k, n_slots, tok_of_pos);
  if (rstd_sorted) {
    const dim3 grid = grid1d(n_slots * 64, 256);
    if (dtype == ROM_DTYPE_BF16)
      hipLaunchKernelGGL(rstd_sorted_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(x),
                         d_model, tok_of_pos, n_slots, eps, rstd_sorted);
    else
      hipLaunchKernelGGL(rstd_sorted_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(x),
                         d_model, tok_of_pos, n_slots, eps, rstd_sorted);
  }
  return hipGetLastError();
}

int xproj_k_splits(int64_t rows, int n_groups, int d_inner) {
  // The x projection has a single column tile, so its grid is the number of 256-row tiles: far
  // fewer than CUs.  Slicing the long inner dimension shortens every workgroup's slab loop but
  // each slice writes fp32 partial sums that split_xdbl has to read back.  Pick the slice count
  // with the smallest estimate  slabs / s * t_slab + s * rows * t_row  (measured on MI355X:
  // about 0.87 us per 64-wide slab and 12 us per slice at 16384 rows), at most one workgroup per CU.
  const int by_len = d_inner / 512;
  const int64_t tiles = rows / 256 + n_groups;
  int64_t s_max = 256 / tiles;
  if (s_max > by_len) s_max = by_len;
  if (s_max > 8) s_max = 8;
  const double slabs = d_inner / 64.0, per_slice = 12.0 * static_cast<double>(rows) / 16384.0;
  int best = 1;
  double best_t = slabs * 0.87 + per_slice;
  for (int s = 2; s <= s_max; ++s) {
    const double t = slabs / s * 0.87 + s * per_slice;
    if (t < best_t) { best_t = t; best = s; }
  }
  return best;
}

hipError_t launch_split_xdbl(int dtype, const float *xdbl, int n_slices, int64_t slice_stride,
                             const int32_t *inv_perm, int top_k, int64_t n_tokens, int dt_rank,
                             void *dt_low, float *bc, hipStream_t s) {
  const dim3 grid = grid1d(n_tokens * (dt_rank + 32), 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(split_xdbl_kernel<bf16_t>, grid, dim3(256), 0, s, xdbl, n_slices, slice_stride,
                       inv_perm, top_k,
                       n_tokens, dt_rank, static_cast<bf16_t *>(dt_low), bc);
  else
    hipLaunchKernelGGL(split_xdbl_kernel<float>, grid, dim3(256), 0, s, xdbl, n_slices, slice_stride,
                       inv_perm, top_k,
                       n_tokens, dt_rank, static_cast<float *>(dt_low), bc);
  return hipGetLastError();
}

hipError_t launch_conv_silu(int dtype, const void *xz, int64_t ld_xz, const float *conv_w,
                            const float *conv_b, const float *state_in, float *state_out, void *u,
                            int64_t B, int64_t L, int d_inner, hipStream_t s) {
  const int V = dtype == ROM_DTYPE_BF16 ? 8 : 4;
  const int groups = d_inner / V;
  const dim3 grid(static_cast<unsigned>(ceil_div(groups, 256)),
                  static_cast<unsigned>(ceil_div(L, kConvRun)), static_cast<unsigned>(B));
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(conv_silu_kernel<bf16_t>, grid, dim3(256), 0, s,
                       static_cast<const bf16_t *>(xz), ld_xz, conv_w, conv_b, state_in, state_out,
                       static_cast<bf16_t *>(u), L, d_inner);
  else
    hipLaunchKernelGGL(conv_silu_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(xz),
                       ld_xz, conv_w, conv_b, state_in, state_out, static_cast<float *>(u), L, d_inner);
  return hipGetLastError();
}

int scan_chunks(int64_t B, int64_t L, int d_inner) {
  // chunk only when there are fewer workgroups than CUs (256): the state-only pass costs about as
  // much as the better occupancy of the full pass gains once every SIMD has a wavefront; chunks are whole tiles and at least 256 steps long
  const int64_t blocks = B * (d_inner / kScanCh);
  int64_t nc = ceil_div(256, blocks > 0 ? blocks : 1);
  const int64_t by_len = L / 256;
  if (nc > by_len) nc = by_len;
  if (nc > 8) nc = 8;
  if (nc < 1) nc = 1;
  return static_cast<int>(nc);
}

size_t scan_chunk_state_bytes(int64_t B, int64_t L, int d_inner) {
  const int nc = scan_chunks(B, L, d_inner);
  return static_cast<size_t>(B) * (nc > 1 ? nc : 0) * d_inner * 16 * sizeof(float);
}

template <typename T>
static hipError_t scan_dispatch(const T *u, const T *dt, const float *bc, const T *z, int64_t ld_z,
                                const float *A_log, const float *D, const float *h_in, float *h_out, T *g,
                                int64_t B, int64_t L, int d_inner, float *chunk_q, float *chunk_p,
                                hipStream_t s) {
  if (L == 1) {
    const int64_t lanes = B * d_inner * 4;
    hipLaunchKernelGGL((scan_step_kernel<T>), dim3(static_cast<unsigned>(ceil_div(lanes, 256))), dim3(256),
                       0, s, u, dt, bc, z, ld_z, A_log, D, h_in, h_out, g, B, d_inner);
    return hipGetLastError();
  }
  const int nc_max = scan_chunks(B, L, d_inner);
  const int64_t chunk_len = ceil_div(ceil_div(L, nc_max), kScanTile) * kScanTile;
  const int nc = static_cast<int>(ceil_div(L, chunk_len));      // no empty chunk after rounding
  const unsigned gx = static_cast<unsigned>(d_inner / kScanCh), gy = static_cast<unsigned>(B);
  if (nc > 1) {
    hipLaunchKernelGGL((scan_kernel<T, true, 1>), dim3(gx, gy, nc - 1), dim3(256), 0, s, u, dt, bc,
                       static_cast<const T *>(nullptr), ld_z, A_log, D, h_in,
                       static_cast<float *>(nullptr), static_cast<T *>(nullptr), L, d_inner, chunk_len, nc,
                       chunk_q, chunk_p);
  }
  // one block per CU or fewer: two tiles in LDS (one barrier per tile); else six small blocks per CU
  // one block per CU or fewer: the software-pipelined kernel with a helper wavefront beside every
  // compute wavefront; up to two blocks per CU: the same kernel without helpers (two tiles in LDS,
  // 58 KiB); beyond that six small blocks per CU
  const int64_t n_blocks = static_cast<int64_t>(gx) * gy * nc;
  if (kScanDouble && n_blocks <= 256)
    hipLaunchKernelGGL((scan_pipe_kernel<T, true>), dim3(gx, gy, nc), dim3(512), 0, s, u, dt, bc, z, ld_z, A_log,
                       D, h_in, h_out, g, L, d_inner, chunk_len, nc, chunk_q, chunk_p);
  else if (kScanDouble && n_blocks <= 512)
    hipLaunchKernelGGL((scan_pipe_kernel<T, false>), dim3(gx, gy, nc), dim3(256), 0, s, u, dt, bc, z, ld_z, A_log,
                       D, h_in, h_out, g, L, d_inner, chunk_len, nc, chunk_q, chunk_p);
  else
    hipLaunchKernelGGL((scan_kernel<T, false, 1>), dim3(gx, gy, nc), dim3(256), 0, s, u, dt, bc, z, ld_z, A_log,
                       D, h_in, h_out, g, L, d_inner, chunk_len, nc, chunk_q, chunk_p);
  return hipGetLastError();
}

hipError_t launch_scan_gate(int dtype, const void *u, const void *dt, const float *bc, const void *z,
                            int64_t ld_z, const float *A_log, const float *D, const float *h_in,
                            float *h_out, void *g, int64_t B, int64_t L, int d_inner, float *chunk_q,
                            float *chunk_p, hipStream_t s) {
  if (dtype == ROM_DTYPE_BF16)
    return scan_dispatch<bf16_t>(static_cast<const bf16_t *>(u), static_cast<const bf16_t *>(dt), bc,
                                 static_cast<const bf16_t *>(z), ld_z, A_log, D, h_in, h_out,
                                 static_cast<bf16_t *>(g), B, L, d_inner, chunk_q, chunk_p, s);
  return scan_dispatch<float>(static_cast<const float *>(u), static_cast<const float *>(dt), bc,
                              static_cast<const float *>(z), ld_z, A_log, D, h_in, h_out,
                              static_cast<float *>(g), B, L, d_inner, chunk_q, chunk_p, s);
}

hipError_t launch_probe_issue(int op, int chains, int n_blocks, int iters, float *out, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>(n_blocks)), block(256);
#define ROM_PROBE(C, OP)                                                                                 \
  if (chains == C && op == OP) {                                                                         \
    hipLaunchKernelGGL((probe_issue_kernel<C, OP>), grid, block, 0, s, out, iters, 0.999f, 1e-3f);       \
    return hipGetLastError();                                                                            \
  }
  ROM_PROBE(1, 0) ROM_PROBE(8, 0) ROM_PROBE(1, 1) ROM_PROBE(8, 1) ROM_PROBE(1, 2) ROM_PROBE(8, 2)
#undef ROM_PROBE
  return hipErrorInvalidValue;
}

hipError_t launch_probe_scan(int parts, int lds, int n_blocks, int tiles, float *out, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>(n_blocks)), block(256);
#define ROM_PROBE(P, M)                                                                     \
  if (parts == P && lds == M) {                                                             \
    hipLaunchKernelGGL((probe_scan_kernel<P, M>), grid, block, 0, s, out, tiles);           \
    return hipGetLastError();                                                               \
  }
  ROM_PROBE(3, 0) ROM_PROBE(6, 0) ROM_PROBE(7, 0) ROM_PROBE(7, 1) ROM_PROBE(7, 2)
#undef ROM_PROBE
  return hipErrorInvalidValue;
}

hipError_t launch_combine(int dtype, const void *op, const int32_t *inv_perm, const float *gate,
                          void *out, int64_t n_tokens, int top_k, int d_model, const void *residual,
                          hipStream_t s) {
  const int V = dtype == ROM_DTYPE_BF16 ? 8 : 4;
  const dim3 grid = grid1d(n_tokens * (d_model / V), 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t *>(op),
                       inv_perm, gate, static_cast<bf16_t *>(out), n_tokens, top_k, d_model,
                       static_cast<const bf16_t *>(residual));
  else
    hipLaunchKernelGGL(combine_kernel<float>, grid, dim3(256), 0, s, static_cast<const float *>(op),
                       inv_perm, gate, static_cast<float *>(out), n_tokens, top_k, d_model,
                       static_cast<const float *>(residual));
  return hipGetLastError();
}

}  // namespace rom
