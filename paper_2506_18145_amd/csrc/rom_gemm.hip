// Expert-grouped GEMM for the routed projections of the RoM layer (Eq. (10), (11), (13)):
//   C[c_row(p), :] = epilogue( A[a_row(p), :] . W[e(p)]^T )   for every sorted position p,
// where positions are grouped by expert (offsets[]) and both operands are K-contiguous
// (activations [rows, K], weights [expert][N, K]).  Rows are gathered / scattered through
// index maps, so no separate token-permute pass is needed.
//
// bf16 path: v_mfma_f32_32x32x16_bf16, 64-lane wavefronts, a workgroup of WM x WN waves owns a
// BM x BN tile; K is walked in slabs of 64 staged through double-buffered, XOR-swizzled LDS.
// Group sizes live in device memory: every workgroup finds its (expert, row tile) by walking
// the offsets, so skewed loads only change how many tiles an expert contributes.
// Epilogues (compile-time variants): plain store, bias + softplus, per-row scale (gate weight or
// 1 / rms), per-row scale + skip rows added, fp32 partial sums of inner-dimension slices, and
// SiLU(gate) * up over a weight whose rows interleave the two halves of a SwiGLU expert.
// fp32 path (and shapes the MFMA kernel does not take): a plain LDS-tiled FMA kernel.
#include <atomic>
#include <mutex>
#include <type_traits>

#include "rom_internal.h"

namespace rom {

namespace {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

__device__ __forceinline__ float softplus_f32(float v) { return v > 20.0f ? v : log1pf(__expf(v)); }
// branch-free softplus for the bf16 epilogues: max(v, 0) + log(1 + e) with e = exp(-|v|) in (0, 1].
// Where 1 + e would lose e to rounding, log(1 + e) = e - e^2/2 + ... is replaced by e itself; at the
// switch point (e = 2^-12) either form is within 1.3e-4 relative of the true value, an order of
// magnitude below the bf16 rounding of the stored result.  The raw exp2 / log2 instructions are used
// on purpose: their arguments are never denormal here, so the library's range fix-ups are dead weight
// in an epilogue that is bound by ALU issue.
__device__ __forceinline__ float softplus_fast(float v) {
  const float e = __builtin_amdgcn_exp2f(-1.44269504088896341f * fabsf(v));
  const float lg = __builtin_amdgcn_logf(1.0f + e) * 0.693147180559945309f;
  return fmaxf(v, 0.0f) + (e < 2.44140625e-4f ? e : lg);
}

struct TileCoord {
  int group;
  int64_t row0, row_end;   // sorted positions covered by this tile: [row0, row_end)
  int n0;
  bool valid;
};

// logical tile id -> (global row tile, column tile) in patches of 32 tiles, PM x PN with PN = up
// to 8 column tiles (fewer when the output is narrower), so that workgroups that run together
// share activation row tiles and weight column tiles.
constexpr int kPatchTiles = 32, kPatchNMax = 8;
constexpr bool kXcdRemap = true;    // hand each XCD (workgroup id mod 8) a contiguous run of tiles

__host__ __device__ __forceinline__ int patch_n_for(int n_tiles) {
  int pn = 1;
  while (pn < kPatchNMax && pn < n_tiles) pn *= 2;
  return pn;
}

__device__ __forceinline__ TileCoord locate_tile(const GemmArgs &a, int BM, int BN) {
  TileCoord tc;
  tc.valid = false;
  const int n_tiles = (a.N + BN - 1) / BN;
  const int pn = patch_n_for(n_tiles), pm = kPatchTiles / pn;
  const int patches_n = (n_tiles + pn - 1) / pn;
  const int G = gridDim.x;
  const int bid = blockIdx.x;
  int t = bid;
  if (kXcdRemap && !a.no_xcd_remap && G % 8 == 0) t = (bid % 8) * (G / 8) + bid / 8;
  const int patch = t / kPatchTiles, in_patch = t % kPatchTiles;
  const int mt = (patch / patches_n) * pm + in_patch % pm;
  const int nt = (patch % patches_n) * pn + in_patch / pm;
  if (nt >= n_tiles) return tc;
  tc.n0 = nt * BN;
  if (a.offsets == nullptr) {
    tc.group = 0;
    tc.row0 = static_cast<int64_t>(mt) * BM;
    tc.row_end = a.M;
    tc.valid = tc.row0 < a.M;
  } else {
    int rem = mt;
    for (int e = 0; e < a.n_groups; ++e) {
      const int lo = a.offsets[e], hi = a.offsets[e + 1];
      const int tiles = (hi - lo + BM - 1) / BM;
      if (rem < tiles) {
        tc.group = e;
        tc.row0 = lo + static_cast<int64_t>(rem) * BM;
        tc.row_end = hi;
        tc.valid = true;
        break;
      }
      rem -= tiles;
    }
  }
  if (tc.valid && tc.row_end > tc.row0 + BM) tc.row_end = tc.row0 + BM;
  return tc;
}

// epilogue variants of the MFMA kernel (compile-time, so the store loop has no branches)
enum { kEpiPlain = 0, kEpiBiasSoftplus = 1, kEpiRowScale = 2, kEpiPlainF32 = 3, kEpiRowScaleResidual = 4,
       kEpiSwiGLU = 5 };

__device__ __forceinline__ void store_out(const GemmArgs &a, int64_t crow, int col, float v) {
  if (a.bias) v += a.bias[col];
  if (a.softplus) v = softplus_f32(v);
  if (a.row_scale) v *= a.row_scale[crow];
  if (a.residual)
    v += a.dtype == ROM_DTYPE_F32 ? static_cast<const float *>(a.residual)[crow * a.ldc + col]
                                  : bf16_to_f32(static_cast<const bf16_t *>(a.residual)[crow * a.ldc + col]);
  if (a.c_is_f32 || a.dtype == ROM_DTYPE_F32)
    static_cast<float *>(a.C)[blockIdx.y * a.c_split_stride + crow * a.ldc + col] = v;
  else
    static_cast<bf16_t *>(a.C)[crow * a.ldc + col] = f32_to_bf16(v);
}

// ------------------------------------------------------------------ bf16 MFMA kernel
constexpr int kBK = 64;                 // K slab, 8 chunks of 8 bf16 (16 bytes) per row
constexpr int kRowChunks = kBK / 8;
// LDS swizzle: chunk c of tile row r lives in slot c ^ lds_swizzle(r) of that row.  Two rows span
// the 64 four-byte banks, and a 16-byte-per-lane read is served 16 lanes (rows) at a time, so 16
// consecutive rows reading the same logical chunk must land in 16 different (row parity, slot)
// pairs; (r & 7) ^ ((r >> 3) & 1) does that and stays conflict-free on 8-row groups as well.
__device__ __forceinline__ int lds_swizzle(int r) { return (r & 7) ^ ((r >> 3) & 1); }

// Epilogue shared by the MFMA kernels.  The weight fragment is the MFMA's row operand, so a lane
// holds, for ONE output row (tile row lane%32), the output columns 8*q + 4*(lane/32) + r of each
// 32-wide tile in accumulator element 4*q + r: four consecutive columns per q.
template <int EPI, int TM, int TN, int WTM, int WTN>
__device__ __forceinline__ void mfma_epilogue(const GemmArgs &a, const TileCoord &tc, f32x16_t (&acc)[TM][TN],
                                              uint4 *smem, int wave, int wm, int wn, int lane) {
  const int frag_row = lane & 31, frag_half = lane >> 5;
  if constexpr (EPI == kEpiPlainF32) {
    // fp32 output: one 16-byte store per q straight from the accumulators
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int64_t p = tc.row0 + wm * WTM + i * 32 + frag_row;
      const bool row_ok = p < tc.row_end;
      const int64_t crow = row_ok ? (a.c_rows ? a.c_rows[p] : p) : 0;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = tc.n0 + wn * WTN + j * 32 + q * 8 + frag_half * 4;
          if (row_ok && col < a.N)
            *reinterpret_cast<float4 *>(static_cast<float *>(a.C) + blockIdx.y * a.c_split_stride +
                                        crow * a.ldc + col) =
                make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        }
      }
    }
  } else if constexpr (EPI == kEpiSwiGLU) {
    // The weight's rows come in blocks of 16: gate features 8b..8b+7, then up features 8b..8b+7.
    // A lane's accumulator elements 8m..8m+3 and 8m+4..8m+7 of a 32-wide tile are then the gate
    // and the up pre-activation of the same four features of the same row, so
    // SiLU(gate) * up is formed in registers and the output tile is half as wide as the product.
    constexpr int kOutW = WTN / 2;
    constexpr int kPitch = kOutW * 2 + 16;
    char *stage = reinterpret_cast<char *>(smem) + wave * (32 * kPitch);
    constexpr int kChunks = kOutW / 8;
    constexpr int kRowsPerPass = 64 / kChunks;
    const int chunk = lane % kChunks, sub = lane / kChunks;
    const int col = (tc.n0 + wn * WTN) / 2 + chunk * 8;
    const int n_out = a.N / 2;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      float scale = 1.0f;
      if (a.row_scale) {                   // pre-norm: 1 / rms of the row, before the activation
        const int64_t p = tc.row0 + wm * WTM + i * 32 + frag_row;
        scale = p < tc.row_end ? a.row_scale[a.c_rows ? a.c_rows[p] : p] : 0.0f;
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int m = 0; m < 2; ++m) {
          float o[4];
#pragma unroll
          for (int r = 0; r < 4; ++r)
            o[r] = silu_f32(acc[i][j][8 * m + r] * scale) * (acc[i][j][8 * m + 4 + r] * scale);
          uint2 pk;
          pk.x = pack_bf16x2(o[0], o[1]);
          pk.y = pack_bf16x2(o[2], o[3]);
          const int lcol = (j * 2 + m) * 8 + frag_half * 4;
          *reinterpret_cast<uint2 *>(stage + frag_row * kPitch + lcol * 2) = pk;
        }
      }
#pragma unroll 4
      for (int r0 = 0; r0 < 32; r0 += kRowsPerPass) {
        const int row = r0 + sub;
        const int64_t p = tc.row0 + wm * WTM + i * 32 + row;
        if (row < 32 && p < tc.row_end && col < n_out) {
          const int64_t crow = a.c_rows ? a.c_rows[p] : p;
          const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * kPitch + chunk * 16);
          *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.C) + crow * a.ldc + col) = v;
        }
      }
    }
  } else {
    // bf16 output: every wave parks 32 rows of its sub-tile at a time (after bias / softplus / row
    // scale) in its own slice of the now idle LDS, then writes them out row by row, 16 bytes per
    // lane, so that each store instruction covers whole 128..256-byte row segments.  No workgroup
    // barrier is needed: after the last slab's barrier nobody reads the operand buffers for real
    // any more, and LDS serves one wave's accesses in program order.
    constexpr int kPitch = WTN * 2 + 16;                 // bytes per parked row (16-byte aligned)
    char *stage = reinterpret_cast<char *>(smem) + wave * (32 * kPitch);
    constexpr int kChunks = WTN / 8;                     // 16-byte chunks per parked row
    constexpr int kRowsPerPass = 64 / kChunks;
    const int chunk = lane % kChunks, sub = lane / kChunks;
    const int col = tc.n0 + wn * WTN + chunk * 8;
    constexpr int kPasses = (32 + kRowsPerPass - 1) / kRowsPerPass;
    // skip connection: the block's input rows, in the output's layout.  All of them are fetched
    // before the first output store: loads and stores retire through one in-order counter, so a
    // load issued behind a store could only be waited for together with that store.
    u32x4_t res[EPI == kEpiRowScaleResidual ? TM : 1][EPI == kEpiRowScaleResidual ? kPasses : 1];
    if constexpr (EPI == kEpiRowScaleResidual) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int ps = 0; ps < kPasses; ++ps) {
          const int row = ps * kRowsPerPass + sub;
          const int64_t p = tc.row0 + wm * WTM + i * 32 + row;
          res[i][ps] = u32x4_t{0u, 0u, 0u, 0u};
          if (row < 32 && p < tc.row_end && col < a.N) {
            const int64_t crow = a.c_rows ? a.c_rows[p] : p;
            res[i][ps] = *reinterpret_cast<const u32x4_t *>(static_cast<const bf16_t *>(a.residual) +
                                                            crow * a.ldc + col);
          }
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      float scale = 1.0f;
      if (EPI == kEpiRowScale || EPI == kEpiRowScaleResidual) {
        const int64_t p = tc.row0 + wm * WTM + i * 32 + frag_row;
        // (the residual epilogue without a row scale: accumulation into the output, scale 1)
        scale = p < tc.row_end ? (a.row_scale ? a.row_scale[a.c_rows ? a.c_rows[p] : p] : 1.0f) : 0.0f;
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int lcol = j * 32 + q * 8 + frag_half * 4;
          float v[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[i][j][4 * q + r];
          if (EPI == kEpiBiasSoftplus) {
            const int bcol = tc.n0 + wn * WTN + lcol;
            float4 b4 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (bcol < a.N) b4 = *reinterpret_cast<const float4 *>(a.bias + bcol);
            v[0] = softplus_fast(v[0] + b4.x); v[1] = softplus_fast(v[1] + b4.y);
            v[2] = softplus_fast(v[2] + b4.z); v[3] = softplus_fast(v[3] + b4.w);
          }
          if (EPI == kEpiRowScale || EPI == kEpiRowScaleResidual) {
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] *= scale;
          }
          uint2 pk;
          pk.x = pack_bf16x2(v[0], v[1]);
          pk.y = pack_bf16x2(v[2], v[3]);
          *reinterpret_cast<uint2 *>(stage + frag_row * kPitch + lcol * 2) = pk;
        }
      }
      if constexpr (EPI == kEpiRowScaleResidual) {
#pragma unroll
        for (int ps = 0; ps < kPasses; ++ps) {
          const int row = ps * kRowsPerPass + sub;
          const int64_t p = tc.row0 + wm * WTM + i * 32 + row;
          if (row < 32 && p < tc.row_end && col < a.N) {
            const int64_t crow = a.c_rows ? a.c_rows[p] : p;
            uint4 v = *reinterpret_cast<const uint4 *>(stage + row * kPitch + chunk * 16);
            // added to the (already rounded) branch output here, where a lane holds 8 consecutive columns
            unsigned int *vw = &v.x;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              const float lo = __uint_as_float(vw[w] << 16) + __uint_as_float(res[i][ps][w] << 16);
              const float hi = __uint_as_float(vw[w] & 0xFFFF0000u) + __uint_as_float(res[i][ps][w] & 0xFFFF0000u);
              vw[w] = pack_bf16x2(lo, hi);
            }
            *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.C) + crow * a.ldc + col) = v;
          }
        }
      } else {
#pragma unroll 4
        for (int r0 = 0; r0 < 32; r0 += kRowsPerPass) {
          const int row = r0 + sub;
          const int64_t p = tc.row0 + wm * WTM + i * 32 + row;
          if (row < 32 && p < tc.row_end && col < a.N) {
            const int64_t crow = a.c_rows ? a.c_rows[p] : p;
            const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * kPitch + chunk * 16);
            *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.C) + crow * a.ldc + col) = v;
          }
        }
      }
    }
  }
}

// Scheduling hints for one 16-wide step: after MFMA number I, one LDS fragment read (while there
// are any) and this MFMA's share of the LDS writes that park the next slab.
template <int MMA, int READS, int PARKS, bool WITH_PARKS, int I> struct InterleaveHints {
  __device__ static __forceinline__ void run() {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA
    if constexpr (I < READS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one DS read
    if constexpr (WITH_PARKS) {
      constexpr int lo = I * PARKS / MMA, hi = (I + 1) * PARKS / MMA;
      if constexpr (hi > lo) __builtin_amdgcn_sched_group_barrier(0x200, hi - lo, 0);   // DS writes
    }
    InterleaveHints<MMA, READS, PARKS, WITH_PARKS, I + 1>::run();
  }
};
template <int MMA, int READS, int PARKS, bool WITH_PARKS>
struct InterleaveHints<MMA, READS, PARKS, WITH_PARKS, MMA> {
  __device__ static __forceinline__ void run() {}
};

// PA / PB: how many K slabs ahead the global loads of the activation / weight operand run
// (1 or 2; each extra slab costs one more register set for that operand).
// KTAIL: K is not a multiple of the slab, the last slab is zero-filled past K.
template <int BM, int BN, int WM, int WN, int EPI, bool KTAIL, int PA = 2, int PB = 2>
__global__ __launch_bounds__(WM *WN * 64) void gemm_bf16_mfma_kernel(const GemmArgs a) {
  constexpr int NT = WM * WN * 64;
  constexpr int WTM = BM / WM, WTN = BN / WN;       // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;       // 32x32 MFMA tiles per wave
  constexpr int A_CH = BM * kRowChunks / NT, B_CH = BN * kRowChunks / NT;
  static_assert(BM * kRowChunks % NT == 0 && BN * kRowChunks % NT == 0, "tile/threads mismatch");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32");

  extern __shared__ __attribute__((aligned(16))) uint4 smem[];
  uint4 *As = smem;                                  // [2][BM * 8] chunks
  uint4 *Bs = smem + 2 * BM * kRowChunks;            // [2][BN * 8] chunks

  const TileCoord tc = locate_tile(a, BM, BN);
  if (!tc.valid) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;
  const bf16_t *Ap = static_cast<const bf16_t *>(a.A);
  const bf16_t *Wp = static_cast<const bf16_t *>(a.W) + static_cast<int64_t>(tc.group) * a.N * a.K;

  // global source of every 16-byte chunk this thread stages.  Rows past the end of the tile are
  // redirected to its first row (their results are never stored), so the loads need no branch;
  // a K tail is zero-filled by a select.
  // (32-bit element offsets from the operand bases: the launcher checks that both operands span
  // less than 2^32 elements, and registers are scarce here)
  uint32_t a_src[A_CH], b_src[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int q = tid + i * NT, r = q / kRowChunks;
    int64_t p = tc.row0 + r;
    if (p >= tc.row_end) p = tc.row0;
    a_src[i] = static_cast<uint32_t>((a.a_rows ? a.a_rows[p] : p) * a.lda);
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int q = tid + i * NT, r = q / kRowChunks;
    const int n = (tc.n0 + r < a.N) ? tc.n0 + r : a.N - 1;
    b_src[i] = static_cast<uint32_t>(n) * static_cast<uint32_t>(a.K);
  }
  // split-K: grid.y slices of k_per_split inner-dimension elements, each with its own fp32 output
  const int k_begin = blockIdx.y * a.k_per_split;
  const int k_len = (a.K - k_begin < a.k_per_split) ? a.K - k_begin : a.k_per_split;
  const int k_chunk = k_begin + (tid % kRowChunks) * 8;
  const int k_last = k_begin + k_len - 8;

  // Register sets for slabs in flight: with depth 2 the global loads of slab kt+2 are issued while
  // slab kt is multiplied, so they have two slab times to land before they are parked in LDS
  // (HBM latency is longer than one slab of MFMA work).
  // (separate arrays with compile-time selection: the compiler keeps them in registers only if
  // every index is a constant and the arrays are never passed around by reference)
  uint4 ra0[A_CH], ra1[A_CH], rb0[B_CH], rb1[B_CH];
  auto load_a = [&](int k0, auto set) __attribute__((always_inline)) {
    constexpr int S = decltype(set)::value;
    const int k = k0 + k_chunk;
    const bool k_ok = !KTAIL || k <= k_last;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (!KTAIL || k0 + kBK <= k_len) v = *reinterpret_cast<const uint4 *>(Ap + a_src[i] + k);
      else if (k_ok) v = *reinterpret_cast<const uint4 *>(Ap + a_src[i] + k);
      if constexpr (S == 0) ra0[i] = v; else ra1[i] = v;
    }
  };
  // 64-row tiles serve launches with a few rows per expert (the recurrent step): every weight is
  // used once or twice, so it is streamed past the caches (non-temporal) and the activations,
  // states and routing arrays keep their place in L2 / the infinity cache (measured: -10 % per step)
  constexpr bool kStreamW = BM == 64;
  auto load_w = [&](const bf16_t *src) __attribute__((always_inline)) {
    if constexpr (kStreamW) {
      const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(src));
      return make_uint4(t.x, t.y, t.z, t.w);
    } else {
      return *reinterpret_cast<const uint4 *>(src);
    }
  };
  auto load_b = [&](int k0, auto set) __attribute__((always_inline)) {
    constexpr int S = decltype(set)::value;
    const int k = k0 + k_chunk;
    const bool k_ok = !KTAIL || k <= k_last;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (!KTAIL || k0 + kBK <= k_len) v = load_w(Wp + b_src[i] + k);
      else if (k_ok) v = load_w(Wp + b_src[i] + k);
      if constexpr (S == 0) rb0[i] = v; else rb1[i] = v;
    }
  };
  auto park_a = [&](int buf, auto set) __attribute__((always_inline)) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int q = tid + i * NT, r = q / kRowChunks, c = q % kRowChunks;
      uint4 v;
      if constexpr (S == 0) v = ra0[i]; else v = ra1[i];
      As[buf * BM * kRowChunks + r * kRowChunks + (c ^ lds_swizzle(r))] = v;
    }
  };
  auto park_b = [&](int buf, auto set) __attribute__((always_inline)) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int q = tid + i * NT, r = q / kRowChunks, c = q % kRowChunks;
      uint4 v;
      if constexpr (S == 0) v = rb0[i]; else v = rb1[i];
      Bs[buf * BN * kRowChunks + r * kRowChunks + (c ^ lds_swizzle(r))] = v;
    }
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int KT = (k_len + kBK - 1) / kBK;
  const int frag_row = lane & 31, frag_half = lane >> 5;
  // LDS chunk index of this lane's fragment for 16-wide K step kk: row * 8 + ((2 kk + half) ^ swizzle(row));
  // the wave / tile row offsets are multiples of 32, so the swizzle term depends on the lane only.
  const int a_base = (wm * WTM + frag_row) * kRowChunks, b_base = (wn * WTN + frag_row) * kRowChunks;
  const int swz = lds_swizzle(frag_row);

  bf16x8_t fa[2][TM], fb[2][TN];
  auto load_frags = [&](int buf, int kk, bf16x8_t(&af)[TM], bf16x8_t(&bfr)[TN]) __attribute__((always_inline)) {
    const int c = (kk * 2 + frag_half) ^ swz;
    const uint4 *Ab = As + buf * BM * kRowChunks + a_base + c;
    const uint4 *Bb = Bs + buf * BN * kRowChunks + b_base + c;
    // issue order = order of first use by mma(): A row 0, then every B column, then the other A rows
    {
      const uint4 v = Ab[0];
      af[0] = *reinterpret_cast<const bf16x8_t *>(&v);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const uint4 v = Bb[j * 32 * kRowChunks];
      bfr[j] = *reinterpret_cast<const bf16x8_t *>(&v);
    }
#pragma unroll
    for (int i = 1; i < TM; ++i) {
      const uint4 v = Ab[i * 32 * kRowChunks];
      af[i] = *reinterpret_cast<const bf16x8_t *>(&v);
    }
  };
  auto mma = [&](const bf16x8_t(&af)[TM], const bf16x8_t(&bfr)[TN]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
  };
  // ask the scheduler to put the next step's LDS fragment reads (and, in one step per slab, the
  // LDS writes that park the next slab) between the MFMAs of this step, one per MFMA
  auto interleave = [&](auto with_parks) __attribute__((always_inline)) {
    InterleaveHints<TM * TN, TM + TN, A_CH + B_CH, decltype(with_parks)::value, 0>::run();
  };

  load_a(0, Set0{});
  load_b(0, Set0{});
  park_a(0, Set0{});
  park_b(0, Set0{});
  const int k_end = (KT - 1) * kBK;      // loads past the last slab are redirected to it (and never used)
  if (PA == 2) load_a(kBK < k_end ? kBK : k_end, Set1{});
  if (PB == 2) load_b(kBK < k_end ? kBK : k_end, Set1{});
  __syncthreads();
  load_frags(0, 0, fa[0], fb[0]);

  // One K slab, free of conditionals: PAR = kt & 1 selects the LDS buffer being read; slab s of an
  // operand with depth P travels in register set s % P.  The slab after the last one is "loaded"
  // and parked like any other (clamped address, buffer nobody reads again).
  auto slab = [&](int kt, auto par) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par)::value;
    using LoadA = std::integral_constant<int, PA == 2 ? PAR : 0>;
    using LoadB = std::integral_constant<int, PB == 2 ? PAR : 0>;
    using ParkA = std::integral_constant<int, PA == 2 ? (PAR ^ 1) : 0>;
    using ParkB = std::integral_constant<int, PB == 2 ? (PAR ^ 1) : 0>;
    const int ka = (kt + PA) * kBK, kb = (kt + PB) * kBK;
    load_a(ka < k_end ? ka : k_end, LoadA{});
    load_b(kb < k_end ? kb : k_end, LoadB{});
    // The next slab (loaded while the previous one was multiplied) is parked in the middle of
    // this slab, its LDS writes spread between MFMAs, instead of in a burst before the barrier.
    constexpr int kParkAt = 3;       // 0..2: interleaved with that 16-wide step; 3: after the third step.
                                     // Measured: any earlier than 3 stalls on the loads still in flight.
    load_frags(PAR, 1, fa[1], fb[1]);
    if (kParkAt == 0) { park_a(PAR ^ 1, ParkA{}); park_b(PAR ^ 1, ParkB{}); }
    mma(fa[0], fb[0]);
    interleave(std::bool_constant<kParkAt == 0>{});
    load_frags(PAR, 2, fa[0], fb[0]);
    if (kParkAt == 1) { park_a(PAR ^ 1, ParkA{}); park_b(PAR ^ 1, ParkB{}); }
    mma(fa[1], fb[1]);
    interleave(std::bool_constant<kParkAt == 1>{});
    load_frags(PAR, 3, fa[1], fb[1]);
    if (kParkAt == 2) { park_a(PAR ^ 1, ParkA{}); park_b(PAR ^ 1, ParkB{}); }
    mma(fa[0], fb[0]);
    interleave(std::bool_constant<kParkAt == 2>{});
    if (kParkAt == 3) { park_a(PAR ^ 1, ParkA{}); park_b(PAR ^ 1, ParkB{}); }
    // every fragment of this slab is in registers and the next slab is parked: overlap the fetch
    // of its first fragments with the last 16-wide step of this one
    __syncthreads();
    load_frags(PAR ^ 1, 0, fa[0], fb[0]);
    mma(fa[1], fb[1]);
  };
  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    slab(kt, Set0{});
    slab(kt + 1, Set1{});
  }
  if (kt < KT) slab(kt, Set0{});

  mfma_epilogue<EPI, TM, TN, WTM, WTN>(a, tc, acc, smem, wave, wm, wn, lane);
}

// ------------------------------------------------------------------ bf16 MFMA kernel, LDS-DMA loads
// Same 256x256 tile and 4x2 wavefront layout, but the operand slabs travel from global memory
// straight into LDS (global_load_lds_dwordx4: lane l of a wave deposits its 16 bytes at M0 + 16 l),
// so no registers, no LDS-write instructions and no load->store dependency sit in the MFMA loop.
// K is walked in 64-wide slabs so that every row contributes one whole 128-byte cache line per
// slab.  A slab is two "half slabs" of 32 KiB (the 256 A rows, then the 256 W rows) and LDS is a
// ring of five such slots: while slab m (two slots) is multiplied, A(m+1), W(m+1) and A(m+2) are in
// flight or landed; the barrier before the last 16-wide step of slab m frees its two slots, which
// then receive W(m+2) and A(m+3).
// The XOR swizzle is applied on the global side: the lane that fills 16-byte position c' of row r
// fetches chunk c' ^ ((r >> 1) & 7), which keeps the 16-lane fragment reads conflict-free for
// 128-byte rows.  The compiler does not see these loads (inline asm), so the waits are explicit:
// every wave issues exactly four loads per half slab, in ring order, and "vmcnt(4)" therefore
// means "everything but the newest half slab I asked for has landed".
constexpr int kDmaBK = 64, kDmaRC = kDmaBK / 8, kDmaSlots = 5;
constexpr bool kUseDma = true;
constexpr int kSkinnyMinWgs = 100;
constexpr int kSkinnyColsMaxWgs = 600;    // fewer 64 x 128 tiles than this (about two per CU): 64 x 64 tiles instead
constexpr bool kUseSmallK = true;
constexpr int kBigWM = 4, kBigWN = 2;     // wave layout of the 256x256 DMA tile

__device__ __forceinline__ void dma_load_16(unsigned lds_addr, unsigned voff, const void *base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n"
               :: "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
}

// BN < 256 (a single, narrow column tile: the x projection) keeps the 256-row activation tile and
// the five 32 KiB ring slots; the weight half slabs just fill less of theirs.  grid.y slices the
// inner dimension (fp32 partial sums, plain epilogue only).
// WT: the weight is stored contraction-major, [group][K][N] (a forward weight used for the input
// gradient without a transposed copy; BN = 256, N a multiple of 256).  Its half slab is then 64
// contraction rows x 256 output columns as they lie in memory, two rows per DMA instruction, chunk c
// of row r at position c ^ 4 (r & 3), and the MFMA fragments - eight consecutive contraction indices of
// one output column per lane - come out of it through the transposing LDS read (ds_read_b64_tr_b16:
// the 16 lanes of a group name four rows x 16 columns, lane i receives column i of the four rows).
template <int BN, int WM, int WN, int EPI, bool WT = false>
__device__ __forceinline__ void dma_tile(const GemmArgs &a, const TileCoord &tc, uint4 *smem) {
  constexpr int BM = 256, NW = WM * WN;
  static_assert(kDmaSlots == 4 || kDmaSlots == 5, "ring of four or five half-slab slots");
  static_assert((NW == 16 || NW == 8 || NW == 4) && BN <= BM && BN % (32 * WN) == 0, "4, 8 or 16 waves, 32-wide MFMA tiles");
  constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
  constexpr int kSlotChunks = BM * kDmaRC;                    // 16-byte chunks per ring slot
  constexpr int kSlotBytes = kSlotChunks * 16;                // 32 KiB
  constexpr int kAInstr = BM / (8 * NW);                      // DMA instructions per wave and half slab: 8 rows each
  constexpr int kWInstr = (BN + 8 * NW - 1) / (8 * NW);       // (rows past BN are clamped re-reads into unused slot space)
  static_assert(!WT || (BN == 256 && NW == 8), "contraction-major weights: the 256 x 256 tile on eight waves");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WM, wn = wave / WM;
  const int k_begin = blockIdx.y * a.k_per_split;
  const int k_len = (a.K - k_begin < a.k_per_split) ? a.K - k_begin : a.k_per_split;
  const bf16_t *Ap = static_cast<const bf16_t *>(a.A) + k_begin;
  const bf16_t *Wp = static_cast<const bf16_t *>(a.W) + static_cast<int64_t>(tc.group) * a.N * a.K +
                     (WT ? static_cast<int64_t>(k_begin) * a.N : k_begin);

  // this lane's share of a half slab: one 16-byte chunk in each of its wave's 8-row groups
  unsigned a_voff[kAInstr], b_voff[kWInstr];
#pragma unroll
  for (int j = 0; j < kAInstr; ++j) {
    const int r = (wave * kAInstr + j) * 8 + (lane >> 3);      // tile row filled by this lane
    const int c = (lane & 7) ^ ((r >> 1) & 7);                 // global chunk that belongs in its position
    int64_t p = tc.row0 + r;
    if (p >= tc.row_end) p = tc.row0;                          // rows past the tile: never stored
    a_voff[j] = static_cast<unsigned>(((a.a_rows ? a.a_rows[p] : p) * a.lda + c * 8) * 2);
  }
#pragma unroll
  for (int j = 0; j < kWInstr; ++j) {
    if constexpr (WT) {
      const int r = (wave * kWInstr + j) * 2 + (lane >> 5);    // contraction row within the slab
      const int c = (lane & 31) ^ (4 * (r & 3));
      b_voff[j] = static_cast<unsigned>((static_cast<int64_t>(r) * a.N + tc.n0 + c * 8) * 2);
    } else {
      const int r = (wave * kWInstr + j) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ ((r >> 1) & 7);
      const int n = (tc.n0 + r < a.N) ? tc.n0 + r : a.N - 1;
      b_voff[j] = static_cast<unsigned>((static_cast<int64_t>(n) * a.K + c * 8) * 2);
    }
  }
  const unsigned lds_base =
      static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) void *)smem));
  const unsigned lds_wave_a = __builtin_amdgcn_readfirstlane(lds_base + wave * (kAInstr * 1024));
  const unsigned lds_wave_w = __builtin_amdgcn_readfirstlane(lds_base + wave * (kWInstr * 1024));
  const int KT = k_len / kDmaBK;

  // half slab h: the A rows (h even) or the W rows (h odd) of slab h / 2, into ring slot h % 5
  auto issue = [&](int h) __attribute__((always_inline)) {
    const int m = h >> 1;
    const int sl = m < KT ? m : KT - 1;                        // past the end: harmless reload
    const unsigned slot = static_cast<unsigned>(h % kDmaSlots) * kSlotBytes;
    if (h & 1) {
      const bf16_t *wb = Wp + (WT ? static_cast<int64_t>(sl) * kDmaBK * a.N : static_cast<int64_t>(sl) * kDmaBK);
#pragma unroll
      for (int j = 0; j < kWInstr; ++j) dma_load_16(lds_wave_w + slot + j * 1024, b_voff[j], wb);
    } else {
      const bf16_t *ab = Ap + sl * kDmaBK;
#pragma unroll
      for (int j = 0; j < kAInstr; ++j) dma_load_16(lds_wave_a + slot + j * 1024, a_voff[j], ab);
    }
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int a_base = (wm * WTM + frag_row) * kDmaRC, b_base = (wn * WTN + frag_row) * kDmaRC;
  const int swz = (frag_row >> 1) & 7;
  // contraction-major W: byte offset of this lane's 8 bytes in the first of its two 4-row reads
  unsigned wt_off[TN];
  if constexpr (WT) {
    const int i16 = lane & 15, grp = lane >> 4;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int chunk = (wn * (WTN / 8) + j * 4 + 2 * (grp & 1) + ((i16 >> 1) & 1)) ^ (4 * (i16 >> 2));
      wt_off[j] = static_cast<unsigned>((8 * (grp >> 1) + (i16 >> 2)) * 512 + chunk * 16 + (i16 & 1) * 8);
    }
  }
  bf16x8_t fa0[TM], fa1[TM], fb0[TN], fb1[TN];
  auto load_frags = [&](int m, int kk, bf16x8_t(&af)[TM], bf16x8_t(&bfr)[TN]) __attribute__((always_inline)) {
    const int c = (kk * 2 + frag_half) ^ swz;
    const uint4 *sa = smem + ((2 * m) % kDmaSlots) * kSlotChunks;
    const uint4 *sb = smem + ((2 * m + 1) % kDmaSlots) * kSlotChunks;
    {
      const uint4 v = sa[a_base + c];
      af[0] = *reinterpret_cast<const bf16x8_t *>(&v);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if constexpr (WT) {
        typedef short i16x4_t __attribute__((ext_vector_type(4)));
        typedef short i16x8_t __attribute__((ext_vector_type(8)));
        typedef __attribute__((address_space(3))) i16x4_t lds_i16x4_t;
        const __attribute__((address_space(3))) unsigned char *pb =
            (const __attribute__((address_space(3))) unsigned char *)sb + kk * (16 * 512) + wt_off[j];
        const i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t *)pb);
        const i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t *)(pb + 4 * 512));
        bfr[j] = __builtin_bit_cast(bf16x8_t, (i16x8_t)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      } else {
        const uint4 v = sb[b_base + j * 32 * kDmaRC + c];
        bfr[j] = *reinterpret_cast<const bf16x8_t *>(&v);
      }
    }
#pragma unroll
    for (int i = 1; i < TM; ++i) {
      const uint4 v = sa[a_base + i * 32 * kDmaRC + c];
      af[i] = *reinterpret_cast<const bf16x8_t *>(&v);
    }
  };
  auto mma = [&](const bf16x8_t(&af)[TM], const bf16x8_t(&bfr)[TN]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    InterleaveHints<TM * TN, TM + TN, 0, false, 0>::run();
  };

#pragma unroll
  for (int h = 0; h < kDmaSlots; ++h) issue(h);
  // slab 0 is in LDS once only A(1), W(1), A(2) are outstanding
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(kDmaSlots == 5 ? 2 * kAInstr + kWInstr : kAInstr + kWInstr) : "memory");
  load_frags(0, 0, fa0, fb0);

  for (int m = 0; m < KT; ++m) {
    load_frags(m, 1, fa1, fb1);
    mma(fa0, fb0);
    load_frags(m, 2, fa0, fb0);
    mma(fa1, fb1);
    load_frags(m, 3, fa1, fb1);
    mma(fa0, fb0);
    // slab m+1 has landed for everyone (only A(m+2) is outstanding) and nobody reads slab m any more
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kDmaSlots == 5 ? kAInstr : 0) : "memory");
    issue(2 * m + kDmaSlots);                                            // W(m+2) into the slot of A(m)
    issue(2 * m + kDmaSlots + 1);                                        // A(m+3) into the slot of W(m)
    load_frags(m + 1, 0, fa0, fb0);
    mma(fa1, fb1);
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS is reused by the epilogue
  mfma_epilogue<EPI, TM, TN, WTM, WTN>(a, tc, acc, smem, wave, wm, wn, lane);
}

template <int BN, int WM, int WN, int EPI, bool WT = false>
__global__ __launch_bounds__(WM *WN * 64) void gemm_bf16_dma_kernel(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint4 smem[];
  const TileCoord tc = locate_tile(a, 256, BN);
  if (!tc.valid) return;
  dma_tile<BN, WM, WN, EPI, WT>(a, tc, smem);
}

// ------------------------------------------------------------------ bf16 MFMA kernel, short inner dimension
// For K <= 128 (the dt projection: K = dt_rank) there is no K loop to pipeline: a tile of the
// general kernel is one load, a few MFMAs and a long epilogue in sequence, and the epilogue
// (bias + softplus, two transcendentals per element) is bound by plain ALU issue, which needs
// about four wavefronts per SIMD to run at full rate.  Here a workgroup of eight waves keeps its
// 128-column slice of W (all of K) and of the bias in LDS and the waves stream 32-row sub-tiles of
// A past it: A fragments come straight from global memory into registers, each 32x64 half of the
// result goes through bias + softplus into the wave's own LDS patch and leaves as whole 128-byte
// row segments.  No workgroup barrier after the W load; registers are capped at 128 so that two
// workgroups (16 waves) share a CU.
constexpr int kSkBM = 512, kSkBN = 128, kSkWaves = 8;

// PLAIN: no bias, no softplus.  RES: the rows of a.residual (the output's layout and row map) are
// added to the sums before bias and activation: the passes of K > 1 accumulate into the output,
// the last one activates.
template <int KSTEPS, bool PLAIN, bool RES = false>
__global__ __launch_bounds__(kSkWaves * 64) __attribute__((amdgpu_waves_per_eu(4, 8)))
void gemm_bf16_smallk_kernel(const GemmArgs a) {
  constexpr int KC = KSTEPS * 2;                       // 16-byte chunks per row of A / W
  static_assert(KC == 4 || KC == 8 || KC == 16, "K must be 32, 64 or 128");
  constexpr int kSwzShift = KC == 16 ? 0 : (KC == 8 ? 1 : 2);   // 16 consecutive rows -> 16 distinct 16-byte banks
  constexpr int kHalf = kSkBN / 2;                     // columns per pass over the accumulators
  constexpr int kPitch = kHalf * 2 + 16;               // bytes per staged output row; the pad holds its C row index

  extern __shared__ __attribute__((aligned(16))) uint4 smem[];
  const TileCoord tc = locate_tile(a, kSkBM, kSkBN);
  if (!tc.valid) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bf16_t *Ap = static_cast<const bf16_t *>(a.A);
  const bf16_t *Wp = static_cast<const bf16_t *>(a.W) + static_cast<int64_t>(tc.group) * a.N * a.K;
  uint4 *Ws = smem;                                                        // [128][KC], swizzled
  float *bias_s = reinterpret_cast<float *>(smem + kSkBN * KC);            // [128]
  char *stage = reinterpret_cast<char *>(bias_s + kSkBN) + wave * (32 * kPitch);

  for (int q = tid; q < kSkBN * KC; q += kSkWaves * 64) {
    const int r = q / KC, c = q % KC;
    const int n = (tc.n0 + r < a.N) ? tc.n0 + r : a.N - 1;
    const u32x4_t v = *reinterpret_cast<const u32x4_t *>(Wp + static_cast<int64_t>(n) * a.K + c * 8);
    Ws[r * KC + (c ^ ((r >> kSwzShift) & (KC - 1)))] = make_uint4(v.x, v.y, v.z, v.w);
  }
  if (tid < kSkBN) bias_s[tid] = PLAIN ? 0.0f : a.bias[(tc.n0 + tid < a.N) ? tc.n0 + tid : a.N - 1];
  __syncthreads();

  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int swz = (frag_row >> kSwzShift) & (KC - 1);
  const int n_sub = static_cast<int>((tc.row_end - tc.row0 + 31) / 32);
  const int chunk = lane & 7, sub_row = lane >> 3;     // store phase: 8 rows x 128 bytes per instruction

  for (int sub = wave; sub < n_sub; sub += kSkWaves) {
    // A fragment: row frag_row of the sub-tile, 8 elements at K offset 16 kk + 8 frag_half
    int64_t p = tc.row0 + sub * 32 + frag_row;
    if (p >= tc.row_end) p = tc.row0;                 // rows past the tile: computed, never stored
    const int64_t ar = a.a_rows ? a.a_rows[p] : p;
    const int crow = static_cast<int>(a.c_rows ? a.c_rows[p] : p);
    const bf16_t *src = Ap + ar * a.lda + frag_half * 8;
    bf16x8_t af[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) af[kk] = *reinterpret_cast<const bf16x8_t *>(src + kk * 16);
    if (frag_half == 0) *reinterpret_cast<int *>(stage + frag_row * kPitch + kHalf * 2) = crow;

#pragma unroll 1
    for (int h = 0; h < 2; ++h) {
      f32x16_t acc[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const int c = (kk * 2 + frag_half) ^ swz;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint4 w = Ws[(h * kHalf + j * 32 + frag_row) * KC + c];
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t *>(&w), af[kk], acc[j], 0, 0, 0);
        }
      }
      // W is the MFMA's row operand: this lane holds, for A row frag_row, the output columns
      // 32 j + 8 q + 4 frag_half + r of this half in acc[j][4 q + r]
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int lcol = j * 32 + q * 8 + frag_half * 4;
          const float4 b4 = *reinterpret_cast<const float4 *>(bias_s + h * kHalf + lcol);
          float v0 = acc[j][4 * q], v1 = acc[j][4 * q + 1], v2 = acc[j][4 * q + 2], v3 = acc[j][4 * q + 3];
          if constexpr (RES) {
            const int gcol = tc.n0 + h * kHalf + lcol;
            if (gcol < a.N) {
              const u32x2_t o = *reinterpret_cast<const u32x2_t *>(static_cast<const bf16_t *>(a.residual) +
                                                                   static_cast<int64_t>(crow) * a.ldc + gcol);
              v0 += __uint_as_float(o.x << 16); v1 += __uint_as_float(o.x & 0xFFFF0000u);
              v2 += __uint_as_float(o.y << 16); v3 += __uint_as_float(o.y & 0xFFFF0000u);
            }
          }
          uint2 pk;
          if constexpr (PLAIN) {
            pk.x = pack_bf16x2(v0, v1);
            pk.y = pack_bf16x2(v2, v3);
          } else {
            pk.x = pack_bf16x2(softplus_fast(v0 + b4.x), softplus_fast(v1 + b4.y));
            pk.y = pack_bf16x2(softplus_fast(v2 + b4.z), softplus_fast(v3 + b4.w));
          }
          *reinterpret_cast<uint2 *>(stage + frag_row * kPitch + lcol * 2) = pk;
        }
      }
      // the wave's own patch: LDS serves one wave's accesses in program order, no barrier needed
      const int col = tc.n0 + h * kHalf + chunk * 8;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = i * 8 + sub_row;
        const int64_t pr = tc.row0 + sub * 32 + row;
        const uint4 v = *reinterpret_cast<const uint4 *>(stage + row * kPitch + chunk * 16);
        const int cr = *reinterpret_cast<const int *>(stage + row * kPitch + kHalf * 2);
        if (pr < tc.row_end && col < a.N)
          *reinterpret_cast<uint4 *>(static_cast<bf16_t *>(a.C) + static_cast<int64_t>(cr) * a.ldc + col) = v;
      }
    }
  }
}

// ------------------------------------------------------------------ plain FMA kernel
constexpr int kSB = 64, kSK = 16;       // 64x64 tile, K slab 16, 256 threads, 4x4 per thread

template <typename T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const GemmArgs a) {
  __shared__ float As[kSK][kSB + 4];
  __shared__ float Bs[kSK][kSB + 4];
  const TileCoord tc = locate_tile(a, kSB, kSB);
  if (!tc.valid) return;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const T *Ap = static_cast<const T *>(a.A);
  const T *Wp = static_cast<const T *>(a.W) + static_cast<int64_t>(tc.group) * a.N * a.K;
  // staging: thread -> (row = tid / 4, 4 consecutive k = (tid % 4) * 4)
  const int s_r = tid / 4, s_k = (tid % 4) * 4;
  const int64_t pa = tc.row0 + s_r;
  const int64_t a_off = (pa < tc.row_end) ? static_cast<int64_t>(a.a_rows ? a.a_rows[pa] : pa) * a.lda : -1;
  const int64_t b_off = (tc.n0 + s_r < a.N) ? static_cast<int64_t>(tc.n0 + s_r) * a.K : -1;
  float acc[4][4] = {};
  const int k_begin = blockIdx.y * a.k_per_split;
  const int k_stop = (a.K - k_begin < a.k_per_split) ? a.K : k_begin + a.k_per_split;
  for (int k0 = k_begin; k0 < k_stop; k0 += kSK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + s_k + i;
      As[s_k + i][s_r] = (a_off >= 0 && k < k_stop) ? to_f32(Ap[a_off + k]) : 0.0f;
      Bs[s_k + i][s_r] = (b_off >= 0 && k < k_stop) ? to_f32(Wp[b_off + k]) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kSK; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[k][ty * 4 + i]; bv[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t p = tc.row0 + ty * 4 + i;
    const bool row_ok = p < tc.row_end;
    const int64_t crow = row_ok ? (a.c_rows ? a.c_rows[p] : p) : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = tc.n0 + tx * 4 + j;
      if (row_ok && col < a.N) store_out(a, crow, col, acc[i][j]);
    }
  }
}

// A kernel that asks for more than 64 KiB of dynamic LDS needs a function attribute, set once
// per device (the attribute belongs to the device's copy of the code object).  One instance per
// kernel instantiation; safe to call from several host threads.
constexpr int kAttrMaxDevices = 64;
struct LdsAttrOnce {
  std::mutex mu;
  std::atomic<bool> done[kAttrMaxDevices] = {};
  hipError_t ensure(const void *kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kAttrMaxDevices) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
    std::lock_guard<std::mutex> lock(mu);
    if (done[dev].load(std::memory_order_relaxed)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done[dev].store(true, std::memory_order_release);
    return e;
  }
};

int grid_tiles(const GemmArgs &a, int BM, int BN) {
  const int64_t m_tiles = a.offsets ? (a.M / BM + a.n_groups) : ceil_div(a.M, BM);
  const int64_t n_tiles = ceil_div(a.N, BN);
  const int pn = patch_n_for(static_cast<int>(n_tiles)), pm = kPatchTiles / pn;
  const int64_t patches = ceil_div(m_tiles, pm) * ceil_div(n_tiles, pn);
  int64_t g = patches * kPatchTiles;
  g = ceil_div(g, 8) * 8;
  return static_cast<int>(g);
}

template <int BM, int BN, int WM, int WN, int EPI, bool KTAIL>
hipError_t launch_mfma_k(const GemmArgs &a, hipStream_t s) {
  constexpr int kLoopSmem = 2 * (BM + BN) * kRowChunks * 16;
  constexpr int kStageSmem = EPI == kEpiPlainF32 ? 0 : WM * WN * 32 * ((BN / WN) * 2 + 16);
  constexpr int kSmem = kLoopSmem > kStageSmem ? kLoopSmem : kStageSmem;
  static LdsAttrOnce attr;         // per instantiation
  const hipError_t e =
      attr.ensure(reinterpret_cast<const void *>(&gemm_bf16_mfma_kernel<BM, BN, WM, WN, EPI, KTAIL>), kSmem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_bf16_mfma_kernel<BM, BN, WM, WN, EPI, KTAIL>),
                     dim3(grid_tiles(a, BM, BN), a.k_splits), dim3(WM * WN * 64), kSmem, s, a);
  return hipGetLastError();
}
template <int BM, int BN, int WM, int WN, int EPI>
hipError_t launch_mfma(const GemmArgs &a, hipStream_t s) {
  if (a.K % kBK == 0 && a.k_per_split % kBK == 0) return launch_mfma_k<BM, BN, WM, WN, EPI, false>(a, s);
  return launch_mfma_k<BM, BN, WM, WN, EPI, true>(a, s);
}

template <int KSTEPS, bool PLAIN, bool RES>
hipError_t launch_smallk_t(const GemmArgs &a, hipStream_t s) {
  constexpr int kSmem = kSkBN * KSTEPS * 2 * 16 + kSkBN * 4 + kSkWaves * 32 * (kSkBN + 16);
  static LdsAttrOnce attr;
  const hipError_t e = attr.ensure(reinterpret_cast<const void *>(&gemm_bf16_smallk_kernel<KSTEPS, PLAIN, RES>), kSmem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_bf16_smallk_kernel<KSTEPS, PLAIN, RES>), dim3(grid_tiles(a, kSkBM, kSkBN)), dim3(kSkWaves * 64), kSmem, s, a);
  return hipGetLastError();
}
template <int KSTEPS, bool PLAIN>
hipError_t launch_smallk(const GemmArgs &a, hipStream_t s) {
  return a.residual ? launch_smallk_t<KSTEPS, PLAIN, true>(a, s) : launch_smallk_t<KSTEPS, PLAIN, false>(a, s);
}
// whether the streaming small-K kernel takes the call (inner dimension 32, 64 or 128, dense rows of A)
bool smallk_takes(const GemmArgs &a) {
  return kUseSmallK && a.lda >= a.K && a.M < (1ll << 31) && (a.K == 128 || a.K == 64 || a.K == 32) &&
         !a.row_scale && !a.c_is_f32;
}

template <int BN, int WM, int WN, int EPI, bool WT = false>
hipError_t launch_dma(const GemmArgs &a, hipStream_t s) {
  constexpr int kSmem = kDmaSlots * 256 * kDmaRC * 16;     // 160 KiB
  static LdsAttrOnce attr;
  const hipError_t e = attr.ensure(reinterpret_cast<const void *>(&gemm_bf16_dma_kernel<BN, WM, WN, EPI, WT>), kSmem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_bf16_dma_kernel<BN, WM, WN, EPI, WT>), dim3(grid_tiles(a, 256, BN), a.k_splits),
                     dim3(WM * WN * 64), kSmem, s, a);
  return hipGetLastError();
}
// the DMA kernel addresses both operands with unsigned 32-bit byte offsets and walks whole 64-wide slabs
inline bool dma_ok(const GemmArgs &a) {
  return kUseDma && a.K % kDmaBK == 0 && a.k_per_split % kDmaBK == 0 && a.lda >= a.K &&
         a.a_span < (1ll << 31) && static_cast<int64_t>(a.N) * a.K < (1ll << 31);
}

template <int EPI>
hipError_t launch_mfma_tiles(const GemmArgs &a, hipStream_t s) {
  const int64_t rows_per_group = a.M / (a.n_groups > 0 ? a.n_groups : 1);
  // a short inner dimension makes the launch epilogue-bound: smaller tiles put several
  // workgroups on a CU so that loads, MFMAs and stores of different tiles overlap
  if (rows_per_group >= 1024 && a.N >= 256 && a.K > 256) {
    // Between one and one and a half rounds of 256 x 256 tiles on the 256 CUs the second round runs
    // nearly empty: 128 x 128 tiles (several workgroups per CU) finish sooner.  16384 x 1024 x 2048
    // out projection, 288 big tiles: 0.106 -> 0.096 ms.  (From two rounds on the big tile wins again:
    // 544 tiles of the 16384 x 2048 x 4096 out projection 0.310 against 0.324 ms.)
    const int64_t tiles256 = (a.M / 256 + (a.n_groups > 0 ? a.n_groups : 1)) * ceil_div(a.N, 256);
    if (tiles256 > 256 && tiles256 < 384 && a.k_splits == 1) return launch_mfma<128, 128, 2, 2, EPI>(a, s);
    if (dma_ok(a) && a.k_splits == 1) return launch_dma<256, kBigWM, kBigWN, EPI>(a, s);
    return launch_mfma<256, 256, 4, 2, EPI>(a, s);
  }
  if (rows_per_group >= 96) return launch_mfma<128, 128, 2, 2, EPI>(a, s);
  // One row tile per group at most (the recurrent step): every weight tile is read by exactly one
  // workgroup, so there is no L2 sharing for the XCD runs to protect, while a run of logical tiles
  // is one expert's column tiles - with few active experts the runs would put all the work on a
  // few XCDs.  Deal the tiles round-robin instead.
  GemmArgs spread = a;
  spread.no_xcd_remap = 1;
  // a narrow output (the step's out projection: 8 experts x 16 column tiles) leaves half of the CUs
  // without a workgroup while the weights stream past once: halve the column tile.  The same helps while
  // there are only about two workgroups per CU (the step's in projection, 8 x 64 tiles: twice the
  // workgroups keep more of the weight stream in flight; 256 sequences: step 173 -> 161 us)
  const int64_t row_tiles = (a.n_groups > 0 ? a.n_groups : 1) * ceil_div(rows_per_group > 0 ? rows_per_group : 1, 64);
  if (row_tiles * ceil_div(a.N, 128) < kSkinnyColsMaxWgs && a.N % 64 == 0) return launch_mfma<64, 64, 2, 2, EPI>(spread, s);
  return launch_mfma<64, 128, 2, 2, EPI>(spread, s);
}

}  // namespace

// whether a call with a contraction-major weight (GemmArgs::w_kmajor) is taken: the 256 x 256 DMA tile with a
// plain epilogue only; the caller otherwise makes a transposed copy of the weight
bool grouped_gemm_takes_kmajor(const GemmArgs &args) {
  GemmArgs a = args;
  a.k_splits = 1;
  a.k_per_split = static_cast<int>(ceil_div(a.K, 64) * 64);
  const int64_t rows_per_group = a.M / (a.n_groups > 0 ? a.n_groups : 1);
  return grouped_gemm_on_mfma(a) && !a.c_is_f32 && !a.bias && !a.row_scale && !a.residual && !a.swiglu &&
         rows_per_group >= 1024 && a.N % 256 == 0 && a.K > 256 && dma_ok(a);
}

// whether the call takes the MFMA kernels (else the plain FMA kernel, which has no fused SwiGLU)
bool grouped_gemm_on_mfma(const GemmArgs &a) {
  const int out_align = a.c_is_f32 ? 4 : 8;      // elements per output store
  return a.dtype == ROM_DTYPE_BF16 && a.K % 8 == 0 && a.lda % 8 == 0 &&
         a.N % out_align == 0 && a.ldc % out_align == 0 && (reinterpret_cast<uintptr_t>(a.A) % 16 == 0) &&
         (reinterpret_cast<uintptr_t>(a.W) % 16 == 0) &&
         (reinterpret_cast<uintptr_t>(a.C) % 16 == 0) && a.a_span < (1ll << 32) &&
         static_cast<int64_t>(a.N) * a.K < (1ll << 32) &&
         !(a.bias && !a.softplus) && !(a.softplus && !a.bias) &&
         !(a.row_scale && (a.bias || a.c_is_f32)) && !(a.bias && a.c_is_f32) &&
         !(a.residual && a.c_is_f32) && (reinterpret_cast<uintptr_t>(a.residual) % 16 == 0) &&
         !(a.swiglu && (a.bias || a.c_is_f32 || a.residual || a.N % 16 != 0));
}

hipError_t launch_grouped_gemm(const GemmArgs &args, hipStream_t s) {
  if (args.M <= 0) return hipSuccess;
  GemmArgs a = args;
  if (a.k_splits < 1 || !a.c_is_f32 || a.bias || a.row_scale || a.residual) a.k_splits = 1;   // partial sums need a plain fp32 output
  a.k_per_split = static_cast<int>(ceil_div(ceil_div(a.K, a.k_splits), 64) * 64);
  a.k_splits = static_cast<int>(ceil_div(a.K, a.k_per_split));
  const bool mfma_ok = grouped_gemm_on_mfma(a);
  if (a.w_kmajor) {                                           // the caller asks grouped_gemm_takes_kmajor first
    if (!grouped_gemm_takes_kmajor(args)) return hipErrorInvalidValue;
    return launch_dma<256, kBigWM, kBigWN, kEpiPlain, true>(a, s);
  }
  if (a.swiglu && !mfma_ok) return hipErrorInvalidValue;      // the caller asks grouped_gemm_on_mfma first
  if (a.swiglu) return launch_mfma_tiles<kEpiSwiGLU>(a, s);
  if (!mfma_ok) {
    const dim3 grid(grid_tiles(a, kSB, kSB), a.k_splits);
    if (a.dtype == ROM_DTYPE_BF16)
      hipLaunchKernelGGL(gemm_simple_kernel<bf16_t>, grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(gemm_simple_kernel<float>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
  }
  if (a.c_is_f32) {
    if (a.N <= 192) {
      // one column tile: every workgroup re-reads the whole weight slice of its group, so take the
      // tallest row tile (256 rows, 128 on four waves, 64 on two) that still puts a workgroup on
      // a good part of the CUs, counting the inner-dimension slices
      const auto wgs = [&](int rows) { return (a.M / rows + a.n_groups) * a.k_splits; };
      const int tile_rows = wgs(256) >= kSkinnyMinWgs ? 256 : (wgs(128) >= kSkinnyMinWgs ? 128 : 64);
      switch ((a.N + 31) / 32) {
#define ROM_SKINNY(NN)                                                               \
  if (tile_rows == 256 && dma_ok(a)) return launch_dma<NN, 8, 1, kEpiPlainF32>(a, s); \
  return tile_rows == 256 ? launch_mfma<256, NN, 4, 1, kEpiPlainF32>(a, s)           \
       : tile_rows == 128 ? launch_mfma<128, NN, 4, 1, kEpiPlainF32>(a, s)           \
                          : launch_mfma<64, NN, 2, 1, kEpiPlainF32>(a, s)
        case 1: ROM_SKINNY(32);
        case 2: ROM_SKINNY(64);
        case 3: ROM_SKINNY(96);
        case 4: ROM_SKINNY(128);
        case 5: ROM_SKINNY(160);
        default: ROM_SKINNY(192);
#undef ROM_SKINNY
      }
    }
    return launch_mfma_tiles<kEpiPlainF32>(a, s);
  }
  if (a.bias) {
    if (smallk_takes(a)) {
      if (a.K == 128) return launch_smallk<8, false>(a, s);
      if (a.K == 64) return launch_smallk<4, false>(a, s);
      return launch_smallk<2, false>(a, s);
    }
    if (a.residual) return hipErrorInvalidValue;       // bias + activation on top of an accumulated output: small-K kernel only
    return launch_mfma_tiles<kEpiBiasSoftplus>(a, s);
  }
  // short inner dimension, many rows, wide output: the streaming kernel without its activation
  if (smallk_takes(a) && a.M >= 4096 && a.N >= 1024) {
    if (a.K == 128) return launch_smallk<8, true>(a, s);
    if (a.K == 64) return launch_smallk<4, true>(a, s);
    return launch_smallk<2, true>(a, s);
  }
  if (a.residual) return launch_mfma_tiles<kEpiRowScaleResidual>(a, s);
  if (a.row_scale) return launch_mfma_tiles<kEpiRowScale>(a, s);
  return launch_mfma_tiles<kEpiPlain>(a, s);
}

}  // namespace rom
