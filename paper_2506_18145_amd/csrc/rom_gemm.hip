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
// fp32 path (and shapes the MFMA kernel does not take): a plain LDS-tiled FMA kernel.
#include "rom_internal.h"

namespace rom {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

__device__ __forceinline__ float softplus_f32(float v) { return v > 20.0f ? v : log1pf(__expf(v)); }

struct TileCoord {
  int group;
  int64_t row0, row_end;   // sorted positions covered by this tile: [row0, row_end)
  int n0;
  bool valid;
};

// logical tile id -> (global row tile, column tile) in patches of PM x PN tiles, column patches
// first, so that workgroups that run together share A row tiles and W column tiles.
constexpr int kPatchM = 4, kPatchN = 8;

__device__ __forceinline__ TileCoord locate_tile(const GemmArgs &a, int BM, int BN) {
  TileCoord tc;
  tc.valid = false;
  const int n_tiles = (a.N + BN - 1) / BN;
  const int patches_n = (n_tiles + kPatchN - 1) / kPatchN;
  // consecutive workgroup ids go round-robin over the 8 XCDs; hand each XCD a contiguous run
  const int G = gridDim.x;
  int t = blockIdx.x;
  if (G % 8 == 0) t = (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8;
  const int patch = t / (kPatchM * kPatchN), in_patch = t % (kPatchM * kPatchN);
  const int mt = (patch / patches_n) * kPatchM + in_patch % kPatchM;
  const int nt = (patch % patches_n) * kPatchN + in_patch / kPatchM;
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

__device__ __forceinline__ void store_out(const GemmArgs &a, int64_t crow, int col, float v) {
  if (a.bias) v += a.bias[col];
  if (a.softplus) v = softplus_f32(v);
  if (a.row_scale) v *= a.row_scale[crow];
  if (a.c_is_f32 || a.dtype == ROM_DTYPE_F32)
    static_cast<float *>(a.C)[crow * a.ldc + col] = v;
  else
    static_cast<bf16_t *>(a.C)[crow * a.ldc + col] = f32_to_bf16(v);
}

// ------------------------------------------------------------------ bf16 MFMA kernel
constexpr int kBK = 64;                 // K slab, 8 chunks of 8 bf16 (16 bytes) per row
constexpr int kRowChunks = kBK / 8;

template <int BM, int BN, int WM, int WN>
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

  // global source of every 16-byte chunk this thread stages (row base offset or -1)
  int64_t a_src[A_CH], b_src[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int q = tid + i * NT, r = q / kRowChunks;
    const int64_t p = tc.row0 + r;
    a_src[i] = -1;
    if (p < tc.row_end) a_src[i] = static_cast<int64_t>(a.a_rows ? a.a_rows[p] : p) * a.lda;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int q = tid + i * NT, r = q / kRowChunks;
    b_src[i] = (tc.n0 + r < a.N) ? static_cast<int64_t>(tc.n0 + r) * a.K : -1;
  }

  uint4 ra[A_CH], rb[B_CH];
  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = (tid + i * NT) % kRowChunks;
      const int k = k0 + c * 8;
      ra[i] = (a_src[i] >= 0 && k < a.K) ? *reinterpret_cast<const uint4 *>(Ap + a_src[i] + k)
                                         : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int c = (tid + i * NT) % kRowChunks;
      const int k = k0 + c * 8;
      rb[i] = (b_src[i] >= 0 && k < a.K) ? *reinterpret_cast<const uint4 *>(Wp + b_src[i] + k)
                                         : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int q = tid + i * NT, r = q / kRowChunks, c = q % kRowChunks;
      As[buf * BM * kRowChunks + r * kRowChunks + (c ^ (r & 7))] = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int q = tid + i * NT, r = q / kRowChunks, c = q % kRowChunks;
      Bs[buf * BN * kRowChunks + r * kRowChunks + (c ^ (r & 7))] = rb[i];
    }
  };

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int KT = (a.K + kBK - 1) / kBK;
  load_global(0);
  store_lds(0);
  __syncthreads();

  const int frag_row = lane & 31, frag_half = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) load_global((kt + 1) * kBK);
    const uint4 *Ab = As + cur * BM * kRowChunks;
    const uint4 *Bb = Bs + cur * BN * kRowChunks;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      const int c = kk * 2 + frag_half;
      bf16x8_t af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int r = wm * WTM + i * 32 + frag_row;
        const uint4 v = Ab[r * kRowChunks + (c ^ (r & 7))];
        af[i] = *reinterpret_cast<const bf16x8_t *>(&v);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r = wn * WTN + j * 32 + frag_row;
        const uint4 v = Bb[r * kRowChunks + (c ^ (r & 7))];
        bfr[j] = *reinterpret_cast<const bf16x8_t *>(&v);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds(cur ^ 1);
    __syncthreads();
  }

  // epilogue: accumulator element v of a 32x32 tile sits at row 8*(v/4) + 4*(lane/32) + v%4,
  // column lane%32
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t p = tc.row0 + wm * WTM + i * 32 + 8 * (v / 4) + 4 * frag_half + (v % 4);
      if (p >= tc.row_end) continue;
      const int64_t crow = a.c_rows ? a.c_rows[p] : p;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = tc.n0 + wn * WTN + j * 32 + frag_row;
        if (col < a.N) store_out(a, crow, col, acc[i][j][v]);
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
  for (int k0 = 0; k0 < a.K; k0 += kSK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + s_k + i;
      As[s_k + i][s_r] = (a_off >= 0 && k < a.K) ? to_f32(Ap[a_off + k]) : 0.0f;
      Bs[s_k + i][s_r] = (b_off >= 0 && k < a.K) ? to_f32(Wp[b_off + k]) : 0.0f;
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
    if (p >= tc.row_end) continue;
    const int64_t crow = a.c_rows ? a.c_rows[p] : p;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = tc.n0 + tx * 4 + j;
      if (col < a.N) store_out(a, crow, col, acc[i][j]);
    }
  }
}

int grid_tiles(const GemmArgs &a, int BM, int BN) {
  const int64_t m_tiles = a.offsets ? (a.M / BM + a.n_groups) : ceil_div(a.M, BM);
  const int64_t n_tiles = ceil_div(a.N, BN);
  const int64_t patches = ceil_div(m_tiles, kPatchM) * ceil_div(n_tiles, kPatchN);
  int64_t g = patches * kPatchM * kPatchN;
  g = ceil_div(g, 8) * 8;
  return static_cast<int>(g);
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_mfma(const GemmArgs &a, hipStream_t s) {
  constexpr int kSmem = 2 * (BM + BN) * kRowChunks * 16;
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_bf16_mfma_kernel<BM, BN, WM, WN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kSmem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_bf16_mfma_kernel<BM, BN, WM, WN>), dim3(grid_tiles(a, BM, BN)),
                     dim3(WM * WN * 64), kSmem, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_grouped_gemm(const GemmArgs &a, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  const bool mfma_ok = a.dtype == ROM_DTYPE_BF16 && a.K % 8 == 0 && a.lda % 8 == 0 &&
                       (reinterpret_cast<uintptr_t>(a.A) % 16 == 0) &&
                       (reinterpret_cast<uintptr_t>(a.W) % 16 == 0);
  if (!mfma_ok) {
    const dim3 grid(grid_tiles(a, kSB, kSB));
    if (a.dtype == ROM_DTYPE_BF16)
      hipLaunchKernelGGL(gemm_simple_kernel<bf16_t>, grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(gemm_simple_kernel<float>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
  }
  const int64_t rows_per_group = a.M / (a.n_groups > 0 ? a.n_groups : 1);
  if (a.N <= 192) {
    switch ((a.N + 31) / 32) {
      case 1: return launch_mfma<128, 32, 4, 1>(a, s);
      case 2: return launch_mfma<128, 64, 4, 1>(a, s);
      case 3: return launch_mfma<128, 96, 4, 1>(a, s);
      case 4: return launch_mfma<128, 128, 4, 1>(a, s);
      case 5: return launch_mfma<128, 160, 4, 1>(a, s);
      default: return launch_mfma<128, 192, 4, 1>(a, s);
    }
  }
  if (rows_per_group >= 1024) return launch_mfma<256, 256, 2, 2>(a, s);
  if (rows_per_group >= 96) return launch_mfma<128, 128, 2, 2>(a, s);
  return launch_mfma<64, 128, 2, 2>(a, s);
}

}  // namespace rom
