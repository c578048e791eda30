// Backward pass of the RoM layer's sequence part and the small gradient kernels around the
// grouped GEMMs (training, Sec. 5.1): adjoint of the selective scan of Eq. (5) with the gate of
// Eq. (6)/(13) and the softplus of the time step folded in, adjoint of the causal conv + SiLU of
// Eq. (2), gradient of the gate weights of Eq. (9)/(12), and the gather / transpose kernels that
// bring activations into the layout the weight-gradient GEMMs contract over.
// Correct-first: plain ALU kernels, deterministic (fixed summation orders, no atomics).
#include <atomic>
#include <mutex>
#include "rom_internal.h"

namespace rom {

namespace {

template <int CTRL> __device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
// sum of v over the 16 lanes of a DPP row, in every lane (fixed order)
__device__ __forceinline__ float row_sum16(float v) {
#pragma clang fp contract(off)
  v = dpp<0x140>(v) + v;      // row_mirror
  v = dpp<0x141>(v) + v;      // row_half_mirror
  v = dpp<0x1B>(v) + v;       // quad_perm [3,2,1,0]
  v = dpp<0xB1>(v) + v;       // quad_perm [1,0,3,2]
  return v;
}

// Sixteen values per lane, each to be summed over the 16 lanes of a row: a butterfly that halves
// the number of live values at every stage (the lanes with bit 3 / 2 / 1 / 0 of n set keep the upper
// half) leaves the row total of p[n] in lane n - 30 DPP adds and 15 selects instead of 64 adds.
__device__ __forceinline__ float transpose_sum16(const float *p, int n) {
#pragma clang fp contract(off)
  float a[8], b[4], c[2];
  const bool hi8 = (n & 8) != 0, hi4 = (n & 4) != 0, hi2 = (n & 2) != 0, hi1 = (n & 1) != 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float lo = dpp<0x140>(p[j]) + p[j];
    const float hi = dpp<0x140>(p[j + 8]) + p[j + 8];
    a[j] = hi8 ? hi : lo;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = dpp<0x141>(a[j]) + a[j];
    const float hi = dpp<0x141>(a[j + 4]) + a[j + 4];
    b[j] = hi4 ? hi : lo;
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const float lo = dpp<0x1B>(b[j]) + b[j];
    const float hi = dpp<0x1B>(b[j + 2]) + b[j + 2];
    c[j] = hi2 ? hi : lo;
  }
  const float lo = dpp<0xB1>(c[0]) + c[0];
  const float hi = dpp<0xB1>(c[1]) + c[1];
  return hi1 ? hi : lo;
}
// the same for eight values: lane n ends up with the row total of p[n & 7]
__device__ __forceinline__ float transpose_sum8(const float *p, int n) {
#pragma clang fp contract(off)
  float a[8], b[4], c[2];
  const bool hi4 = (n & 4) != 0, hi2 = (n & 2) != 0, hi1 = (n & 1) != 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) a[j] = dpp<0x140>(p[j]) + p[j];       // pairs (i, 15 - i): both halves of the row alike
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = dpp<0x141>(a[j]) + a[j];
    const float hi = dpp<0x141>(a[j + 4]) + a[j + 4];
    b[j] = hi4 ? hi : lo;
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const float lo = dpp<0x1B>(b[j]) + b[j];
    const float hi = dpp<0x1B>(b[j + 2]) + b[j + 2];
    c[j] = hi2 ? hi : lo;
  }
  const float lo = dpp<0xB1>(c[0]) + c[0];
  const float hi = dpp<0xB1>(c[1]) + c[1];
  return hi1 ? hi : lo;
}

__device__ __forceinline__ float sigmoid_f32(float v) { return fast_rcp(1.0f + fast_exp2(-1.44269504088896341f * v)); }

inline dim3 grid1d(int64_t work, int block) { return dim3(static_cast<unsigned>(ceil_div(work, block))); }

// Workgroup barrier for data that travels through LDS only.  __syncthreads() also waits for the
// wavefront's outstanding global stores (its fence covers global memory), which puts a memory round
// trip behind every barrier that follows a store; threads of these kernels never read what another
// thread wrote to global memory, so waiting for the LDS counter is enough.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// ------------------------------------------------------------------ adjoint of the selective scan
// Same lane = (channel, state) layout as the forward kernel.  A 256-thread block is one unit of work:
// 16 channels of one sequence over one chunk of its steps; the grid is (channel blocks, sequences x
// chunks).  A lone wavefront per SIMD issues an instruction every five clocks at best and hides no
// LDS latency, so the launcher cuts the sequences into enough chunks for two blocks per CU.  Per unit:
//   prologue: the state at the chunk's start and the adjoint state flowing in at its end, from the
//           per-chunk carries (decay product P, end state Q from a zero start, start adjoint R from a
//           zero end) that scan_bwd_carry_kernel left, combined in chunk order;
//   pass 1 (forward in time): the state recurrence alone, leaving the state at the start of every
//           16-step group in the checkpoint buffer;
//   pass 2 (backward in time, 64-step tiles of four groups): a group's states are recomputed from
//           its checkpoint into registers, then the adjoint recurrence d_h[t-1] = exp(dt_t a) d_h[t]
//           walks the group backwards.  The group body is unrolled, the loop over groups is not
//           (unrolled over a whole tile the body spills registers).
// Sums over the 16 states of a channel (d_dt, d_u, y) are DPP row sums; sums over the block's 16
// channels (d_B, d_C) go through LDS in channel order; the sum of those over the channel groups of
// the whole layer is left to bwd_reduce_bc_kernel (per-block partial rows in global memory); the
// parameter gradients of a unit go to per-unit partials that scan_bwd_finish_kernel sums in unit order.
constexpr int kBwdTile = 64, kBwdCh = 16, kBwdPitch = kBwdCh + 1, kBwdGroup = 16, kBwdHalf = 8;
constexpr int kGroupsPerTile = kBwdTile / kBwdGroup;

// Scratch of the adjoint scan, all f32.  Units are numbered (sequence * n_chunks + chunk) * n_cb + channel block.
struct ScanBwdLayout {
  int n_cb, n_chunks, n_fine;  // channel blocks; chunks of the main kernel and of the carry kernel per sequence
  int64_t chunk_len, fine_len; // steps per chunk, multiples of the tile; chunk_len is a multiple of fine_len
  int64_t n_units;
  size_t ckpt, carry_p, carry_q, carry_r, part_a, part_d, part_bias, total;   // offsets in floats
};
inline ScanBwdLayout scan_bwd_layout(int64_t B, int64_t L, int d_inner) {
  ScanBwdLayout l;
  l.n_cb = d_inner / kBwdCh;
  const int64_t tiles = ceil_div(L, kBwdTile);
  int64_t nc = ceil_div(512, static_cast<int64_t>(l.n_cb) * B);       // two blocks for each of the 256 CUs
  const int64_t max_nc = tiles / 8 > 0 ? tiles / 8 : 1;                 // a chunk is at least 512 steps
  nc = nc < 1 ? 1 : (nc > max_nc ? max_nc : nc);
  int64_t tiles_per_chunk = ceil_div(tiles, nc);
  // the carry kernel is light and latency-bound: it gets chunks of at most 16 tiles, so that many
  // more of its (small) blocks are resident; the main kernel folds the fine carries
  const int64_t tiles_per_fine = tiles_per_chunk >= 16 ? 16 : tiles_per_chunk;
  tiles_per_chunk = ceil_div(tiles_per_chunk, tiles_per_fine) * tiles_per_fine;
  l.n_chunks = static_cast<int>(ceil_div(tiles, tiles_per_chunk));
  l.n_fine = static_cast<int>(ceil_div(tiles, tiles_per_fine));
  l.chunk_len = tiles_per_chunk * kBwdTile;
  l.fine_len = tiles_per_fine * kBwdTile;
  l.n_units = B * l.n_chunks * l.n_cb;
  const size_t n_fine_units = static_cast<size_t>(B) * l.n_fine * l.n_cb;
  size_t off = 0;
  auto take = [&](size_t n) { size_t o = off; off += (n + 63) / 64 * 64; return o; };
  l.ckpt = take(static_cast<size_t>(l.n_units) * tiles_per_chunk * kGroupsPerTile * 256);
  l.carry_p = take(n_fine_units * 256);
  l.carry_q = take(n_fine_units * 256);
  l.carry_r = take(n_fine_units * 256);
  l.part_a = take(static_cast<size_t>(l.n_units) * 256);
  l.part_d = take(static_cast<size_t>(l.n_units) * kBwdCh);
  l.part_bias = take(static_cast<size_t>(l.n_units) * kBwdCh);
  l.total = off;
  return l;
}

struct BwdSmem {
  // per (step, channel), prepared once when the tile is loaded: dt, u, d y = gate * dg * SiLU(z) and
  // the factor gate * dg * SiLU'(z) of d z
  float dt[kBwdTile][kBwdPitch], u[kBwdTile][kBwdPitch], dy[kBwdTile][kBwdPitch], dzf[kBwdTile][kBwdPitch];
  float bc[kBwdTile][33];                    // B_0..15, C_0..15 of every step
  float o_pre[kBwdTile][kBwdPitch], o_u[kBwdTile][kBwdPitch], o_z[kBwdTile][kBwdPitch];   // outputs of the tile
  float o_bc[kBwdTile][33];                  // this block's share of d_B, d_C of the tile
  // [step in half group][channel][state] terms of d_B, d_C.  The channel sums read both arrays with
  // one instruction (32 lanes per step: 16 states of each); the pad puts part_c half the banks away
  // from part_b, so that the 64 lanes of a wave (two steps) touch 64 different banks.
  float part_b[kBwdHalf][kBwdCh][17];
  float bank_pad[32];
  float part_c[kBwdHalf][kBwdCh][17];
};

// What the carry kernel needs of a tile: a third of the LDS, so that seven of its blocks fit a CU
struct BwdCarrySmem {
  float dt[kBwdTile][kBwdPitch], u[kBwdTile][kBwdPitch], dy[kBwdTile][kBwdPitch];     // (u: dt * u)
  float bc[kBwdTile][33];
};

// A tile travels from global memory to LDS in two steps, so that the loads of the next tile are in
// flight while this one is worked on: bwd_fetch_tile (global -> registers), bwd_park_tile (registers -> LDS).
struct BwdTileRegs {
  float dt[4], u[4], z[4], dg[4], bc[8];
};

typedef unsigned int bwd_u32x2 __attribute__((ext_vector_type(2)));
typedef float bwd_f32x4 __attribute__((ext_vector_type(4)));
// four consecutive elements as floats, one 8-byte (bf16) or 16-byte (f32) load
__device__ __forceinline__ void bwd_load4(const bf16_t *p, float *f) {
  const bwd_u32x2 w = *reinterpret_cast<const bwd_u32x2 *>(p);
  f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xFFFF0000u);
  f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xFFFF0000u);
}
__device__ __forceinline__ void bwd_load4(const float *p, float *f) {
  const bwd_f32x4 w = *reinterpret_cast<const bwd_f32x4 *>(p);
  f[0] = w.x; f[1] = w.y; f[2] = w.z; f[3] = w.w;
}

__device__ __forceinline__ void bwd_store4(bf16_t *p, const float *f) {
  bwd_u32x2 w;
  w.x = pack_bf16x2(f[0], f[1]);
  w.y = pack_bf16x2(f[2], f[3]);
  *reinterpret_cast<bwd_u32x2 *>(p) = w;
}
__device__ __forceinline__ void bwd_store4(float *p, const float *f) {
  bwd_f32x4 w;
  w.x = f[0]; w.y = f[1]; w.z = f[2]; w.w = f[3];
  *reinterpret_cast<bwd_f32x4 *>(p) = w;
}

// thread -> (step row = tid / 4, channels 4 (tid % 4) .. + 3) of every [64][16] tensor and the
// eight B/C values 8 (tid % 4) .. + 7 of that step
template <typename T>
__device__ __forceinline__ void bwd_fetch_tile(BwdTileRegs &r, const T *u_b, const T *dt_b, const T *z_b, int64_t ld_z,
                                               const T *dg_b, const float *bc_b, const float *gate_b, int64_t t0,
                                               int64_t t_end, int d_inner, int tid, bool full) {
  const int row = tid >> 2, c = (tid & 3) * 4;
  const int64_t t = t0 + row;
  if (t < t_end) {
    bwd_load4(dt_b + t * d_inner + c, r.dt);
    bwd_load4(u_b + t * d_inner + c, r.u);
    if (full) {
      bwd_load4(z_b + t * ld_z + c, r.z);
      bwd_load4(dg_b + t * d_inner + c, r.dg);
      const float gw = gate_b ? gate_b[t] : 1.0f;                    // gate weight of Eq. (12)
#pragma unroll
      for (int q = 0; q < 4; ++q) r.dg[q] *= gw;
    }
    bwd_load4(bc_b + t * 32 + (tid & 3) * 8, r.bc);
    bwd_load4(bc_b + t * 32 + (tid & 3) * 8 + 4, r.bc + 4);
  } else {
#pragma unroll
    for (int q = 0; q < 4; ++q) r.dt[q] = r.u[q] = r.z[q] = r.dg[q] = 0.0f;
#pragma unroll
    for (int q = 0; q < 8; ++q) r.bc[q] = 0.0f;
  }
}

// kWithDz: the full set of factors the main kernel's second pass needs; without it (the carry kernel)
// the u slot holds dt * u, the only form that kernel uses u in
template <typename Smem, bool kWithDz>
__device__ __forceinline__ void bwd_park_tile(Smem &sm, const BwdTileRegs &r, int tid, bool full) {
  const int row = tid >> 2, c = (tid & 3) * 4;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    sm.dt[row][c + q] = r.dt[q];
    sm.u[row][c + q] = kWithDz ? r.u[q] : r.dt[q] * r.u[q];
    if (full) {
      const float zs = r.z[q], dgs = r.dg[q];
      const float sig = sigmoid_f32(zs);
      sm.dy[row][c + q] = dgs * zs * sig;                             // g = y * SiLU(z)
      if constexpr (kWithDz) sm.dzf[row][c + q] = dgs * sig * (1.0f + zs * (1.0f - sig));
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) sm.bc[row][(tid & 3) * 8 + q] = r.bc[q];
}

// Carries of one fine chunk (only launched when the sequences are cut into chunks): grid (n_cb, B * n_fine).
//   P = prod_t exp(dt_t a)                       decay over the chunk
//   Q = state at the chunk's end from a zero state at its start
//   R = adjoint state leaving the chunk's start from a zero adjoint state at its end
template <typename T>
__global__ __launch_bounds__(256) void scan_bwd_carry_kernel(
    const T *__restrict__ u, const T *__restrict__ dt, const float *__restrict__ bc, const T *__restrict__ z,
    int64_t ld_z, const T *__restrict__ dg, const float *__restrict__ gate, const float *__restrict__ A_log, int64_t L,
    int d_inner, int n_chunks, int64_t chunk_len, int fine_per_main, int n_main, float *__restrict__ carry_p,
    float *__restrict__ carry_q, float *__restrict__ carry_r) {
  __shared__ BwdCarrySmem sm;
  const int tid = threadIdx.x;
  const int n = tid & 15, cl = tid >> 4;
  const int c0 = blockIdx.x * kBwdCh, ch = c0 + cl;
  const int64_t b = blockIdx.y / n_chunks, k = blockIdx.y % n_chunks;
  const int64_t ts = k * chunk_len, te = ts + chunk_len < L ? ts + chunk_len : L;
  const int64_t n_tiles = (te - ts + kBwdTile - 1) / kBwdTile;
  const float a2 = -__expf(A_log[static_cast<int64_t>(ch) * 16 + n]) * 1.44269504088896341f;
  const T *u_b = u + b * L * d_inner + c0;
  const T *dt_b = dt + b * L * d_inner + c0;
  const T *z_b = z + b * L * ld_z + c0;
  const T *dg_b = dg + b * L * d_inner + c0;
  const float *bc_b = bc + b * L * 32;
  const float *gate_b = gate ? gate + b * L : nullptr;

  // The main kernel folds end states of the fine chunks that lie before its own chunk and start
  // adjoints of those that lie after it: a fine chunk of the last main chunk needs no end state, one of
  // the first main chunk no start adjoint (with two main chunks every block runs one pass, not two).
  // The decay product is needed either way and comes from whichever pass runs.
  const int64_t main_idx = k / fine_per_main;
  const bool need_fwd = main_idx + 1 < n_main, need_bwd = main_idx >= 1;
  BwdTileRegs regs;
  float h = 0.0f, sum_dt = 0.0f;
  if (need_fwd) {
    bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts, te, d_inner, tid, false);
    for (int64_t ti = 0; ti < n_tiles; ++ti) {
      lds_barrier();
      bwd_park_tile<BwdCarrySmem, false>(sm, regs, tid, false);
      lds_barrier();
      if (ti + 1 < n_tiles)
        bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts + (ti + 1) * kBwdTile, te, d_inner, tid, false);
      else
        bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts + ti * kBwdTile, te, d_inner, tid, true);
#pragma unroll 16
      for (int s2 = 0; s2 < kBwdTile; ++s2) {
        const float dts = sm.dt[s2][cl];
        sum_dt += dts;
        h = fmaf(fast_exp2(dts * a2), h, sm.u[s2][cl] * sm.bc[s2][n]);      // (u slot: dt * u)
      }
    }
  } else {
    bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts + (n_tiles - 1) * kBwdTile, te, d_inner, tid, true);
  }
  float gq = 0.0f;
  if (need_bwd || !need_fwd) {                  // (a lone main chunk never launches this kernel; kept total)
    for (int64_t ti = n_tiles - 1; ti >= 0; --ti) {
      lds_barrier();
      bwd_park_tile<BwdCarrySmem, false>(sm, regs, tid, true);
      lds_barrier();
      if (ti > 0)
        bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts + (ti - 1) * kBwdTile, te, d_inner, tid, true);
      if (need_fwd) {
#pragma unroll 16
        for (int s2 = kBwdTile - 1; s2 >= 0; --s2)
          gq = fmaf(sm.bc[s2][16 + n], sm.dy[s2][cl], gq) * fast_exp2(sm.dt[s2][cl] * a2);
      } else {
#pragma unroll 16
        for (int s2 = kBwdTile - 1; s2 >= 0; --s2) {
          const float dts = sm.dt[s2][cl];
          sum_dt += dts;
          gq = fmaf(sm.bc[s2][16 + n], sm.dy[s2][cl], gq) * fast_exp2(dts * a2);
        }
      }
    }
  }
  const int64_t unit = (static_cast<int64_t>(blockIdx.y)) * gridDim.x + blockIdx.x;
  carry_p[unit * 256 + tid] = fast_exp2(sum_dt * a2);
  carry_q[unit * 256 + tid] = h;
  carry_r[unit * 256 + tid] = gq;
}

// grid (n_cb, B * n_chunks).  ckpt: f32 [unit][groups of the chunk][16 channels][16 states].
// d_bc_part: f32 [n_cb][N][32].  Outputs d_pre (w.r.t. the softplus argument), d_u, d_z have type T.
template <typename T>
__global__ __launch_bounds__(256) void scan_bwd_kernel(
    const T *__restrict__ u, const T *__restrict__ dt, const float *__restrict__ bc, const T *__restrict__ z,
    int64_t ld_z, const T *__restrict__ dg, const float *__restrict__ gate, const float *__restrict__ A_log,
    const float *__restrict__ D, int64_t n_seq, int64_t L, int d_inner, int n_chunks, int64_t chunk_len, int n_fine,
    int fine_per_chunk, float *__restrict__ ckpt, const float *__restrict__ carry_p, const float *__restrict__ carry_q,
    const float *__restrict__ carry_r, T *__restrict__ d_pre, T *__restrict__ d_u, T *__restrict__ d_z, int64_t ld_dz,
    float *__restrict__ d_bc_part, float *__restrict__ part_a, float *__restrict__ part_d,
    float *__restrict__ part_bias) {
  __shared__ BwdSmem sm;
  const int tid = threadIdx.x;
  const int n = tid & 15, cl = tid >> 4;
  const int c0 = blockIdx.x * kBwdCh, ch = c0 + cl;
  const int64_t b = blockIdx.y / n_chunks, k = blockIdx.y % n_chunks;
  const int64_t ts = k * chunk_len, te = ts + chunk_len < L ? ts + chunk_len : L;
  const int64_t n_tiles = (te - ts + kBwdTile - 1) / kBwdTile;
  const int64_t unit = static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x;
  const float a_nat = -__expf(A_log[static_cast<int64_t>(ch) * 16 + n]);      // A = -exp(A_log)
  const float a2 = a_nat * 1.44269504088896341f;
  const float d_skip = D[ch];
  float *ck = ckpt + unit * (chunk_len / kBwdGroup) * 256;
  const int64_t n_tok = n_seq * L;
  float acc_a = 0.0f, acc_d = 0.0f, acc_bias = 0.0f;       // d_A (this lane's state); d_D, d_dt_bias (the steps this lane finishes)

  const T *u_b = u + b * L * d_inner + c0;
  const T *dt_b = dt + b * L * d_inner + c0;
  const T *z_b = z + b * L * ld_z + c0;
  const T *dg_b = dg + b * L * d_inner + c0;
  const float *bc_b = bc + b * L * 32;
  const float *gate_b = gate ? gate + b * L : nullptr;

  // ---- prologue: the carries of the fine chunks before (state) and after (adjoint state) this chunk
  float h = 0.0f, dh = 0.0f;
  if (n_chunks > 1) {
    const int64_t unit0 = b * n_fine * gridDim.x + blockIdx.x;        // fine chunk 0 of this sequence and channel block
    const int64_t f0 = k * fine_per_chunk;
    for (int64_t j = 0; j < f0; ++j) {
      const int64_t at = (unit0 + j * gridDim.x) * 256 + tid;
      h = fmaf(carry_p[at], h, carry_q[at]);
    }
    for (int64_t j = n_fine - 1; j >= f0 + fine_per_chunk; --j) {
      const int64_t at = (unit0 + j * gridDim.x) * 256 + tid;
      dh = fmaf(carry_p[at], dh, carry_r[at]);
    }
  }

  // ---- pass 1: the state at the start of every group
  BwdTileRegs regs;
  bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts, te, d_inner, tid, false);
  for (int64_t ti = 0; ti < n_tiles; ++ti) {
    lds_barrier();
    bwd_park_tile<BwdSmem, true>(sm, regs, tid, false);
    lds_barrier();
    if (ti + 1 < n_tiles)      // the next tile; after the last one, the same tile again with the factors pass 2 needs
      bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts + (ti + 1) * kBwdTile, te, d_inner, tid, false);
    else
      bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, ts + ti * kBwdTile, te, d_inner, tid, true);
#pragma unroll 1
    for (int grp = 0; grp < kGroupsPerTile; ++grp) {
      ck[(ti * kGroupsPerTile + grp) * 256 + tid] = h;
#pragma unroll
      for (int j = 0; j < kBwdGroup; ++j) {
        const int s2 = grp * kBwdGroup + j;
        const float dts = sm.dt[s2][cl];
        h = fmaf(fast_exp2(dts * a2), h, dts * sm.u[s2][cl] * sm.bc[s2][n]);
      }
    }
  }

  // ---- pass 2: tiles in reverse, groups in reverse
  for (int64_t ti = n_tiles - 1; ti >= 0; --ti) {
    const int64_t t0 = ts + ti * kBwdTile;
    // the checkpoint of a group is fetched one group ahead of its use
    float ck_next = ck[(ti * kGroupsPerTile + kGroupsPerTile - 1) * 256 + tid];
    lds_barrier();
    bwd_park_tile<BwdSmem, true>(sm, regs, tid, true);
    lds_barrier();
    if (ti > 0)
      bwd_fetch_tile<T>(regs, u_b, dt_b, z_b, ld_z, dg_b, bc_b, gate_b, t0 - kBwdTile, te, d_inner, tid, true);
#pragma unroll 1
    for (int grp = kGroupsPerTile - 1; grp >= 0; --grp) {
      float hs[kBwdGroup + 1], da[kBwdGroup], dts[kBwdGroup], dtu[kBwdGroup], bn[kBwdGroup];
      hs[0] = ck_next;
      if (grp > 0) ck_next = ck[(ti * kGroupsPerTile + grp - 1) * 256 + tid];
#pragma unroll
      for (int j = 0; j < kBwdGroup; ++j) {
        const int s2 = grp * kBwdGroup + j;
        dts[j] = sm.dt[s2][cl];
        dtu[j] = dts[j] * sm.u[s2][cl];
        bn[j] = sm.bc[s2][n];
        da[j] = fast_exp2(dts[j] * a2);
        hs[j + 1] = fmaf(da[j], hs[j], dtu[j] * bn[j]);
      }
#pragma unroll
      for (int half = 1; half >= 0; --half) {
        // the eight steps' LDS operands in one batch: one wait instead of one per step behind the
        // step's own LDS writes
        float us8[kBwdHalf], cn8[kBwdHalf], dy8[kBwdHalf];
#pragma unroll
        for (int jj = 0; jj < kBwdHalf; ++jj) {
          const int s2 = grp * kBwdGroup + half * kBwdHalf + jj;
          us8[jj] = sm.u[s2][cl];
          cn8[jj] = sm.bc[s2][16 + n];
          dy8[jj] = sm.dy[s2][cl];
        }
        // per (step, state) part: the adjoint recurrence and the terms whose sums over the 16 states
        // the step's outputs need: y (p16[jj]), the input term (p16[8 + jj]), d dt (q8[jj])
        float p16[2 * kBwdHalf], q8[kBwdHalf];
#pragma unroll
        for (int jj = kBwdHalf - 1; jj >= 0; --jj) {
          const int j = half * kBwdHalf + jj;
          dh = fmaf(cn8[jj], dy8[jj], dh);                      // y_t = C_t . h_t
          p16[jj] = cn8[jj] * hs[j + 1];
          const float darg = dh * hs[j] * da[j];                // d / d (dt_t * A)
          const float inj = dh * bn[j];                         // input term dt * B * u
          p16[kBwdHalf + jj] = inj;
          q8[jj] = fmaf(darg, a_nat, inj * us8[jj]);
          acc_a = fmaf(darg, dts[j], acc_a);
          sm.part_b[jj][cl][n] = dh * dtu[j];
          sm.part_c[jj][cl][n] = dy8[jj] * hs[j + 1];
          dh *= da[j];
        }
        // sums over the states, transposed: lane n < 8 holds C.h of step n, lane n >= 8 the input-term
        // sum of step n - 8, every lane the d dt sum of step n & 7
        const float yi = transpose_sum16(p16, n);
        const float ddt = transpose_sum8(q8, n);
        // per (step, channel) part, once per step instead of once per lane: lane n works on step n & 7
        {
          const int s2 = grp * kBwdGroup + half * kBwdHalf + (n & 7);
          const float dt_k = sm.dt[s2][cl], u_k = sm.u[s2][cl], dy_k = sm.dy[s2][cl];
          if (n < 8) {
            sm.o_z[s2][cl] = sm.dzf[s2][cl] * fmaf(d_skip, u_k, yi);
            // dt = softplus(pre): d pre = d dt * sigmoid(pre) = d dt * (1 - exp(-dt))
            const float dpre = ddt * (1.0f - fast_exp2(-1.44269504088896341f * dt_k));
            sm.o_pre[s2][cl] = dpre;
            acc_bias += dpre;
            acc_d = fmaf(dy_k, u_k, acc_d);
          } else {
            sm.o_u[s2][cl] = fmaf(yi, dt_k, d_skip * dy_k);
          }
        }
        lds_barrier();
        // d_B, d_C of these eight steps: sum over the block's channels in channel order
        {
          const int jj = tid / 32, c = tid % 32;             // 8 steps x 32 values = 256 threads
          const float(*src)[kBwdCh][17] = c < 16 ? sm.part_b : sm.part_c;
          float tot = 0.0f;
#pragma unroll
          for (int q = 0; q < kBwdCh; ++q) tot += src[jj][q][c & 15];
          sm.o_bc[grp * kBwdGroup + half * kBwdHalf + jj][c] = tot;
        }
        lds_barrier();
      }
    }
    // the tile's outputs, in the fetch's thread map
    {
      const int row = tid >> 2, c = (tid & 3) * 4;
      const int64_t t = t0 + row;
      if (t < te) {
        const int64_t at = (b * L + t) * d_inner + c0 + c;
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = sm.o_pre[row][c + q];
        bwd_store4(d_pre + at, v);
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = sm.o_u[row][c + q];
        bwd_store4(d_u + at, v);
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = sm.o_z[row][c + q];
        bwd_store4(d_z + (b * L + t) * ld_dz + c0 + c, v);
        float *dst = d_bc_part + (static_cast<int64_t>(blockIdx.x) * n_tok + b * L + t) * 32 + (tid & 3) * 8;
        float w[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) w[q] = sm.o_bc[row][(tid & 3) * 8 + q];
        bwd_store4(dst, w);
        bwd_store4(dst + 4, w + 4);
      }
    }
  }
  part_a[unit * 256 + tid] = acc_a * a_nat;                            // d A_log = d A * A
  // (lanes 0..7 of a channel each hold the sums over the steps they worked on, lanes 8..15 zero)
  acc_d = row_sum16(acc_d);
  acc_bias = row_sum16(acc_bias);
  if (n == 0) {
    part_d[unit * kBwdCh + cl] = acc_d;
    part_bias[unit * kBwdCh + cl] = acc_bias;
  }
}

// d_A_log, d_D, d_dt_bias: the units' partials summed in unit order.  One thread per (channel, state).
__global__ __launch_bounds__(256) void scan_bwd_finish_kernel(const float *__restrict__ part_a,
                                                              const float *__restrict__ part_d,
                                                              const float *__restrict__ part_bias, int n_cb,
                                                              int64_t n_rep, float *__restrict__ d_A_log,
                                                              float *__restrict__ d_D, float *__restrict__ d_dt_bias) {
  const int cb = blockIdx.x, tid = threadIdx.x;
  float a = 0.0f;
  for (int64_t r = 0; r < n_rep; ++r) a += part_a[(r * n_cb + cb) * 256 + tid];
  d_A_log[static_cast<int64_t>(cb) * 256 + tid] = a;
  if (tid < 2 * kBwdCh) {
    const float *src = tid < kBwdCh ? part_d : part_bias;
    const int c = tid % kBwdCh;
    float v = 0.0f;
    for (int64_t r = 0; r < n_rep; ++r) v += src[(r * n_cb + cb) * kBwdCh + c];
    (tid < kBwdCh ? d_D : d_dt_bias)[cb * kBwdCh + c] = v;
  }
}

// d_bc[t, :] = sum over the channel-group partials, in group order
__global__ __launch_bounds__(256) void bwd_reduce_bc_kernel(const float *__restrict__ part, int n_parts, int64_t n_tok,
                                                            float *__restrict__ d_bc) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= n_tok * 32) return;
  float tot = 0.0f;
  for (int p = 0; p < n_parts; ++p) tot += part[static_cast<int64_t>(p) * n_tok * 32 + i];
  d_bc[i] = tot;
}

// ------------------------------------------------------------------ gate weights, Eq. (9)/(12)
// d_gate[r] = a[ia(r), :] . b[ib(r), :], one wavefront per row r.
// top-1: d_gate[n] = d_out[n, :] . (W_out[e_n] g[n, :]) = (W_out[e_n]^T d_out[n, :]) . g[n, :] = dg_raw[n, :] . g[n, :]
// (both in token order, no maps).  top-K: r is a slot, a = d_out by the slot's token (r / K), b = the
// expert output W_out[e] g that the forward pass left per sorted position (row inv_perm[r]).
template <typename T>
__global__ __launch_bounds__(256) void gate_bwd_kernel(const T *__restrict__ a, const T *__restrict__ b,
                                                       const int32_t *__restrict__ b_rows, int a_div, int64_t n_rows,
                                                       int n_cols, float *__restrict__ d_gate) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
  if (r >= n_rows) return;
  const int64_t ra = r / a_div, rb = b_rows ? b_rows[r] : r;
  float acc = 0.0f;
  if (n_cols % 8 == 0) {            // rows are 16-byte aligned: eight (bf16) or two times four (fp32) columns per lane and trip
    for (int c = lane * 8; c < n_cols; c += 512) {
      float va[8], vb[8];
      bwd_load4(a + ra * n_cols + c, va);
      bwd_load4(a + ra * n_cols + c + 4, va + 4);
      bwd_load4(b + rb * n_cols + c, vb);
      bwd_load4(b + rb * n_cols + c + 4, vb + 4);
#pragma unroll
      for (int q = 0; q < 8; ++q) acc = fmaf(va[q], vb[q], acc);
    }
  } else {
    for (int c = lane; c < n_cols; c += 64) acc = fmaf(to_f32(a[ra * n_cols + c]), to_f32(b[rb * n_cols + c]), acc);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) d_gate[r] = acc;
}

// d_logits [N, E] from d_gate [N, K]: softmax over all E experts, gate = P of the selected
// (gate_mode 1: divided by their sum).  One thread per token.
__global__ __launch_bounds__(256) void router_bwd_kernel(const float *__restrict__ logits,
                                                         const int32_t *__restrict__ expert_idx,
                                                         const float *__restrict__ d_gate, int64_t n_tok, int n_experts,
                                                         int top_k, int gate_mode, float *__restrict__ d_logits) {
  const int64_t n = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (n >= n_tok) return;
  const float *l = logits + n * n_experts;
  float m = l[0];
  for (int e = 1; e < n_experts; ++e) m = fmaxf(m, l[e]);
  float den = 0.0f;
  for (int e = 0; e < n_experts; ++e) den += __expf(l[e] - m);
  const float inv = 1.0f / den;
  // d P of the selected experts
  float s_sel = 0.0f, dot = 0.0f;
  for (int k = 0; k < top_k; ++k) {
    const float p = __expf(l[expert_idx[n * top_k + k]] - m) * inv;
    s_sel += p;
    dot = fmaf(d_gate[n * top_k + k], p, dot);               // sum_k d_gate_k P_k
  }
  // mode 1: gate_k = P_k / S  ->  dP_k = (d_gate_k - sum_j d_gate_j gate_j) / S ;  mode 0: dP_k = d_gate_k
  // (a single renormalised pick is the constant 1: its gradient is exactly zero, not rounding noise)
  const float shift = gate_mode == 1 ? (top_k == 1 ? d_gate[n] : dot / s_sel) : 0.0f;
  const float scale = gate_mode == 1 ? 1.0f / s_sel : 1.0f;
  float pdp = 0.0f;                                          // sum_e P_e dP_e
  for (int k = 0; k < top_k; ++k) {
    const float p = __expf(l[expert_idx[n * top_k + k]] - m) * inv;
    pdp = fmaf(p, (d_gate[n * top_k + k] - shift) * scale, pdp);
  }
  for (int e = 0; e < n_experts; ++e) {
    float dp = 0.0f;
    for (int k = 0; k < top_k; ++k)
      if (expert_idx[n * top_k + k] == e) dp = (d_gate[n * top_k + k] - shift) * scale;
    d_logits[n * n_experts + e] = __expf(l[e] - m) * inv * (dp - pdp);
  }
}

// partial[chunk][e][d] = sum over the chunk's tokens of d_logits[n, e] * x[n, d]  (d = d_model is the
// bias column: x = 1).  grid (ceil((d_model + 1) / 256), n_chunks); a thread owns one column.
constexpr int kRouterChunk = 128;    // (512: 288 blocks on 256 CUs, one wavefront per SIMD walking 512 dependent rows: 0.24 ms at 16K tokens)
template <typename T, int EMAX>
__global__ __launch_bounds__(256) void router_wgrad_partial_kernel(const float *__restrict__ d_logits,
                                                                   const T *__restrict__ x, int64_t n_tok, int d_model,
                                                                   int n_experts, float *__restrict__ partial) {
  __shared__ float dl[64][EMAX];                    // [token in round][expert]
  const int d = blockIdx.x * 256 + threadIdx.x;
  const int64_t n0 = static_cast<int64_t>(blockIdx.y) * kRouterChunk;
  const int64_t n1 = n0 + kRouterChunk < n_tok ? n0 + kRouterChunk : n_tok;
  float acc[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) acc[e] = 0.0f;
  for (int64_t r0 = n0; r0 < n1; r0 += 64) {
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * EMAX; i += 256) {
      const int64_t n = r0 + i / EMAX;
      const int e = i % EMAX;
      dl[i / EMAX][e] = (n < n1 && e < n_experts) ? d_logits[n * n_experts + e] : 0.0f;
    }
    __syncthreads();
    if (d <= d_model) {
      for (int i = 0; i < 64 && r0 + i < n1; ++i) {
        const float xv = d < d_model ? to_f32(x[(r0 + i) * d_model + d]) : 1.0f;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) acc[e] = fmaf(dl[i][e], xv, acc[e]);
      }
    }
  }
  if (d <= d_model)
#pragma unroll
    for (int e = 0; e < EMAX; ++e)
      if (e < n_experts) partial[(static_cast<int64_t>(blockIdx.y) * n_experts + e) * (d_model + 1) + d] = acc[e];
}

__global__ __launch_bounds__(256) void router_wgrad_finish_kernel(const float *__restrict__ partial, int n_chunks,
                                                                  int d_model, int n_experts,
                                                                  float *__restrict__ d_w_router,
                                                                  float *__restrict__ d_b_router) {
  // (four waves per 64 outputs, as in conv_bwd_finish_kernel)
  __shared__ float sums[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + lane;
  const bool live = i < n_experts * (d_model + 1);
  float acc = 0.0f;
  if (live)
    for (int c = q; c < n_chunks; c += 4) acc += partial[static_cast<int64_t>(c) * n_experts * (d_model + 1) + i];
  sums[q][lane] = acc;
  __syncthreads();
  if (q != 0 || !live) return;
  const float tot = (sums[0][lane] + sums[1][lane]) + (sums[2][lane] + sums[3][lane]);
  const int e = i / (d_model + 1), d = i % (d_model + 1);
  if (d < d_model) d_w_router[e * d_model + d] = tot;
  else if (d_b_router) d_b_router[e] = tot;
}

// d_x[n, d] = dx_in[n, d] + sum_e d_logits[n, e] * W_r[e, d]; a thread owns four consecutive columns
template <typename T>
__global__ __launch_bounds__(256) void dx_finish_kernel(const T *__restrict__ dx_in, const float *__restrict__ d_logits,
                                                        const T *__restrict__ w_router, int64_t n_tok, int d_model,
                                                        int n_experts, T *__restrict__ d_x) {
  // eight consecutive columns of one token per thread (d_model is a multiple of 8)
  const int64_t i = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) * 8;
  if (i >= n_tok * d_model) return;
  const int64_t n = i / d_model;
  const int d = static_cast<int>(i % d_model);
  float v[8], wv[8];
  bwd_load4(dx_in + i, v);
  bwd_load4(dx_in + i + 4, v + 4);
  for (int e = 0; e < n_experts; ++e) {
    const float dl = d_logits[n * n_experts + e];
    bwd_load4(w_router + static_cast<int64_t>(e) * d_model + d, wv);
    bwd_load4(w_router + static_cast<int64_t>(e) * d_model + d + 4, wv + 4);
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = fmaf(dl, wv[q], v[q]);
  }
  bwd_store4(d_x + i, v);
  bwd_store4(d_x + i + 4, v + 4);
}

// ------------------------------------------------------------------ adjoint of conv + SiLU, Eq. (2)
// A thread owns one channel and a run of kConvBwdRun steps of one sequence.  c_t = b + sum_j w_j x_{t-3+j}
// is recomputed, d_c_t = (du_a + du_b)_t * SiLU'(c_t); d_x_{t} = sum_j w_j d_c_{t+3-j} needs d_c of three
// later steps (zero past the sequence end), so the thread runs three steps into the next run.
// Per-run partial sums of d_w[i, j] = sum_t d_c_t x_{t-3+j} and d_b = sum_t d_c_t go to
// partial[run][5][channel] and are added in run order by conv_bwd_finish_kernel.
constexpr int kConvBwdRun = 128;
constexpr int kConvBwdAhead = 8;     // steps whose rows are requested together
// two consecutive channels of a row (4- or 8-byte accesses; the launcher checks evenness and alignment)
__device__ __forceinline__ void conv_ld2(const bf16_t *p, float (&f)[2]) {
  const unsigned u = *reinterpret_cast<const unsigned *>(p);
  f[0] = bf16_to_f32(static_cast<bf16_t>(u & 0xffffu));
  f[1] = bf16_to_f32(static_cast<bf16_t>(u >> 16));
}
__device__ __forceinline__ void conv_ld2(const float *p, float (&f)[2]) {
  const float2 v = *reinterpret_cast<const float2 *>(p);
  f[0] = v.x; f[1] = v.y;
}
__device__ __forceinline__ void conv_st2(bf16_t *p, const float (&f)[2]) {
  *reinterpret_cast<unsigned *>(p) = static_cast<unsigned>(f32_to_bf16(f[0])) | (static_cast<unsigned>(f32_to_bf16(f[1])) << 16);
}
__device__ __forceinline__ void conv_st2(float *p, const float (&f)[2]) { *reinterpret_cast<float2 *>(p) = make_float2(f[0], f[1]); }

// V = 2: a thread owns two neighbouring channels (half the memory instructions, twice their width)
template <typename T, int V>
__global__ __launch_bounds__(256) void conv_bwd_kernel(const T *__restrict__ xz, int64_t ld_xz,
                                                       const float *__restrict__ conv_w,
                                                       const float *__restrict__ conv_b, const T *__restrict__ du_a,
                                                       const T *__restrict__ du_b, int64_t L, int d_inner,
                                                       T *__restrict__ d_xpre, int64_t ld_dx,
                                                       float *__restrict__ partial) {
  static_assert(V == 1 || V == 2, "one or two channels per thread");
  const int ch = (blockIdx.x * blockDim.x + threadIdx.x) * V;
  if (ch >= d_inner) return;
  const int64_t b = blockIdx.z, run = blockIdx.y;
  const int64_t t0 = run * kConvBwdRun;
  const int64_t t1 = t0 + kConvBwdRun < L ? t0 + kConvBwdRun : L;
  float w[V][4], bias[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    const float4 wv = *reinterpret_cast<const float4 *>(conv_w + static_cast<int64_t>(ch + v) * 4);
    w[v][0] = wv.x; w[v][1] = wv.y; w[v][2] = wv.z; w[v][3] = wv.w;
    bias[v] = conv_b ? conv_b[ch + v] : 0.0f;
  }
  const T *xr = xz + b * L * ld_xz + ch;
  const int64_t tok0 = b * L;
  auto load = [&](const T *p, float (&f)[V]) __attribute__((always_inline)) {
    if constexpr (V == 2) conv_ld2(p, f); else f[0] = to_f32(*p);
  };
  // the rows a step needs from memory: x_{t+3} and the two d u rows of step t+3 (zeros outside the sequence)
  auto fetch = [&](int64_t t, float (&x)[V], float (&ua)[V], float (&ub)[V]) __attribute__((always_inline)) {
    if (t >= 0 && t < L) {
      load(xr + t * ld_xz, x);
      load(du_a + (tok0 + t) * d_inner + ch, ua);
      load(du_b + (tok0 + t) * d_inner + ch, ub);
    } else {
#pragma unroll
      for (int v = 0; v < V; ++v) x[v] = ua[v] = ub[v] = 0.0f;
    }
  };
  // d loss / d c_t from the four inputs x_{t-3..t} of c_t and d u_t (d u = 0 outside the sequence gives 0)
  auto dc_of = [&](const float (&x0)[V], const float (&x1)[V], const float (&x2)[V], const float (&x3)[V],
                   const float (&ua)[V], const float (&ub)[V], float (&d)[V]) __attribute__((always_inline)) {
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const float c = bias[v] + w[v][0] * x0[v] + w[v][1] * x1[v] + w[v][2] * x2[v] + w[v][3] * x3[v];
      const float sig = sigmoid_f32(c);
      d[v] = (ua[v] + ub[v]) * sig * (1.0f + c * (1.0f - sig));
    }
  };
  float acc_w[V][4], acc_b[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    acc_b[v] = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) acc_w[v][j] = 0.0f;
  }
  // the inputs x_{t-3} .. x_{t+3} and d_c of t .. t+3 slide along the run: one new x row, one new pair
  // of d u rows and one output row per step.  The rows of kConvBwdAhead steps are requested together
  // before any of them is used: a thread's loop is otherwise one memory round trip per step.
  float xs[7][V], d0[V], d1[V], d2[V], d3[V];
  {
    float ua[3][V], ub[3][V], unused_a[V], unused_b[V];
#pragma unroll
    for (int k = 0; k < 3; ++k) fetch(t0 - 3 + k, xs[k], unused_a, unused_b);
#pragma unroll
    for (int k = 0; k < 3; ++k) fetch(t0 + k, xs[3 + k], ua[k], ub[k]);
    dc_of(xs[0], xs[1], xs[2], xs[3], ua[0], ub[0], d0);
    dc_of(xs[1], xs[2], xs[3], xs[4], ua[1], ub[1], d1);
    dc_of(xs[2], xs[3], xs[4], xs[5], ua[2], ub[2], d2);
  }
  for (int64_t tb = t0; tb < t1; tb += kConvBwdAhead) {
    float xn[kConvBwdAhead][V], una[kConvBwdAhead][V], unb[kConvBwdAhead][V];
#pragma unroll
    for (int k = 0; k < kConvBwdAhead; ++k) fetch(tb + 3 + k, xn[k], una[k], unb[k]);
#pragma unroll
    for (int k = 0; k < kConvBwdAhead; ++k) {
      const int64_t t = tb + k;
      if (t < t1) {
#pragma unroll
        for (int v = 0; v < V; ++v) xs[6][v] = xn[k][v];
        dc_of(xs[3], xs[4], xs[5], xs[6], una[k], unb[k], d3);
        // x_t feeds c_t (tap 3), c_{t+1} (tap 2), c_{t+2} (tap 1), c_{t+3} (tap 0)
        float o[V];
#pragma unroll
        for (int v = 0; v < V; ++v) {
          o[v] = w[v][3] * d0[v] + w[v][2] * d1[v] + w[v][1] * d2[v] + w[v][0] * d3[v];
          acc_b[v] += d0[v];
          acc_w[v][0] = fmaf(d0[v], xs[0][v], acc_w[v][0]);
          acc_w[v][1] = fmaf(d0[v], xs[1][v], acc_w[v][1]);
          acc_w[v][2] = fmaf(d0[v], xs[2][v], acc_w[v][2]);
          acc_w[v][3] = fmaf(d0[v], xs[3][v], acc_w[v][3]);
          d0[v] = d1[v]; d1[v] = d2[v]; d2[v] = d3[v];
        }
        if constexpr (V == 2) conv_st2(d_xpre + (tok0 + t) * ld_dx + ch, o);
        else d_xpre[(tok0 + t) * ld_dx + ch] = from_f32<T>(o[0]);
#pragma unroll
        for (int j = 0; j < 6; ++j)
#pragma unroll
          for (int v = 0; v < V; ++v) xs[j][v] = xs[j + 1][v];
      }
    }
  }
  const int64_t n_runs = gridDim.y;
#pragma unroll
  for (int v = 0; v < V; ++v) {
    float *dst = partial + ((b * n_runs + run) * 5) * d_inner + ch + v;
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[j * d_inner] = acc_w[v][j];
    dst[4 * d_inner] = acc_b[v];
  }
}

__global__ __launch_bounds__(256) void conv_bwd_finish_kernel(const float *__restrict__ partial, int64_t n_parts,
                                                              int d_inner, float *__restrict__ d_conv_w,
                                                              float *__restrict__ d_conv_b) {
  // a block owns 64 outputs; its four waves each add every fourth partial in order, then the four sums
  // are added in wave order (one thread walking all partials is a chain of dependent memory round trips)
  __shared__ float sums[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + lane;
  const bool live = i < 5 * d_inner;
  const int j = live ? i / d_inner : 0, ch = live ? i % d_inner : 0;
  float acc = 0.0f;
  if (live)
    for (int64_t p = q; p < n_parts; p += 4) acc += partial[(p * 5 + j) * d_inner + ch];
  sums[q][lane] = acc;
  __syncthreads();
  if (q != 0 || !live) return;
  const float tot = (sums[0][lane] + sums[1][lane]) + (sums[2][lane] + sums[3][lane]);
  if (j < 4) d_conv_w[ch * 4 + j] = tot;
  else if (d_conv_b) d_conv_b[ch] = tot;
}

// ------------------------------------------------------------------ weight transposes for the input gradients
// dst[e][c][r] = src[e][r][c]: the grouped GEMM contracts over the contiguous index of both operands,
// and d_inp = d_out W contracts over W's row index.  64 x 64 tiles through LDS; when rows and cols
// are multiples of 4, both the global reads and the global writes move four consecutive elements.
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ src, T *__restrict__ dst, int rows,
                                                        int cols, int vec) {
  __shared__ float tile[64][65];
  const int64_t base = static_cast<int64_t>(blockIdx.z) * rows * cols;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  if (vec) {
    // thread -> (row i = tid / 16 + 16 q, columns 4 (tid % 16) .. + 3)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = (threadIdx.x >> 4) + 16 * q, j = (threadIdx.x & 15) * 4;
      float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (r0 + i < rows && c0 + j < cols) bwd_load4(src + base + static_cast<int64_t>(r0 + i) * cols + c0 + j, v);
#pragma unroll
      for (int e = 0; e < 4; ++e) tile[i][j + e] = v[e];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = (threadIdx.x >> 4) + 16 * q, j = (threadIdx.x & 15) * 4;     // output row c0 + i, columns r0 + j ..
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = tile[j + e][i];
      if (c0 + i < cols && r0 + j < rows) bwd_store4(dst + base + static_cast<int64_t>(c0 + i) * rows + r0 + j, v);
    }
  } else {
    for (int k = threadIdx.x; k < 64 * 64; k += 256) {
      const int i = k / 64, j = k % 64;
      if (r0 + i < rows && c0 + j < cols) tile[i][j] = to_f32(src[base + static_cast<int64_t>(r0 + i) * cols + c0 + j]);
    }
    __syncthreads();
    for (int k = threadIdx.x; k < 64 * 64; k += 256) {
      const int i = k / 64, j = k % 64;
      if (c0 + i < cols && r0 + j < rows) dst[base + static_cast<int64_t>(c0 + i) * rows + r0 + j] = from_f32<T>(tile[j][i]);
    }
  }
}

// d_xdbl [N, R + 32] (type T) = [ d_dt_low (f32 [N, R]) | d_bc (f32 [N, 32]) ]
template <typename T>
__global__ __launch_bounds__(256) void pack_dxdbl_kernel(const float *__restrict__ d_dt_low,
                                                         const float *__restrict__ d_bc, int64_t n_tok, int dt_rank,
                                                         T *__restrict__ d_xdbl) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  const int cols = dt_rank + 32;
  if (i >= n_tok * cols) return;
  const int64_t n = i / cols;
  const int c = static_cast<int>(i % cols);
  d_xdbl[i] = from_f32<T>(c < dt_rank ? d_dt_low[n * dt_rank + c] : d_bc[n * 32 + (c - dt_rank)]);
}

// ------------------------------------------------------------------ weight gradients
//   d_W[e][m][n] = sum over the sorted positions p of expert e of s_p * A[a_row(p)][m] * B[b_row(p)][n]
// (A = the gradient of the projection's output, B = its input, s = gate weight for the out projection).
// Both operands are stored position-major, so the contraction index is the slow one: a 128 x 128
// output tile walks the expert's positions in slabs of 32, each thread fetches 16-byte pieces
// (eight consecutive m or n of one position) and scatters them transposed into LDS, from where the
// MFMA fragments (eight consecutive positions of one m / n) are read.  fp32 result, fixed order.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kWgTile = 128, kWgSlab = 64, kWgPitch = kWgSlab + 8;     // halfs per LDS row (144 bytes: 16-byte aligned rows)

// eight 16-byte pieces (eight consecutive columns of eight consecutive positions) -> for each of the
// eight columns the eight positions as one 16-byte LDS row segment: word a of column m's segment
// holds positions 2a, 2a+1, which v_perm_b32 picks out of word m/2 of the two position rows
__device__ __forceinline__ void wgrad_park8x8(const u32x4_t (&v)[8], bf16_t (*dst)[kWgPitch], int col0, int pos0) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {          // word w of a piece = columns 2w, 2w+1
    u32x4_t lo, hi;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const unsigned int p0 = v[2 * a][w], p1 = v[2 * a + 1][w];
      lo[a] = __builtin_amdgcn_perm(p1, p0, 0x05040100u);      // (p0.lo16, p1.lo16)
      hi[a] = __builtin_amdgcn_perm(p1, p0, 0x07060302u);      // (p0.hi16, p1.hi16)
    }
    *reinterpret_cast<u32x4_t *>(&dst[col0 + 2 * w][pos0]) = lo;
    *reinterpret_cast<u32x4_t *>(&dst[col0 + 2 * w + 1][pos0]) = hi;
  }
}

__global__ __launch_bounds__(256) void wgrad_bf16_kernel(const bf16_t *__restrict__ A, int64_t lda, int M,
                                                         const bf16_t *__restrict__ Bm, int64_t ldb, int N,
                                                         const int32_t *__restrict__ rows_a,
                                                         const int32_t *__restrict__ rows_b,
                                                         const int32_t *__restrict__ offsets, int64_t n_pos,
                                                         float *__restrict__ C) {
  __shared__ __attribute__((aligned(16))) bf16_t As[kWgTile][kWgPitch];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[kWgTile][kWgPitch];
  const int e = blockIdx.z;
  const int64_t p_lo = offsets ? offsets[e] : 0, p_hi = offsets ? offsets[e + 1] : n_pos;
  const int m0 = blockIdx.y * kWgTile, n0 = blockIdx.x * kWgTile;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;                       // 2 x 2 waves, 64 x 64 each
  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
  const int frag_row = lane & 31, frag_half = lane >> 5;
  // staging: a slab is 64 positions; threads 0..127 bring the A operand, 128..255 the B operand, each an
  // 8-position x 8-column block: (position group pg = 0..7, column piece = 0..15)
  const bool is_a = __builtin_amdgcn_readfirstlane(tid < 128 ? 1 : 0) != 0;      // wave-uniform
  const int t2 = tid & 127, pg = t2 & 7, piece = t2 >> 3;       // 16 consecutive lanes park into 64 distinct banks
  const bf16_t *src = is_a ? A : Bm;
  const int32_t *rows = is_a ? rows_a : rows_b;      // position -> row of this operand (NULL: the position itself)
  const int64_t ld = is_a ? lda : ldb;
  const int col = (is_a ? m0 : n0) + piece * 8;
  const bool col_ok = col < (is_a ? M : N);
  bf16_t(*dst)[kWgPitch] = is_a ? As : Bs;
  for (int64_t p0 = p_lo; p0 < p_hi; p0 += kWgSlab) {
    // (branch-free, indices first: see the 256 x 256 kernel)
    u32x4_t v[8];
    int64_t r[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t p = p0 + pg * 8 + i;
      r[i] = p < p_hi ? p : p_hi - 1;
    }
    if (rows) {
#pragma unroll
      for (int i = 0; i < 8; ++i) r[i] = rows[r[i]];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const u32x4_t *>(src + r[i] * ld + (col_ok ? col : 0));
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (p0 + pg * 8 + i >= p_hi || !col_ok) v[i] = u32x4_t{0u, 0u, 0u, 0u};
    __syncthreads();                       // the slab before this one has been multiplied
    wgrad_park8x8(v, dst, piece * 8, pg * 8);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kWgSlab / 16; ++kk) {
      bf16x8_t fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8_t *>(&As[wm * 64 + i * 32 + frag_row][kk * 16 + frag_half * 8]);
        fb[i] = *reinterpret_cast<const bf16x8_t *>(&Bs[wn * 64 + i * 32 + frag_row][kk * 16 + frag_half * 8]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
  }
  // the B fragment is the MFMA's row operand: this lane holds, for output row m = frag_row, the
  // columns 8 q + 4 frag_half + r of each 32-wide tile in accumulator element 4 q + r
  float *Ce = C + static_cast<int64_t>(e) * M * N;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = m0 + wm * 64 + i * 32 + frag_row;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int cc = n0 + wn * 64 + j * 32 + q * 8 + frag_half * 4;
        if (m < M && cc + 3 < N)
          *reinterpret_cast<float4 *>(Ce + static_cast<int64_t>(m) * N + cc) =
              make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        else
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (m < M && cc + r < N) Ce[static_cast<int64_t>(m) * N + cc + r] = acc[i][j][4 * q + r];
      }
  }
}

// The same contraction for outputs of at least 256 x 256 per expert (the in and out projections):
// a 256 x 256 tile on eight waves (4 x 2, 64 x 128 each: 2 x 4 MFMA accumulators, six fragment
// reads per eight MFMAs instead of four per four, because the fragment reads out of LDS are what
// bounds the small tile), two LDS buffers so that the next slab is fetched into registers while
// this one is multiplied and parked into the other buffer afterwards: one barrier per slab.
constexpr int kWgBig = 256;
constexpr int kWgBigSmem = 2 * 2 * kWgBig * kWgPitch * 2;      // two buffers x (A, B) x 256 rows x 144 bytes
__global__ __launch_bounds__(512) void wgrad_bf16_big_kernel(const bf16_t *__restrict__ A, int64_t lda, int M,
                                                             const bf16_t *__restrict__ Bm, int64_t ldb, int N,
                                                             const int32_t *__restrict__ rows_a,
                                                             const int32_t *__restrict__ rows_b,
                                                             const int32_t *__restrict__ offsets, int64_t n_pos,
                                                             int n_groups, float *__restrict__ C) {
  extern __shared__ __attribute__((aligned(16))) unsigned char wg_smem[];
  typedef bf16_t (*Tile)[kWgPitch];
  // Workgroup ids go round the eight XCDs; logical tiles (column tile fastest, then row tile, then
  // expert) are dealt so that an XCD works on a contiguous run of them: the 32 tiles its CUs hold at
  // a time share their A and B column blocks in that XCD's L2 instead of each fetching its own.
  const int tn = (N + kWgBig - 1) / kWgBig, tm = (M + kWgBig - 1) / kWgBig;
  const int per_xcd = gridDim.x / 8;                             // the grid is padded to a multiple of 8
  const int t = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (t >= tn * tm * n_groups) return;
  const int e = t / (tn * tm);
  const int64_t p_lo = offsets ? offsets[e] : 0, p_hi = offsets ? offsets[e + 1] : n_pos;
  const int m0 = ((t / tn) % tm) * kWgBig, n0 = (t % tn) * kWgBig;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 3, wn = wave >> 2;                       // 4 x 2 waves, 64 x 128 each
  f32x16_t acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
  const int frag_row = lane & 31, frag_half = lane >> 5;
  // staging: threads 0..255 bring the A operand, 256..511 the B operand, each an 8-position x 8-column
  // block of the slab's 64 positions x 256 columns: (position group pg = 0..7, column piece = 0..31)
  // (wave-uniform, and said so: with a per-lane operand choice the row map's NULL test is a divergent
  // branch around every index load, each followed by its own wait)
  const bool is_a = __builtin_amdgcn_readfirstlane(tid < 256 ? 1 : 0) != 0;
  const int t2 = tid & 255, pg = t2 & 7, piece = t2 >> 3;
  const bf16_t *src = is_a ? A : Bm;
  const int32_t *rows = is_a ? rows_a : rows_b;
  const int64_t ld = is_a ? lda : ldb;
  const int col = (is_a ? m0 : n0) + piece * 8;
  const bool col_ok = col < (is_a ? M : N);
  auto tile_of = [&](int buf, bool a_side) {
    return reinterpret_cast<Tile>(wg_smem + (static_cast<size_t>(buf) * 2 + (a_side ? 0 : 1)) * kWgBig * kWgPitch * 2);
  };
  u32x4_t v[8];
  // Branch-free: the eight row indices first, then the eight rows (positions past the group's end
  // re-read its last row, columns past the matrix re-read column 0, and are zeroed afterwards) - with
  // a branch per row the compiler waits for each index and each row in turn, sixteen dependent
  // memory round trips per slab.
  const int col_c = col_ok ? col : 0;
  // (requesting the row indices a further slab ahead, so that their round trip is hidden too,
  // measured slower: 0.78 -> 0.94 ms)
  auto fetch = [&](int64_t p0) __attribute__((always_inline)) {
    int64_t r[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t p = p0 + pg * 8 + i;
      r[i] = p < p_hi ? p : p_hi - 1;
    }
    if (rows) {
#pragma unroll
      for (int i = 0; i < 8; ++i) r[i] = rows[r[i]];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const u32x4_t *>(src + r[i] * ld + col_c);
  };
  // zeroes what fetch(p0) read past the group's end or past the matrix; called where the rows are
  // parked, not where they are requested, so that the wait for them comes after the MFMAs
  auto mask = [&](int64_t p0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (p0 + pg * 8 + i >= p_hi || !col_ok) v[i] = u32x4_t{0u, 0u, 0u, 0u};
  };
  if (p_lo < p_hi) {
    fetch(p_lo);
    mask(p_lo);
    wgrad_park8x8(v, tile_of(0, is_a), piece * 8, pg * 8);
  }
  __syncthreads();
  int buf = 0;
  for (int64_t p0 = p_lo; p0 < p_hi; p0 += kWgSlab, buf ^= 1) {
    const bool has_next = p0 + kWgSlab < p_hi;
    if (has_next) fetch(p0 + kWgSlab);                 // in flight while this slab is multiplied
    const Tile As = tile_of(buf, true), Bs = tile_of(buf, false);
#pragma unroll
    for (int kk = 0; kk < kWgSlab / 16; ++kk) {
      bf16x8_t fa[2], fb[4];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const bf16x8_t *>(&As[wm * 64 + i * 32 + frag_row][kk * 16 + frag_half * 8]);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        fb[j] = *reinterpret_cast<const bf16x8_t *>(&Bs[wn * 128 + j * 32 + frag_row][kk * 16 + frag_half * 8]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    // the other buffer was last read in the iteration before this one, which every wave has left
    if (has_next) {
      mask(p0 + kWgSlab);
      wgrad_park8x8(v, tile_of(buf ^ 1, is_a), piece * 8, pg * 8);
    }
    __syncthreads();
  }
  // the B fragment is the MFMA's row operand: this lane holds, for output row m = frag_row, the
  // columns 8 q + 4 frag_half + r of each 32-wide tile in accumulator element 4 q + r
  float *Ce = C + static_cast<int64_t>(e) * M * N;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = m0 + wm * 64 + i * 32 + frag_row;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int cc = n0 + wn * 128 + j * 32 + q * 8 + frag_half * 4;
        if (m < M && cc + 3 < N)
          *reinterpret_cast<float4 *>(Ce + static_cast<int64_t>(m) * N + cc) =
              make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        else
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (m < M && cc + r < N) Ce[static_cast<int64_t>(m) * N + cc + r] = acc[i][j][4 * q + r];
      }
  }
}

// The 256 x 256 contraction once more, for outputs that are whole multiples of the tile: the operand
// rows go from global memory straight into LDS exactly as they lie in memory - position-major, 256
// columns = 512 bytes per position (global_load_lds_dwordx4: lane l of a wave deposits its 16 bytes
// at M0 + 16 l) - and the MFMA fragments, which want eight consecutive POSITIONS of one column per
// lane, are read with the transposing LDS read (ds_read_b64_tr_b16: the 16 lanes of a group name four
// rows of 16 columns, lane i receives column i of the four rows).  No register transposes, no LDS
// writes and no load -> park dependency are left in the loop.  A slab is 64 positions; LDS is a
// ring of five half-slab slots of 32 KiB (A rows of slab m, B rows of slab m, A rows of slab m + 1, ...)
// filled in ring order, four DMA instructions per wave and half slab, so that "vmcnt(4)" means
// "everything but the newest half slab I asked for has landed".  The 16-byte chunk c of row r lies
// at position c ^ 4 (r & 3) of its row (the swizzle is applied where the global address is formed):
// the four rows x 64 bytes that 32 lanes read at a time then cover all 64 banks once.
// Row indices (positions -> rows of the operand) are uniform per wave and instruction half: they
// are read through the scalar cache one slab before the DMA that uses them is issued.
// Positions past the group's end are fetched from whatever valid row follows and zeroed in LDS
// before the last slab is multiplied.
constexpr bool kUseWgradDma = true;
constexpr int kWdSlots = 5;
constexpr int kWdSlotBytes = kWgSlab * kWgBig * 2;         // 64 positions x 256 columns x 2 bytes
constexpr int kWdSmem = kWdSlots * kWdSlotBytes;           // 160 KiB
constexpr int kWdInstr = 4;                                // DMA instructions per wave and half slab (2 rows each)
typedef short i16x4_t __attribute__((ext_vector_type(4)));
typedef short i16x8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;

__device__ __forceinline__ void wd_dma_16(unsigned lds_addr, unsigned voff, const void *base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n"
               :: "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
}

// eight consecutive positions of this lane's column: two transposing reads four rows apart
__device__ __forceinline__ bf16x8_t wd_frag(const lds_byte_t *p) {
  typedef __attribute__((address_space(3))) i16x4_t lds_i16x4_t;
  const i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t *)(p));
  const i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_t *)(p + 4 * kWgBig * 2));
  const i16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, v);
}

// MAP_A / MAP_B: the operand's rows are rows_x[position] (else the position itself)
template <bool MAP_A, bool MAP_B>
__global__ __launch_bounds__(512) void wgrad_bf16_dma_kernel(const bf16_t *__restrict__ A, int64_t lda, int M,
                                                             const bf16_t *__restrict__ Bm, int64_t ldb, int N,
                                                             const int32_t *__restrict__ rows_a,
                                                             const int32_t *__restrict__ rows_b,
                                                             const int32_t *__restrict__ offsets, int64_t n_pos,
                                                             int n_groups, float *__restrict__ C) {
  extern __shared__ __attribute__((aligned(16))) unsigned char wd_smem[];
  const int tn = N / kWgBig, tm = M / kWgBig;                      // (the launcher checks divisibility)
  const int per_xcd = gridDim.x / 8;                             // tiles dealt to XCDs in contiguous runs
  const int t = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (t >= tn * tm * n_groups) return;
  const int e = t / (tn * tm);
  const int64_t p_lo = offsets ? offsets[e] : 0, p_hi = offsets ? offsets[e + 1] : n_pos;
  const int m0 = ((t / tn) % tm) * kWgBig, n0 = (t % tn) * kWgBig;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave & 3, wn = wave >> 2;                       // 4 x 2 waves, 64 x 128 each
  f32x16_t acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int64_t n_grp = p_hi - p_lo;
  const int KT = static_cast<int>((n_grp + kWgSlab - 1) / kWgSlab);

  if (KT > 0) {
    const lds_byte_t *lds = (const lds_byte_t *)wd_smem;
    const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) void *)wd_smem));
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds_base + wave * (kWdInstr * 1024));

    // DMA side: instruction j of a half slab fills rows 8 wave + 2 j and + 1 of the slot; this lane
    // brings position lane & 31 of row 2 j + (lane >> 5), i.e. the chunk that belongs there
    const int half = lane >> 5;
    unsigned col_a[kWdInstr], col_b[kWdInstr];
#pragma unroll
    for (int j = 0; j < kWdInstr; ++j) {
      const int r = 2 * j + half;                                 // (8 wave is a multiple of 4)
      const unsigned c = static_cast<unsigned>((lane & 31) ^ (4 * (r & 3)));
      col_a[j] = (static_cast<unsigned>(m0) + c * 8) * 2;
      col_b[j] = (static_cast<unsigned>(n0) + c * 8) * 2;
    }
    const unsigned lda2 = static_cast<unsigned>(lda) * 2, ldb2 = static_cast<unsigned>(ldb) * 2;

    // the eight operand rows a wave brings for half slab h (uniform: scalar loads; the index only - its
    // first use, the multiply in issue(), is where the compiler waits for the load)
    auto row_idx = [&](int h, unsigned (&row)[8]) __attribute__((always_inline)) {
      const int m = h >> 1, sl = m < KT ? m : KT - 1;             // past the end: harmless reload
      const int64_t pb = p_lo + static_cast<int64_t>(sl) * kWgSlab + wave * 8;
      const int32_t *rows = (h & 1) ? rows_b : rows_a;
      const bool mapped = (h & 1) ? MAP_B : MAP_A;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int64_t pp = pb + i < n_pos ? pb + i : n_pos - 1;
        row[i] = mapped ? static_cast<unsigned>(rows[pp]) : static_cast<unsigned>(pp);
      }
    };
    auto issue = [&](int h, const unsigned (&row)[8]) __attribute__((always_inline)) {
      const unsigned slot = lds_wave + static_cast<unsigned>(h % kWdSlots) * kWdSlotBytes;
      const void *base = (h & 1) ? static_cast<const void *>(Bm) : static_cast<const void *>(A);
      const unsigned ld2 = (h & 1) ? ldb2 : lda2;
#pragma unroll
      for (int j = 0; j < kWdInstr; ++j) {
        // (the launcher checks that row * ld2 fits 32 bits)
        const unsigned voff = (half ? row[2 * j + 1] : row[2 * j]) * ld2 + ((h & 1) ? col_b[j] : col_a[j]);
        wd_dma_16(slot + j * 1024, voff, base);
      }
    };

    // fragment side: lane i of a 16-lane group names row i >> 2 (of four), columns 4 (i & 3) .. + 3 of
    // its group's 16 columns and receives column i; groups 0/1 hold tile rows 0-15 / 16-31 of
    // positions 0-7, groups 2/3 the same of positions 8-15
    const int i16 = lane & 15, grp = lane >> 4;
    const int row_l = 8 * (grp >> 1) + (i16 >> 2);
    const int sw = 4 * (i16 >> 2);
    unsigned a_off[2], b_off[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int chunk = (wm * 8 + i * 4 + 2 * (grp & 1) + ((i16 >> 1) & 1)) ^ sw;
      a_off[i] = static_cast<unsigned>(row_l * (kWgBig * 2) + chunk * 16 + (i16 & 1) * 8);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int chunk = (wn * 16 + j * 4 + 2 * (grp & 1) + ((i16 >> 1) & 1)) ^ sw;
      b_off[j] = static_cast<unsigned>(row_l * (kWgBig * 2) + chunk * 16 + (i16 & 1) * 8);
    }
    bf16x8_t fa0[2], fa1[2], fb0[4], fb1[4];
    auto load_frags = [&](int m, int kk, bf16x8_t(&af)[2], bf16x8_t(&bfr)[4]) __attribute__((always_inline)) {
      const lds_byte_t *sa = lds + ((2 * m) % kWdSlots) * kWdSlotBytes + kk * (16 * kWgBig * 2);
      const lds_byte_t *sb = lds + ((2 * m + 1) % kWdSlots) * kWdSlotBytes + kk * (16 * kWgBig * 2);
      af[0] = wd_frag(sa + a_off[0]);
#pragma unroll
      for (int j = 0; j < 4; ++j) bfr[j] = wd_frag(sb + b_off[j]);
      af[1] = wd_frag(sa + a_off[1]);
    };
    auto mma = [&](const bf16x8_t(&af)[2], const bf16x8_t(&bfr)[4]) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    };
    // rows of slab m past the group's end, both operands; ends in a barrier
    const int tail = static_cast<int>(n_grp % kWgSlab);
    auto zero_tail = [&](int m) __attribute__((always_inline)) {
      __attribute__((address_space(3))) unsigned char *sa =
          (__attribute__((address_space(3))) unsigned char *)wd_smem + ((2 * m) % kWdSlots) * kWdSlotBytes;
      __attribute__((address_space(3))) unsigned char *sb =
          (__attribute__((address_space(3))) unsigned char *)wd_smem + ((2 * m + 1) % kWdSlots) * kWdSlotBytes;
      const int first = tail * (kWgBig * 2), bytes = (kWgSlab - tail) * (kWgBig * 2);
      for (int q = tid * 16; q < bytes; q += 512 * 16) {
        *(__attribute__((address_space(3))) u32x4_t *)(sa + first + q) = u32x4_t{0u, 0u, 0u, 0u};
        *(__attribute__((address_space(3))) u32x4_t *)(sb + first + q) = u32x4_t{0u, 0u, 0u, 0u};
      }
      __syncthreads();
    };

    {
      unsigned off[kWdSlots][8];                                  // all index loads first: one round trip, not five
#pragma unroll
      for (int h = 0; h < kWdSlots; ++h) row_idx(h, off[h]);
#pragma unroll
      for (int h = 0; h < kWdSlots; ++h) issue(h, off[h]);
    }
    // slab 0 is in LDS once only A(1), B(1), A(2) are outstanding
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(3 * kWdInstr) : "memory");
    if (tail != 0 && KT == 1) zero_tail(0);
    load_frags(0, 0, fa0, fb0);

    for (int m = 0; m < KT; ++m) {
      unsigned off_b[8], off_a[8];
      row_idx(2 * m + kWdSlots, off_b);                           // B(m+2) and A(m+3), issued after this slab
      row_idx(2 * m + kWdSlots + 1, off_a);
      // the index loads leave now, a slab's worth of MFMAs before they are used (left to itself the
      // scheduler sinks them to their use behind the barrier, a scalar-memory round trip per slab)
      __builtin_amdgcn_sched_barrier(0);
      load_frags(m, 1, fa1, fb1);
      mma(fa0, fb0);
      load_frags(m, 2, fa0, fb0);
      mma(fa1, fb1);
      load_frags(m, 3, fa1, fb1);
      mma(fa0, fb0);
      // slab m+1 has landed for everyone (only A(m+2) is outstanding) and nobody reads slab m any more
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(kWdInstr) : "memory");
      issue(2 * m + kWdSlots, off_b);                             // B(m+2) into the slot of A(m)
      issue(2 * m + kWdSlots + 1, off_a);                         // A(m+3) into the slot of B(m)
      if (tail != 0 && m + 2 == KT) zero_tail(m + 1);
      load_frags(m + 1, 0, fa0, fb0);
      mma(fa1, fb1);
    }
    // no DMA may be in flight into LDS that the next workgroup on this CU owns
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  }

  // the B fragment is the MFMA's row operand: this lane holds, for output row m = frag_row, the
  // columns 8 q + 4 frag_half + r of each 32-wide tile in accumulator element 4 q + r
  float *Ce = C + static_cast<int64_t>(e) * M * N;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = m0 + wm * 64 + i * 32 + frag_row;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int cc = n0 + wn * 128 + j * 32 + q * 8 + frag_half * 4;
        *reinterpret_cast<float4 *>(Ce + static_cast<int64_t>(m) * N + cc) =
            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
      }
  }
}

// rows scaled by a per-row factor (the gate weight of Eq. (12) on d_out):
// dst[r, :] = scale[scale_idx ? scale_idx[r] : r] * src[src_idx ? src_idx[r] : r, :]
// (top-K: r is a sorted position, src_idx its token, scale_idx its slot)
template <typename T>
__global__ __launch_bounds__(256) void scale_rows_kernel(const T *__restrict__ src, const float *__restrict__ scale,
                                                         const int32_t *__restrict__ src_idx,
                                                         const int32_t *__restrict__ scale_idx, int64_t n_rows,
                                                         int n_cols, T *__restrict__ dst) {
  const int64_t i = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) * 4;   // four consecutive columns
  if (i >= n_rows * n_cols) return;
  const int64_t r = i / n_cols, c = i % n_cols;
  const int64_t rs = src_idx ? src_idx[r] : r, rg = scale_idx ? scale_idx[r] : r;
  const float g = scale[rg];
  float v[4];
  bwd_load4(src + rs * n_cols + c, v);
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] *= g;
  bwd_store4(dst + i, v);
}

// the same contraction on the plain ALUs (fp32, or bf16 shapes the MFMA kernel does not take): 64 x 64 tiles
template <typename T>
__global__ __launch_bounds__(256) void wgrad_simple_kernel(const T *__restrict__ A, int64_t lda, int M,
                                                           const T *__restrict__ Bm, int64_t ldb, int N,
                                                           const int32_t *__restrict__ rows_a,
                                                           const int32_t *__restrict__ rows_b,
                                                           const float *__restrict__ row_scale,
                                                           const int32_t *__restrict__ offsets, int64_t n_pos,
                                                           float *__restrict__ C) {
  __shared__ float As[16][64 + 4], Bs[16][64 + 4];
  const int e = blockIdx.z;
  const int64_t p_lo = offsets ? offsets[e] : 0, p_hi = offsets ? offsets[e + 1] : n_pos;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int64_t p0 = p_lo; p0 < p_hi; p0 += 16) {
    __syncthreads();
    for (int i = tid; i < 16 * 64; i += 256) {
      const int pp = i / 64, c = i % 64;
      const int64_t p = p0 + pp;
      float va = 0.0f, vb = 0.0f;
      if (p < p_hi) {
        const int64_t ra = rows_a ? rows_a[p] : p, rb = rows_b ? rows_b[p] : p;
        const float sc = row_scale ? row_scale[ra] : 1.0f;
        if (m0 + c < M) va = to_f32(A[ra * lda + m0 + c]) * sc;
        if (n0 + c < N) vb = to_f32(Bm[rb * ldb + n0 + c]);
      }
      As[pp][c] = va;
      Bs[pp][c] = vb;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[k][ty * 4 + i]; bv[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
  }
  float *Ce = C + static_cast<int64_t>(e) * M * N;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
      if (m < M && col < N) Ce[static_cast<int64_t>(m) * N + col] = acc[i][j];
    }
}

}  // namespace

size_t scan_bwd_ckpt_bytes(int64_t B, int64_t L, int d_inner) {
  return scan_bwd_layout(B, L, d_inner).total * sizeof(float);
}
size_t scan_bwd_part_bytes(int64_t n_tok, int d_inner) {
  return static_cast<size_t>(d_inner / kBwdCh) * static_cast<size_t>(n_tok) * 32 * sizeof(float);
}

template <typename T>
static hipError_t launch_scan_backward_t(const void *u, const void *dt, const float *bc, const void *z, int64_t ld_z,
                                         const void *dg, const float *gate, const float *A_log, const float *D, int64_t B,
                                         int64_t L, int d_inner, float *ws, float *d_bc_part, void *d_pre, void *d_u,
                                         void *d_z, int64_t ld_dz, float *d_A_log, float *d_D, float *d_dt_bias,
                                         hipStream_t s) {
  const ScanBwdLayout l = scan_bwd_layout(B, L, d_inner);
  const dim3 grid(static_cast<unsigned>(l.n_cb), static_cast<unsigned>(B * l.n_chunks));
  if (l.n_chunks > 1) {
    const dim3 fine_grid(static_cast<unsigned>(l.n_cb), static_cast<unsigned>(B * l.n_fine));
    hipLaunchKernelGGL((scan_bwd_carry_kernel<T>), fine_grid, dim3(256), 0, s, static_cast<const T *>(u),
                       static_cast<const T *>(dt), bc, static_cast<const T *>(z), ld_z, static_cast<const T *>(dg), gate,
                       A_log, L, d_inner, l.n_fine, l.fine_len, static_cast<int>(l.chunk_len / l.fine_len), l.n_chunks,
                       ws + l.carry_p, ws + l.carry_q, ws + l.carry_r);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((scan_bwd_kernel<T>), grid, dim3(256), 0, s, static_cast<const T *>(u), static_cast<const T *>(dt),
                     bc, static_cast<const T *>(z), ld_z, static_cast<const T *>(dg), gate, A_log, D, B, L, d_inner,
                     l.n_chunks, l.chunk_len, l.n_fine, static_cast<int>(l.chunk_len / l.fine_len), ws + l.ckpt, ws + l.carry_p, ws + l.carry_q, ws + l.carry_r,
                     static_cast<T *>(d_pre), static_cast<T *>(d_u), static_cast<T *>(d_z), ld_dz, d_bc_part,
                     ws + l.part_a, ws + l.part_d, ws + l.part_bias);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(scan_bwd_finish_kernel, dim3(static_cast<unsigned>(l.n_cb)), dim3(256), 0, s, ws + l.part_a,
                     ws + l.part_d, ws + l.part_bias, l.n_cb, B * l.n_chunks, d_A_log, d_D, d_dt_bias);
  return hipGetLastError();
}

hipError_t launch_scan_backward(int dtype, const void *u, const void *dt, const float *bc, const void *z, int64_t ld_z,
                                const void *dg, const float *gate, const float *A_log, const float *D, int64_t B,
                                int64_t L, int d_inner, float *ckpt, float *d_bc_part, void *d_pre, void *d_u, void *d_z,
                                int64_t ld_dz, float *d_bc, float *d_A_log, float *d_D, float *d_dt_bias,
                                hipStream_t s) {
  if (B * scan_bwd_layout(B, L, d_inner).n_fine > 65535) return hipErrorInvalidValue;
  hipError_t e = dtype == ROM_DTYPE_BF16
                     ? launch_scan_backward_t<bf16_t>(u, dt, bc, z, ld_z, dg, gate, A_log, D, B, L, d_inner, ckpt, d_bc_part,
                                                      d_pre, d_u, d_z, ld_dz, d_A_log, d_D, d_dt_bias, s)
                     : launch_scan_backward_t<float>(u, dt, bc, z, ld_z, dg, gate, A_log, D, B, L, d_inner, ckpt, d_bc_part,
                                                     d_pre, d_u, d_z, ld_dz, d_A_log, d_D, d_dt_bias, s);
  if (e != hipSuccess) return e;
  const int64_t n_tok = B * L;
  hipLaunchKernelGGL(bwd_reduce_bc_kernel, grid1d(n_tok * 32, 256), dim3(256), 0, s, d_bc_part, d_inner / kBwdCh, n_tok,
                     d_bc);
  return hipGetLastError();
}

hipError_t launch_gate_backward(int dtype, const void *a, const void *b, const int32_t *b_rows, int a_div,
                                int64_t n_rows, int n_cols, float *d_gate, hipStream_t s) {
  const dim3 grid = grid1d(n_rows * 64, 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL((gate_bwd_kernel<bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(a),
                       static_cast<const bf16_t *>(b), b_rows, a_div, n_rows, n_cols, d_gate);
  else
    hipLaunchKernelGGL((gate_bwd_kernel<float>), grid, dim3(256), 0, s, static_cast<const float *>(a),
                       static_cast<const float *>(b), b_rows, a_div, n_rows, n_cols, d_gate);
  return hipGetLastError();
}

size_t router_bwd_partial_bytes(int64_t n_tok, int d_model, int n_experts) {
  return static_cast<size_t>(ceil_div(n_tok, kRouterChunk)) * n_experts * (d_model + 1) * sizeof(float);
}

hipError_t launch_router_backward(int dtype, const float *logits, const int32_t *expert_idx, const float *d_gate,
                                  const void *x, int64_t n_tok, int d_model, int n_experts, int top_k, int gate_mode,
                                  float *d_logits, float *partial, float *d_w_router, float *d_b_router, hipStream_t s) {
  hipLaunchKernelGGL(router_bwd_kernel, grid1d(n_tok, 256), dim3(256), 0, s, logits, expert_idx, d_gate, n_tok, n_experts,
                     top_k, gate_mode, d_logits);
  const int n_chunks = static_cast<int>(ceil_div(n_tok, kRouterChunk));
  const dim3 grid(static_cast<unsigned>(ceil_div(d_model + 1, 256)), static_cast<unsigned>(n_chunks));
#define ROM_RW(T, EMAX)                                                                                       \
  hipLaunchKernelGGL((router_wgrad_partial_kernel<T, EMAX>), grid, dim3(256), 0, s, d_logits, static_cast<const T *>(x), \
                     n_tok, d_model, n_experts, partial)
  if (dtype == ROM_DTYPE_BF16) {
    if (n_experts <= 8) ROM_RW(bf16_t, 8); else if (n_experts <= 16) ROM_RW(bf16_t, 16); else ROM_RW(bf16_t, 64);
  } else {
    if (n_experts <= 8) ROM_RW(float, 8); else if (n_experts <= 16) ROM_RW(float, 16); else ROM_RW(float, 64);
  }
#undef ROM_RW
  hipLaunchKernelGGL(router_wgrad_finish_kernel, grid1d(static_cast<int64_t>(n_experts) * (d_model + 1), 64), dim3(256), 0,
                     s, partial, n_chunks, d_model, n_experts, d_w_router, d_b_router);
  return hipGetLastError();
}

hipError_t launch_dx_finish(int dtype, const void *dx_in, const float *d_logits, const void *w_router, int64_t n_tok,
                            int d_model, int n_experts, void *d_x, hipStream_t s) {
  const dim3 grid = grid1d(n_tok * d_model / 8, 256);      // d_model is a multiple of 8
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL((dx_finish_kernel<bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(dx_in), d_logits,
                       static_cast<const bf16_t *>(w_router), n_tok, d_model, n_experts, static_cast<bf16_t *>(d_x));
  else
    hipLaunchKernelGGL((dx_finish_kernel<float>), grid, dim3(256), 0, s, static_cast<const float *>(dx_in), d_logits,
                       static_cast<const float *>(w_router), n_tok, d_model, n_experts, static_cast<float *>(d_x));
  return hipGetLastError();
}

size_t conv_bwd_partial_bytes(int64_t B, int64_t L, int d_inner) {
  return static_cast<size_t>(B) * static_cast<size_t>(ceil_div(L, kConvBwdRun)) * 5 * d_inner * sizeof(float);
}

hipError_t launch_conv_backward(int dtype, const void *xz, int64_t ld_xz, const float *conv_w, const float *conv_b,
                                const void *du_a, const void *du_b, int64_t B, int64_t L, int d_inner, void *d_xpre,
                                int64_t ld_dx, float *partial, float *d_conv_w, float *d_conv_b, hipStream_t s) {
  const int64_t n_runs = ceil_div(L, kConvBwdRun);
  const size_t eb = dtype == ROM_DTYPE_BF16 ? 2 : 4;
  const auto al = [&](const void *p) { return reinterpret_cast<uintptr_t>(p) % (2 * eb) == 0; };
  const bool two = d_inner % 2 == 0 && ld_xz % 2 == 0 && ld_dx % 2 == 0 && al(xz) && al(du_a) && al(du_b) && al(d_xpre);
  const dim3 grid(static_cast<unsigned>(ceil_div(d_inner, two ? 512 : 256)), static_cast<unsigned>(n_runs),
                  static_cast<unsigned>(B));
#define ROM_CONV_BWD(T, V)                                                                                          \
  hipLaunchKernelGGL((conv_bwd_kernel<T, V>), grid, dim3(256), 0, s, static_cast<const T *>(xz), ld_xz, conv_w, conv_b, \
                     static_cast<const T *>(du_a), static_cast<const T *>(du_b), L, d_inner, static_cast<T *>(d_xpre),  \
                     ld_dx, partial)
  if (dtype == ROM_DTYPE_BF16) {
    if (two) ROM_CONV_BWD(bf16_t, 2); else ROM_CONV_BWD(bf16_t, 1);
  } else {
    if (two) ROM_CONV_BWD(float, 2); else ROM_CONV_BWD(float, 1);
  }
#undef ROM_CONV_BWD
  hipLaunchKernelGGL(conv_bwd_finish_kernel, grid1d(5 * d_inner, 64), dim3(256), 0, s, partial, B * n_runs, d_inner,
                     d_conv_w, d_conv_b);
  return hipGetLastError();
}

hipError_t launch_transpose(int dtype, const void *src, void *dst, int n_mats, int rows, int cols, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>(ceil_div(cols, 64)), static_cast<unsigned>(ceil_div(rows, 64)),
                  static_cast<unsigned>(n_mats));
  const int vec = rows % 4 == 0 && cols % 4 == 0 && reinterpret_cast<uintptr_t>(src) % 16 == 0 &&
                  reinterpret_cast<uintptr_t>(dst) % 16 == 0;
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL((transpose_kernel<bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(src),
                       static_cast<bf16_t *>(dst), rows, cols, vec);
  else
    hipLaunchKernelGGL((transpose_kernel<float>), grid, dim3(256), 0, s, static_cast<const float *>(src),
                       static_cast<float *>(dst), rows, cols, vec);
  return hipGetLastError();
}

hipError_t launch_pack_dxdbl(int dtype, const float *d_dt_low, const float *d_bc, int64_t n_tok, int dt_rank,
                             void *d_xdbl, hipStream_t s) {
  const dim3 grid = grid1d(n_tok * (dt_rank + 32), 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL((pack_dxdbl_kernel<bf16_t>), grid, dim3(256), 0, s, d_dt_low, d_bc, n_tok, dt_rank,
                       static_cast<bf16_t *>(d_xdbl));
  else
    hipLaunchKernelGGL((pack_dxdbl_kernel<float>), grid, dim3(256), 0, s, d_dt_low, d_bc, n_tok, dt_rank,
                       static_cast<float *>(d_xdbl));
  return hipGetLastError();
}

hipError_t launch_scale_rows(int dtype, const void *src, const float *scale, const int32_t *src_idx,
                             const int32_t *scale_idx, int64_t n_rows, int n_cols, void *dst, hipStream_t s) {
  if (n_cols % 4 != 0) return hipErrorInvalidValue;       // (d_model is a multiple of 8)
  const dim3 grid = grid1d(n_rows * n_cols / 4, 256);
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL((scale_rows_kernel<bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(src), scale,
                       src_idx, scale_idx, n_rows, n_cols, static_cast<bf16_t *>(dst));
  else
    hipLaunchKernelGGL((scale_rows_kernel<float>), grid, dim3(256), 0, s, static_cast<const float *>(src), scale,
                       src_idx, scale_idx, n_rows, n_cols, static_cast<float *>(dst));
  return hipGetLastError();
}

namespace {
// ---- RMS norm of the pre-norm block, forward (materialised for the backward pass) and adjoint
// One wavefront per token row.  xn = x r norm_w, r = 1 / sqrt(mean(x^2) + eps), r kept per token.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const T *__restrict__ x, const float *__restrict__ norm_w,
                                                          float eps, int64_t n_rows, int d_model, T *__restrict__ xn,
                                                          float *__restrict__ rstd) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const T *xr = x + row * d_model;
  float ss = 0.0f;
  for (int c = lane * 4; c < d_model; c += 256) {
    float v[4];
    bwd_load4(xr + c, v);
#pragma unroll
    for (int q = 0; q < 4; ++q) ss = fmaf(v[q], v[q], ss);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  const float r = 1.0f / sqrtf(ss / static_cast<float>(d_model) + eps);
  if (lane == 0) rstd[row] = r;
  for (int c = lane * 4; c < d_model; c += 256) {
    float v[4];
    bwd_load4(xr + c, v);
    const float4 g = *reinterpret_cast<const float4 *>(norm_w + c);
    v[0] *= r * g.x; v[1] *= r * g.y; v[2] *= r * g.z; v[3] *= r * g.w;
    bwd_store4(xn + row * d_model + c, v);
  }
}

// d_x = d_skip + r (d_xn norm_w - x^ mean_d(d_xn norm_w x^)),  x^ = x r   (d_skip may be NULL: no skip connection)
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T *__restrict__ x, const float *__restrict__ norm_w,
                                                          const float *__restrict__ rstd, const T *__restrict__ d_xn,
                                                          const T *__restrict__ d_skip, int64_t n_rows, int d_model,
                                                          T *__restrict__ d_x) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const T *xr = x + row * d_model, *dr = d_xn + row * d_model;
  const float r = rstd[row];
  float dot = 0.0f;
  for (int c = lane * 4; c < d_model; c += 256) {
    float v[4], dv[4];
    bwd_load4(xr + c, v);
    bwd_load4(dr + c, dv);
    const float4 g = *reinterpret_cast<const float4 *>(norm_w + c);
    dot = fmaf(dv[0] * g.x, v[0] * r, dot);
    dot = fmaf(dv[1] * g.y, v[1] * r, dot);
    dot = fmaf(dv[2] * g.z, v[2] * r, dot);
    dot = fmaf(dv[3] * g.w, v[3] * r, dot);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
  const float m = dot / static_cast<float>(d_model);
  for (int c = lane * 4; c < d_model; c += 256) {
    float v[4], dv[4], sk[4], o[4];
    bwd_load4(xr + c, v);
    bwd_load4(dr + c, dv);
    if (d_skip) bwd_load4(d_skip + row * d_model + c, sk);
    else sk[0] = sk[1] = sk[2] = sk[3] = 0.0f;
    const float4 g = *reinterpret_cast<const float4 *>(norm_w + c);
    o[0] = sk[0] + r * (dv[0] * g.x - v[0] * r * m);
    o[1] = sk[1] + r * (dv[1] * g.y - v[1] * r * m);
    o[2] = sk[2] + r * (dv[2] * g.z - v[2] * r * m);
    o[3] = sk[3] + r * (dv[3] * g.w - v[3] * r * m);
    bwd_store4(d_x + row * d_model + c, o);
  }
}

// d_norm_w partials: part[blockIdx.y][c] = sum over the block's rows of d_xn[n, c] x[n, c] r[n]; thread = column
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_wgrad_partial_kernel(const T *__restrict__ x,
                                                                    const float *__restrict__ rstd,
                                                                    const T *__restrict__ d_xn, int64_t n_rows,
                                                                    int d_model, int rows_per_block,
                                                                    float *__restrict__ part) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d_model) return;
  const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < n_rows ? r0 + rows_per_block : n_rows;
  float acc = 0.0f;
  for (int64_t n = r0; n < r1; ++n)
    acc = fmaf(to_f32(d_xn[n * d_model + c]) * to_f32(x[n * d_model + c]), rstd[n], acc);
  part[static_cast<int64_t>(blockIdx.y) * d_model + c] = acc;
}

// out[c] = sum over parts: a block owns 64 columns, its four waves each add every fourth part in part
// order, then the four sums are added in wave order (a fixed order either way)
__global__ __launch_bounds__(256) void colsum_kernel(const float *__restrict__ part, int n_parts, int n_cols,
                                                     float *__restrict__ out) {
  __shared__ float sums[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float acc = 0.0f;
  if (c < n_cols)
    for (int p = q; p < n_parts; p += 4) acc += part[static_cast<int64_t>(p) * n_cols + c];
  sums[q][lane] = acc;
  __syncthreads();
  if (q == 0 && c < n_cols) out[c] = (sums[0][lane] + sums[1][lane]) + (sums[2][lane] + sums[3][lane]);
}
}  // namespace

int rmsnorm_wgrad_parts(int64_t n_rows) {
  const int64_t parts = (n_rows + 63) / 64;
  return static_cast<int>(parts < 512 ? (parts < 1 ? 1 : parts) : 512);
}

hipError_t launch_rmsnorm_forward(int dtype, const void *x, const float *norm_w, float eps, int64_t n_rows, int d_model,
                                  void *xn, float *rstd, hipStream_t s) {
  if (d_model % 4 != 0) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(ceil_div(n_rows, 4)));
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL((rmsnorm_fwd_kernel<bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(x), norm_w, eps,
                       n_rows, d_model, static_cast<bf16_t *>(xn), rstd);
  else
    hipLaunchKernelGGL((rmsnorm_fwd_kernel<float>), grid, dim3(256), 0, s, static_cast<const float *>(x), norm_w, eps,
                       n_rows, d_model, static_cast<float *>(xn), rstd);
  return hipGetLastError();
}

hipError_t launch_rmsnorm_backward(int dtype, const void *x, const float *norm_w, const float *rstd, const void *d_xn,
                                   const void *d_skip, int64_t n_rows, int d_model, void *d_x, float *part,
                                   float *d_norm_w, hipStream_t s) {
  if (d_model % 4 != 0) return hipErrorInvalidValue;
  const dim3 grid(static_cast<unsigned>(ceil_div(n_rows, 4)));
  const int parts = rmsnorm_wgrad_parts(n_rows);
  const int rows_per_block = static_cast<int>(ceil_div(n_rows, parts));
  const dim3 grid_w(static_cast<unsigned>(ceil_div(d_model, 256)), static_cast<unsigned>(parts));
  if (dtype == ROM_DTYPE_BF16) {
    hipLaunchKernelGGL((rmsnorm_bwd_kernel<bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(x), norm_w, rstd,
                       static_cast<const bf16_t *>(d_xn), static_cast<const bf16_t *>(d_skip), n_rows, d_model,
                       static_cast<bf16_t *>(d_x));
    hipLaunchKernelGGL((rmsnorm_wgrad_partial_kernel<bf16_t>), grid_w, dim3(256), 0, s, static_cast<const bf16_t *>(x),
                       rstd, static_cast<const bf16_t *>(d_xn), n_rows, d_model, rows_per_block, part);
  } else {
    hipLaunchKernelGGL((rmsnorm_bwd_kernel<float>), grid, dim3(256), 0, s, static_cast<const float *>(x), norm_w, rstd,
                       static_cast<const float *>(d_xn), static_cast<const float *>(d_skip), n_rows, d_model,
                       static_cast<float *>(d_x));
    hipLaunchKernelGGL((rmsnorm_wgrad_partial_kernel<float>), grid_w, dim3(256), 0, s, static_cast<const float *>(x),
                       rstd, static_cast<const float *>(d_xn), n_rows, d_model, rows_per_block, part);
  }
  hipLaunchKernelGGL(colsum_kernel, dim3(static_cast<unsigned>(ceil_div(d_model, 64))), dim3(256), 0, s, part, parts,
                     d_model, d_norm_w);
  return hipGetLastError();
}

hipError_t launch_wgrad(int dtype, const void *A, int64_t lda, int M, const void *Bm, int64_t ldb, int N,
                        const int32_t *rows_a, const int32_t *rows_b, const float *row_scale, const int32_t *offsets,
                        int n_groups, int64_t n_pos, float *C, hipStream_t s) {
  const bool mfma = dtype == ROM_DTYPE_BF16 && M % 8 == 0 && N % 8 == 0 && lda % 8 == 0 && ldb % 8 == 0 &&
                    reinterpret_cast<uintptr_t>(A) % 16 == 0 && reinterpret_cast<uintptr_t>(Bm) % 16 == 0;
  if (mfma && !row_scale && M % kWgBig == 0 && N % kWgBig == 0 && M > 0 && N > 0 && n_pos > 0 && kUseWgradDma &&
      static_cast<uint64_t>(n_pos) * static_cast<uint64_t>(lda) * 2 < (1ull << 32) &&
      static_cast<uint64_t>(n_pos) * static_cast<uint64_t>(ldb) * 2 < (1ull << 32)) {
    // (operand rows are rows_x[p] < n_pos or p itself: 32-bit byte offsets reach every one of them)
    static std::mutex mu;
    static std::atomic<bool> done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!done[dev].load(std::memory_order_acquire)) {
      std::lock_guard<std::mutex> lock(mu);
      if (!done[dev].load(std::memory_order_relaxed)) {
        const void *fns[4] = {reinterpret_cast<const void *>(&wgrad_bf16_dma_kernel<false, false>),
                              reinterpret_cast<const void *>(&wgrad_bf16_dma_kernel<false, true>),
                              reinterpret_cast<const void *>(&wgrad_bf16_dma_kernel<true, false>),
                              reinterpret_cast<const void *>(&wgrad_bf16_dma_kernel<true, true>)};
        for (const void *fn : fns) {
          e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kWdSmem);
          if (e != hipSuccess) return e;
        }
        done[dev].store(true, std::memory_order_release);
      }
    }
    const int64_t tiles = static_cast<int64_t>(N / kWgBig) * (M / kWgBig) * n_groups;
    const dim3 grid(static_cast<unsigned>(ceil_div(tiles, 8) * 8));
    auto kernel = rows_a ? (rows_b ? &wgrad_bf16_dma_kernel<true, true> : &wgrad_bf16_dma_kernel<true, false>)
                         : (rows_b ? &wgrad_bf16_dma_kernel<false, true> : &wgrad_bf16_dma_kernel<false, false>);
    hipLaunchKernelGGL(kernel, grid, dim3(512), kWdSmem, s, static_cast<const bf16_t *>(A), lda, M,
                       static_cast<const bf16_t *>(Bm), ldb, N, rows_a, rows_b, offsets, n_pos, n_groups, C);
    return hipGetLastError();
  }
  if (mfma && !row_scale && M >= kWgBig && N >= kWgBig) {
    // more than 64 KiB of dynamic LDS: a function attribute, set once per device
    static std::mutex mu;
    static std::atomic<bool> done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!done[dev].load(std::memory_order_acquire)) {
      std::lock_guard<std::mutex> lock(mu);
      if (!done[dev].load(std::memory_order_relaxed)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_bf16_big_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kWgBigSmem);
        if (e != hipSuccess) return e;
        done[dev].store(true, std::memory_order_release);
      }
    }
    const int64_t tiles = ceil_div(N, kWgBig) * ceil_div(M, kWgBig) * n_groups;
    const dim3 grid(static_cast<unsigned>(ceil_div(tiles, 8) * 8));
    hipLaunchKernelGGL(wgrad_bf16_big_kernel, grid, dim3(512), kWgBigSmem, s, static_cast<const bf16_t *>(A), lda, M,
                       static_cast<const bf16_t *>(Bm), ldb, N, rows_a, rows_b, offsets, n_pos, n_groups, C);
    return hipGetLastError();
  }
  if (mfma && !row_scale) {
    const dim3 grid(static_cast<unsigned>(ceil_div(N, kWgTile)), static_cast<unsigned>(ceil_div(M, kWgTile)),
                    static_cast<unsigned>(n_groups));
    hipLaunchKernelGGL(wgrad_bf16_kernel, grid, dim3(256), 0, s, static_cast<const bf16_t *>(A), lda, M,
                       static_cast<const bf16_t *>(Bm), ldb, N, rows_a, rows_b, offsets, n_pos, C);
    return hipGetLastError();
  }
  const dim3 grid(static_cast<unsigned>(ceil_div(N, 64)), static_cast<unsigned>(ceil_div(M, 64)),
                  static_cast<unsigned>(n_groups));
  if (dtype == ROM_DTYPE_BF16)
    hipLaunchKernelGGL((wgrad_simple_kernel<bf16_t>), grid, dim3(256), 0, s, static_cast<const bf16_t *>(A), lda, M,
                       static_cast<const bf16_t *>(Bm), ldb, N, rows_a, rows_b, row_scale, offsets, n_pos, C);
  else
    hipLaunchKernelGGL((wgrad_simple_kernel<float>), grid, dim3(256), 0, s, static_cast<const float *>(A), lda, M,
                       static_cast<const float *>(Bm), ldb, N, rows_a, rows_b, row_scale, offsets, n_pos, C);
  return hipGetLastError();
}

}  // namespace rom
