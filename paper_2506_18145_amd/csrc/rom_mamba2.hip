// RoM on a Mamba2 layer (Sec. 5.2, Table 3): the sequence part between the routed input and output
// projections - Mamba2's recurrence per head
//     H_t = exp(dt_t A) H_{t-1} + dt_t x_t B_t^T   (H: P x N),     y_t = H_t C_t + D x_t
// followed by the SiLU(z) gate, and the RMS norm of the gated rows.  gfx950 only, bf16 activations.
//
// The recurrence runs in its chunked ("dual") form on the matrix cores: over a chunk of Q = 64 steps
// with cum_t = sum_{r <= t} dt_r A inside the chunk,
//     y_t   = exp(cum_t) C_t . H_prev + sum_{s <= t} (C_t . B_s) exp(cum_t - cum_s) dt_s x_s
//     H_new = exp(cum_Q) H_prev + sum_s exp(cum_Q - cum_s) dt_s B_s x_s^T
// which is four small matrix products per chunk (scores C B^T, scores x inputs, C x state, B^T x
// inputs); every exponent is <= 0, so nothing overflows however strong the decay.  A workgroup
// (4 wavefronts) owns one (sequence, head, segment of the sequence) and walks its chunks in order
// with the state H in MFMA accumulators (fp32): wavefront w holds H[:, 16w .. 16w+15] and produces
// the same 16 output channels, so the state never leaves its registers - as the B operand of
// C x state it is read straight from the accumulators (the contraction index is permuted the same
// way on the C side).  Sequences are cut into segments until there are two workgroups per CU; a
// first pass (the same kernel without its output part) leaves every segment's end state from a
// zero start and its total log decay, which the main pass folds in segment order.
#include "rom_chunk.h"

#include <atomic>
#include <mutex>

namespace rom {
namespace {

using namespace chunk;

constexpr int kP = 64;          // channels per head

// LDS of one workgroup.  Rows are padded by 8 halfs (16 bytes): the 16-byte fragment reads of 16
// consecutive rows then fall into different banks.
template <int NS>
struct SsdSmem {
  union {
    bf16_t b[kQ][NS + 8];       // B, step-major (operand of the scores)
    float y[kQ][kP + 4];        // later in the chunk: the output tile, for row-wise stores
  } u;
  bf16_t c[kQ][NS + 8];         // C, step-major
  bf16_t bw_t[NS][kQ + 8];      // exp(cum_Q - cum_s) dt_s B_s, state-major (operand of the state update)
  bf16_t xd_t[kP][kQ + 8];      // x, channel-major
  bf16_t g[kQ][kQ + 8];         // masked, decayed, dt-weighted scores [t][s]
  float cum[kQ], ecum[kQ], dt[kQ];   // cum_t, exp(cum_t), dt_t
};

// Grid (n_heads, B * n_seg).  CARRY: the state-only pass (segments before the last one).
//   xbc   bf16 [B*L, ld_xbc]: x of head h at columns x_col + 64 h, B at b_col, C at c_col (after conv + SiLU)
//   dt_raw bf16 [B*L, ld_dt]: column dt_col + h, before bias and softplus;   z bf16 [B*L, ld_z]: column 64 h
//   carry_state f32 [B][n_seg][H][NS][64], carry_decay f32 [B][n_seg][H]
//   h_in / h_out f32 [B][H][NS][64] or NULL: the state before the first and after the last step
//   yz    bf16 [B*L, ld_y]: (y + D x) * SiLU(z)
template <int NS, bool CARRY>
__global__ __launch_bounds__(256, 2) void ssd_kernel(const bf16_t *__restrict__ xbc, int64_t ld_xbc, int x_col, int b_col,
                                                  int c_col, const bf16_t *__restrict__ dt_raw, int64_t ld_dt,
                                                  int dt_col, const bf16_t *__restrict__ z, int64_t ld_z,
                                                  const float *__restrict__ dt_bias, const float *__restrict__ A_log,
                                                  const float *__restrict__ Dp, int64_t L, int n_seg, int64_t seg_len,
                                                  float *__restrict__ carry_state, float *__restrict__ carry_decay,
                                                  const float *h_in, float *h_out, bf16_t *__restrict__ yz,
                                                  int64_t ld_y) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  SsdSmem<NS> &sm = *reinterpret_cast<SsdSmem<NS> *>(smem_raw);
  constexpr int kNB = NS / 16;          // 16-row blocks of the state
  constexpr int kKS = NS / 32;          // 32-wide steps of a contraction over the state index
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  const int h = blockIdx.x, n_heads = gridDim.x;
  const int64_t b = blockIdx.y / n_seg;
  const int seg = static_cast<int>(blockIdx.y % n_seg);
  if (CARRY && seg == n_seg - 1) return;            // nobody needs the last segment's end state
  const int64_t ts = seg * seg_len, te = ts + seg_len < L ? ts + seg_len : L;
  const float a = -__expf(A_log[h]);
  const float bias = dt_bias[h];
  const bf16_t *xbc_b = xbc + b * L * ld_xbc;
  const bf16_t *dt_b = dt_raw + b * L * ld_dt + dt_col + h;
  const int xc = x_col + h * kP;

  // state: hacc[nb][r] = H[n = 16 nb + 4 g + r][p = 16 wave + c]
  f32x4_t hacc[kNB];
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb) hacc[nb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
  const int64_t carry_stride = static_cast<int64_t>(NS) * kP;
  if (!CARRY) {
    if (h_in) {
      const float *sp = h_in + (b * n_heads + h) * carry_stride + wave * 16 + c;
#pragma unroll
      for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) hacc[nb][r] = sp[(16 * nb + 4 * g + r) * kP];
    }
    // fold the earlier segments' (decay, end state from zero) in order
    for (int j = 0; j < seg; ++j) {
      const int64_t unit = (b * n_seg + j) * n_heads + h;
      const float dec = fast_exp2(carry_decay[unit] * kLog2e);
      const float *sp = carry_state + unit * carry_stride + wave * 16 + c;
#pragma unroll
      for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) hacc[nb][r] = fmaf(dec, hacc[nb][r], sp[(16 * nb + 4 * g + r) * kP]);
    }
  }
  float log_decay_total = 0.0f;

  // roles while a chunk is parked: threads [0, NS) transpose B, the next 64 transpose x
  const bool is_b = tid < NS;
  const bool is_x = tid >= NS && tid < NS + 64;
  const int lt = is_b ? tid : tid - NS;
  // eight steps 8 so .., eight columns 8 co ..; consecutive lanes take consecutive column blocks of
  // the same steps (whole rows per request, and the step-major copy of B lands in distinct banks)
  const int n_co = is_b ? NS / 8 : kP / 8;
  const int so = lt / n_co, co = lt % n_co;
  // The channel-major arrays keep their 16-byte step pieces in swizzled order: piece j of row r
  // sits at position j ^ ((r >> 3) & 7), so that the eight lanes that write the same steps of eight
  // different column blocks (rows 8 apart: the same banks otherwise) hit distinct banks.
  const int so_phys = so ^ (co & 7);
  const int t_col = is_b ? b_col + 8 * co : xc + 8 * co;
  // output rows: a wavefront stores the 16 channels it computed, two 8-channel pieces per step
  const int e_row = lane >> 1, e_po = 2 * wave + (lane & 1);

  // A chunk's inputs are requested one chunk ahead (rows beyond the segment's end: the last valid
  // row, zeroed when parked - no branch around a load, so that the requests go out back to back):
  // what the parking needs right after the chunk before has been parked, what the output rows need
  // (x for the D skip, z) after the chunk before has been stored.
  u32x4_t pv[8], pc[NS / 32], ex[2], ez[2];
  unsigned short p_dt = 0;
  // this thread's rows in the chunk to fetch next; the pointers advance by a chunk per fetch (no
  // 64-bit multiplies per row), and only the segment's last, ragged chunk takes the clamped path
  const bf16_t *dt_ptr = dt_b + (ts + lane) * ld_dt;
  const bf16_t *pv_ptr = xbc_b + (ts + 8 * so) * ld_xbc + t_col;
  const bf16_t *pc_ptr[NS / 32];
#pragma unroll
  for (int i = 0; i < NS / 32; ++i) {               // C: 64 rows of NS / 8 pieces
    const int piece = tid + 256 * i;
    pc_ptr[i] = xbc_b + (ts + piece / (NS / 8)) * ld_xbc + c_col + 8 * (piece % (NS / 8));
  }
  const bf16_t *ex_ptr = xbc_b + (ts + e_row) * ld_xbc + xc + 8 * e_po;
  const bf16_t *ez_ptr = z + (b * L + ts + e_row) * ld_z + h * kP + 8 * e_po;
  auto fetch_main = [&](int64_t t0) {
    if (t0 >= te) return;
    if (t0 + kQ <= te) {
      p_dt = *dt_ptr;
      if (is_b || is_x) {
        const bf16_t *row = pv_ptr;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          pv[i] = *reinterpret_cast<const u32x4_t *>(row);
          row += ld_xbc;
        }
      }
      if (!CARRY) {
#pragma unroll
        for (int i = 0; i < NS / 32; ++i) pc[i] = *reinterpret_cast<const u32x4_t *>(pc_ptr[i]);
      }
    } else {
      const int64_t last = te - 1 - t0;               // last valid row of the chunk
      p_dt = dt_ptr[(lane <= last ? 0 : last - lane) * ld_dt];
      if (is_b || is_x) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int64_t r = 8 * so + i;
          pv[i] = *reinterpret_cast<const u32x4_t *>(pv_ptr + (r <= last ? i : last - 8 * so) * ld_xbc);
        }
      }
      if (!CARRY) {
#pragma unroll
        for (int i = 0; i < NS / 32; ++i) {
          const int64_t r = (tid + 256 * i) / (NS / 8);
          pc[i] = *reinterpret_cast<const u32x4_t *>(pc_ptr[i] + (r <= last ? 0 : last - r) * ld_xbc);
        }
      }
    }
    dt_ptr += kQ * ld_dt;
    pv_ptr += kQ * ld_xbc;
#pragma unroll
    for (int i = 0; i < NS / 32; ++i) pc_ptr[i] += kQ * ld_xbc;
  };
  auto fetch_out = [&](int64_t t0) {
    if (CARRY || t0 >= te) return;
    const int64_t last = te - 1 - t0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t r = e_row + 32 * i;
      const int64_t back = r <= last ? r - e_row : last - e_row;      // rows relative to this thread's first
      ex[i] = *reinterpret_cast<const u32x4_t *>(ex_ptr + back * ld_xbc);
      ez[i] = *reinterpret_cast<const u32x4_t *>(ez_ptr + back * ld_z);
    }
    ex_ptr += kQ * ld_xbc;
    ez_ptr += kQ * ld_z;
  };
  fetch_main(ts);
  fetch_out(ts);

  for (int64_t t0 = ts; t0 < te; t0 += kQ) {
    // time steps of the chunk, one per lane (every wavefront computes them for itself)
    float dtv = 0.0f;
    if (t0 + lane < te) dtv = softplus_f32(bf16_to_f32(p_dt) + bias);
    const float cum = wave_inclusive_sum(dtv * a);
    const float cum_last = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cum), 63));
    log_decay_total += cum_last;

    __syncthreads();                // the chunk before this one is done with the LDS
    if (is_b || is_x) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (t0 + 8 * so + i >= te) pv[i] = u32x4_t{0u, 0u, 0u, 0u};
      if (is_b) {
        // this lane's weight w_s = exp(cum_Q - cum_s) dt_s; the eight steps of the block come from their lanes
        const float w_lane = fast_exp2((cum_last - cum) * kLog2e) * dtv;
        float f[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = __shfl(w_lane, 8 * so + i);
        if (!CARRY) {
#pragma unroll
          for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4_t *>(&sm.u.b[8 * so + i][8 * co]) = pv[i];
        }
        park_scaled_8x8<kQ + 8>(pv, f, sm.bw_t, 8 * co, 8 * so_phys);
      } else {
        park_8x8<kQ + 8>(pv, sm.xd_t, 8 * co, 8 * so_phys);
      }
    }
    if (!CARRY) {
#pragma unroll
      for (int i = 0; i < NS / 32; ++i) {
        const int piece = tid + 256 * i;
        const int row = piece / (NS / 8);
        if (t0 + row >= te) pc[i] = u32x4_t{0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4_t *>(&sm.c[row][8 * (piece % (NS / 8))]) = pc[i];
      }
      if (wave == 3) {                // the wavefront with no block to transpose
        sm.cum[lane] = cum;
        sm.ecum[lane] = fast_exp2(cum * kLog2e);
        sm.dt[lane] = dtv;
      }
    }
    __syncthreads();
    fetch_main(t0 + kQ);

    f32x4_t yacc[4];
    if (!CARRY) {
      // scores, this wavefront's 16 steps t = 16 wave + c against all s: G^T[s][t] = B_s . C_t, then the
      // causal mask, the decay exp(cum_t - cum_s) and the step size dt_s; stored [t][s]
      const float cum_t = sm.cum[16 * wave + c];
#pragma unroll
      for (int sb = 0; sb < 4; ++sb) {
        f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        if (sb <= wave) {
#pragma unroll
          for (int ks = 0; ks < kKS; ++ks) {
            const bf16x8_t fa = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.u.b[16 * sb + c][32 * ks + 8 * g]));
            const bf16x8_t fb = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.c[16 * wave + c][32 * ks + 8 * g]));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, acc, 0, 0, 0);
          }
        }
        const f32x4_t cum_s = *reinterpret_cast<const f32x4_t *>(&sm.cum[16 * sb + 4 * g]);
        const f32x4_t dt_s = *reinterpret_cast<const f32x4_t *>(&sm.dt[16 * sb + 4 * g]);
        float val[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int s = 16 * sb + 4 * g + r, t = 16 * wave + c;
          val[r] = s <= t ? acc[r] * dt_s[r] * fast_exp2((cum_t - cum_s[r]) * kLog2e) : 0.0f;
        }
        const u32x2_t packed = {pack_bf16x2(val[0], val[1]), pack_bf16x2(val[2], val[3])};
        *reinterpret_cast<u32x2_t *>(&sm.g[16 * wave + c][16 * sb + 4 * g]) = packed;
      }
      // contribution of the state the chunk starts from: Y[t][p] = exp(cum_t) sum_n C[t][n] H[n][p].
      // The accumulators are the B operand as they are: slot (g, e) of a 32-wide step holds
      // n = 32 ks + 4 g + e (e < 4) or 32 ks + 16 + 4 g + e - 4, and C is read in the same order.
      bf16x8_t hop[kKS];
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) {
        const u32x4_t hv = {pack_bf16x2(hacc[2 * ks][0], hacc[2 * ks][1]), pack_bf16x2(hacc[2 * ks][2], hacc[2 * ks][3]),
                            pack_bf16x2(hacc[2 * ks + 1][0], hacc[2 * ks + 1][1]),
                            pack_bf16x2(hacc[2 * ks + 1][2], hacc[2 * ks + 1][3])};
        hop[ks] = as_frag(hv);
      }
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
        yacc[tb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ks = 0; ks < kKS; ++ks) {
          const u32x2_t lo = *reinterpret_cast<const u32x2_t *>(&sm.c[16 * tb + c][32 * ks + 4 * g]);
          const u32x2_t hi = *reinterpret_cast<const u32x2_t *>(&sm.c[16 * tb + c][32 * ks + 16 + 4 * g]);
          yacc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag_from_halves(lo, hi), hop[ks], yacc[tb], 0, 0, 0);
        }
        const f32x4_t e = *reinterpret_cast<const f32x4_t *>(&sm.ecum[16 * tb + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r) yacc[tb][r] *= e[r];
      }
      __syncthreads();              // all scores are in LDS; nobody reads B's step-major copy any more
    }

    // x of this wavefront's 16 channels, all 64 steps: B operand of both remaining products
    bf16x8_t xop[2];
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2)
      xop[k2] = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.xd_t[16 * wave + c][8 * ((4 * k2 + g) ^ ((2 * wave + (c >> 3)) & 7))]));
    if (!CARRY) {
      // inside the chunk: Y[t][p] += sum_{s <= t} G[t][s] x_s[p]; steps 32.. only reach t >= 32
#pragma unroll
      for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
          if (k2 == 0 || tb >= 2) {
            const bf16x8_t fa = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.g[16 * tb + c][32 * k2 + 8 * g]));
            yacc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, xop[k2], yacc[tb], 0, 0, 0);
          }
    }
    // state at the chunk's end: H = exp(cum_Q) H + sum_s (exp(cum_Q - cum_s) dt_s B_s) x_s^T
    {
      const float dec = fast_exp2(cum_last * kLog2e);
#pragma unroll
      for (int nb = 0; nb < kNB; ++nb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) hacc[nb][r] *= dec;
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          const bf16x8_t fa = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.bw_t[16 * nb + c][8 * ((4 * k2 + g) ^ ((2 * nb + (c >> 3)) & 7))]));
          hacc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, xop[k2], hacc[nb], 0, 0, 0);
        }
      }
    }
    if (!CARRY) {
      // output tile through LDS (over B's step-major copy) so that rows go out in 16-byte pieces, with
      // the D skip and the SiLU(z) gate applied on the way; a wavefront reads back only the 16
      // columns it wrote itself, so no barrier is needed between the two
#pragma unroll
      for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int r = 0; r < 4; ++r) sm.u.y[16 * tb + 4 * g + r][16 * wave + c] = yacc[tb][r];
      const float d_skip = Dp[h];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = e_row + 32 * i;
        const int64_t t = t0 + row;
        const f32x4_t y0 = *reinterpret_cast<const f32x4_t *>(&sm.u.y[row][8 * e_po]);
        const f32x4_t y1 = *reinterpret_cast<const f32x4_t *>(&sm.u.y[row][8 * e_po + 4]);
        float o[8];
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          const float yv = (m < 4 ? y0[m & 3] : y1[m & 3]) + d_skip * bf16_elem(ex[i], m);
          o[m] = yv * silu_f32(bf16_elem(ez[i], m));
        }
        const u32x4_t ov = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]),
                            pack_bf16x2(o[6], o[7])};
        if (t < te) *reinterpret_cast<u32x4_t *>(yz + (b * L + t) * ld_y + h * kP + 8 * e_po) = ov;
      }
      fetch_out(t0 + kQ);
    }
  }

  if (CARRY) {
    const int64_t unit = (b * n_seg + seg) * n_heads + h;
    float *sp = carry_state + unit * carry_stride + wave * 16 + c;
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
      for (int r = 0; r < 4; ++r) sp[(16 * nb + 4 * g + r) * kP] = hacc[nb][r];
    if (tid == 0) carry_decay[unit] = log_decay_total;
  } else if (h_out && seg == n_seg - 1) {
    float *sp = h_out + (b * n_heads + h) * carry_stride + wave * 16 + c;
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
      for (int r = 0; r < 4; ++r) sp[(16 * nb + 4 * g + r) * kP] = hacc[nb][r];
  }
}

// One step per sequence (L == 1): grid (n_heads, B); thread = (channel p, quarter of the states).
// The state is read and written once, 64 consecutive channels per state index.
template <int NS>
__global__ __launch_bounds__(256) void ssd_step_kernel(const bf16_t *__restrict__ xbc, int64_t ld_xbc, int x_col, int b_col,
                                                       int c_col, const bf16_t *__restrict__ dt_raw, int64_t ld_dt,
                                                       int dt_col, const bf16_t *__restrict__ z, int64_t ld_z,
                                                       const float *__restrict__ dt_bias, const float *__restrict__ A_log,
                                                       const float *__restrict__ Dp, const float *h_in, float *h_out,
                                                       bf16_t *__restrict__ yz, int64_t ld_y) {
  __shared__ float part[4][kP];
  const int tid = threadIdx.x, p = tid & 63, q = tid >> 6;
  const int h = blockIdx.x, n_heads = gridDim.x;
  const int64_t b = blockIdx.y;
  const float dt = softplus_f32(bf16_to_f32(dt_raw[b * ld_dt + dt_col + h]) + dt_bias[h]);
  const float dec = fast_exp2(-__expf(A_log[h]) * dt * kLog2e);
  const bf16_t *row = xbc + b * ld_xbc;
  const float xv = bf16_to_f32(row[x_col + h * kP + p]);
  const float dtx = dt * xv;
  const int64_t base = (b * n_heads + h) * static_cast<int64_t>(NS) * kP + p;
  float acc = 0.0f;
#pragma unroll 8
  for (int j = 0; j < NS / 4; ++j) {
    const int n = q * (NS / 4) + j;
    const float hv = fmaf(dec, h_in ? h_in[base + static_cast<int64_t>(n) * kP] : 0.0f, dtx * bf16_to_f32(row[b_col + n]));
    if (h_out) h_out[base + static_cast<int64_t>(n) * kP] = hv;
    acc = fmaf(bf16_to_f32(row[c_col + n]), hv, acc);
  }
  part[q][p] = acc;
  __syncthreads();
  if (q == 0) {
    const float y = part[0][p] + part[1][p] + part[2][p] + part[3][p] + Dp[h] * xv;
    yz[b * ld_y + h * kP + p] = f32_to_bf16(y * silu_f32(bf16_to_f32(z[b * ld_z + h * kP + p])));
  }
}

// g[n, :] = yz[n, :] / sqrt(mean(yz[n, :]^2) + eps) * w: one wavefront per row, fp32 sums
__global__ __launch_bounds__(256) void rms_rows_kernel(const bf16_t *__restrict__ yz, const float *__restrict__ w,
                                                       float eps, int64_t n_rows, int n_cols, bf16_t *__restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const bf16_t *src = yz + row * n_cols;
  float ss = 0.0f;
  for (int c0 = lane * 8; c0 < n_cols; c0 += 512) {
    const u32x4_t v = *reinterpret_cast<const u32x4_t *>(src + c0);
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      const float f = bf16_elem(v, m);
      ss = fmaf(f, f, ss);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  const float rstd = rsqrtf(ss / static_cast<float>(n_cols) + eps);
  bf16_t *dst = out + row * n_cols;
  for (int c0 = lane * 8; c0 < n_cols; c0 += 512) {
    const u32x4_t v = *reinterpret_cast<const u32x4_t *>(src + c0);
    const f32x4_t w0 = *reinterpret_cast<const f32x4_t *>(w + c0), w1 = *reinterpret_cast<const f32x4_t *>(w + c0 + 4);
    float o[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) o[m] = bf16_elem(v, m) * rstd * (m < 4 ? w0[m & 3] : w1[m & 3]);
    const u32x4_t ov = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])};
    *reinterpret_cast<u32x4_t *>(dst + c0) = ov;
  }
}

struct SsdPlan {
  int n_seg;
  int64_t seg_len;
};
SsdPlan ssd_plan(int64_t B, int64_t L, int n_heads) {
  // two workgroups for each of the 256 CUs; a segment is whole chunks and at least four of them
  const int64_t chunks = ceil_div(L, kQ);
  int64_t n_seg = ceil_div(512, B * n_heads);
  const int64_t max_seg = chunks / 4 > 0 ? chunks / 4 : 1;
  n_seg = n_seg < 1 ? 1 : (n_seg > max_seg ? max_seg : n_seg);
  SsdPlan p;
  p.seg_len = ceil_div(chunks, n_seg) * kQ;
  p.n_seg = static_cast<int>(ceil_div(L, p.seg_len));
  return p;
}

template <int NS, bool CARRY>
hipError_t ssd_allow_lds() {
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
      e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ssd_kernel<NS, CARRY>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizeof(SsdSmem<NS>)));
      if (e != hipSuccess) return e;
      done[dev].store(true, std::memory_order_release);
    }
  }
  return hipSuccess;
}

template <int NS>
hipError_t ssd_dispatch(const bf16_t *xbc, int64_t ld_xbc, int x_col, int b_col, int c_col, const bf16_t *dt_raw,
                        int64_t ld_dt, int dt_col, const bf16_t *z, int64_t ld_z, const float *dt_bias,
                        const float *A_log, const float *D, const float *h_in, float *h_out, int64_t B, int64_t L,
                        int n_heads, float *carry, bf16_t *yz, int64_t ld_y, hipStream_t s) {
  if (L == 1) {
    hipLaunchKernelGGL((ssd_step_kernel<NS>), dim3(static_cast<unsigned>(n_heads), static_cast<unsigned>(B)), dim3(256), 0,
                       s, xbc, ld_xbc, x_col, b_col, c_col, dt_raw, ld_dt, dt_col, z, ld_z, dt_bias, A_log, D, h_in, h_out,
                       yz, ld_y);
    return hipGetLastError();
  }
  const SsdPlan p = ssd_plan(B, L, n_heads);
  float *carry_state = carry;
  float *carry_decay = carry + static_cast<size_t>(B) * p.n_seg * n_heads * NS * kP;
  const dim3 grid(static_cast<unsigned>(n_heads), static_cast<unsigned>(B * p.n_seg));
  const size_t lds = sizeof(SsdSmem<NS>);
  hipError_t e;
  if (p.n_seg > 1) {
    if ((e = ssd_allow_lds<NS, true>()) != hipSuccess) return e;
    hipLaunchKernelGGL((ssd_kernel<NS, true>), grid, dim3(256), lds, s, xbc, ld_xbc, x_col, b_col, c_col, dt_raw, ld_dt,
                       dt_col, z, ld_z, dt_bias, A_log, D, L, p.n_seg, p.seg_len, carry_state, carry_decay, h_in, h_out, yz,
                       ld_y);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if ((e = ssd_allow_lds<NS, false>()) != hipSuccess) return e;
  hipLaunchKernelGGL((ssd_kernel<NS, false>), grid, dim3(256), lds, s, xbc, ld_xbc, x_col, b_col, c_col, dt_raw, ld_dt,
                     dt_col, z, ld_z, dt_bias, A_log, D, L, p.n_seg, p.seg_len, carry_state, carry_decay, h_in, h_out, yz,
                     ld_y);
  return hipGetLastError();
}

}  // namespace

size_t ssd_carry_bytes(int64_t B, int64_t L, int n_heads, int d_state) {
  const SsdPlan p = ssd_plan(B, L, n_heads);
  if (p.n_seg <= 1) return 0;
  return static_cast<size_t>(B) * p.n_seg * n_heads * (static_cast<size_t>(d_state) * kP + 1) * sizeof(float);
}

bool ssd_supported(int d_state, int headdim) { return headdim == kP && (d_state == 64 || d_state == 128); }

hipError_t launch_ssd_scan(const void *xbc, int64_t ld_xbc, int x_col, int b_col, int c_col, const void *dt_raw,
                           int64_t ld_dt, int dt_col, const void *z, int64_t ld_z, const float *dt_bias,
                           const float *A_log, const float *D, const float *h_in, float *h_out, int64_t B, int64_t L,
                           int n_heads, int d_state, float *carry, void *yz, int64_t ld_y, hipStream_t s) {
  if (B * L <= 0) return hipSuccess;
  if (B * ssd_plan(B, L, n_heads).n_seg > 65535) return hipErrorInvalidValue;
  const bf16_t *xp = static_cast<const bf16_t *>(xbc), *dp = static_cast<const bf16_t *>(dt_raw);
  const bf16_t *zp = static_cast<const bf16_t *>(z);
  if (d_state == 128)
    return ssd_dispatch<128>(xp, ld_xbc, x_col, b_col, c_col, dp, ld_dt, dt_col, zp, ld_z, dt_bias, A_log, D, h_in, h_out, B,
                             L, n_heads, carry, static_cast<bf16_t *>(yz), ld_y, s);
  if (d_state == 64)
    return ssd_dispatch<64>(xp, ld_xbc, x_col, b_col, c_col, dp, ld_dt, dt_col, zp, ld_z, dt_bias, A_log, D, h_in, h_out, B,
                            L, n_heads, carry, static_cast<bf16_t *>(yz), ld_y, s);
  return hipErrorInvalidValue;
}

hipError_t launch_rms_rows(const void *yz, const float *w, float eps, int64_t n_rows, int n_cols, void *out,
                           hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(rms_rows_kernel, dim3(static_cast<unsigned>(ceil_div(n_rows, 4))), dim3(256), 0, s,
                     static_cast<const bf16_t *>(yz), w, eps, n_rows, n_cols, static_cast<bf16_t *>(out));
  return hipGetLastError();
}

}  // namespace rom
