// RoM on a Gated DeltaNet layer (Sec. 5.2, Table 3): the sequence part between the routed input and
// output projections - per head the gated delta rule on the state S (d_v x d_k)
//     S_t = exp(g_t) S_{t-1} (I - beta_t k_t k_t^T) + beta_t v_t k_t^T,     o_t = S_t q_t
// with q, k L2-normalised per head, then the per-head RMS norm and the SiLU(z) gate.  gfx950 only,
// bf16 activations, d_v = 64, d_k = 64 or 128.
//
// Chunked form (chunks of 64 steps, cum_t = sum_{r <= t} g_r inside the chunk, gamma = exp(cum)): the
// rank-one updates u_t = beta_t (v_t - exp(g_t) S_{t-1} k_t) of a chunk obey the unit lower-triangular
// system
//     (I + A) U = diag(beta) (V - diag(gamma) K S_0^T),   A[t][s] = beta_t exp(cum_t - cum_s) (k_t . k_s), s < t,
// and then  O = diag(gamma) Q S_0^T + (Q K^T o exp(cum_t - cum_s), s <= t) U,
//           S_new = gamma_64 S_0 + sum_s exp(cum_64 - cum_s) u_s k_s^T.
// Everything but the inverse is a small matrix product on v_mfma_f32_16x16x32_bf16; T = (I + A)^-1 is
// computed in fp32 by one wavefront: the four 16 x 16 diagonal blocks by forward substitution (a lane
// per column), the six blocks below them by block substitution on v_mfma_f32_16x16x4_f32.
// A workgroup (4 wavefronts) owns one (sequence, head, segment of the sequence) and walks its chunks in
// order.  Few (sequence, head) pairs: the sequences are cut into segments.  A segment's effect on the
// state is S_end = S_start Phi + Z with Phi = prod_t exp(g_t)(I - beta_t k_t k_t^T) a d_k x d_k MATRIX, so
// the carry pass runs the same rule on the state augmented by d_k more "value" rows that start from the
// identity and see v = 0 (their end value is Phi), a small kernel folds (Phi, Z) along each sequence, and
// the main pass starts every segment from its folded state.  Wavefront w
// holds the state columns S^T[:, 16w .. 16w+15] (d_k x 16 values of d_v) in accumulators, as the
// Mamba2 kernel does, and the products that contract over steps or over d_k take their second
// operand straight from accumulators (the contraction index permuted alike on the other side).
#include "rom_chunk.h"

#include <atomic>
#include <mutex>

namespace rom {
namespace {

using namespace chunk;

constexpr int kV = 64;          // value channels per head
constexpr float kL2Eps = 1e-6f;

template <int NS>
struct GdnSmem {
  union {
    struct {
      bf16_t kn[kQ][NS + 8];    // normalised keys, step-major
      bf16_t qr[kQ][NS + 8];    // raw queries, step-major
    } in;
    float tm[kQ][kQ + 4];       // after the scores: T = (I + A)^-1 in fp32
  } u;
  union {
    float am[kQ][kQ + 4];       // A (strictly lower triangle), fp32
    float y[kQ][kV + 4];        // later in the chunk: the output tile
  } a;
  bf16_t vt[kQ][kV + 8];        // values, step-major
  bf16_t kw_t[NS][kQ + 8];      // exp(cum_64 - cum_s) k_s, channel-major, 16-byte pieces swizzled
  bf16_t tb[kQ][kQ + 8];        // T in bf16 [t][s]
  bf16_t gs[kQ][kQ + 8];        // exp(cum_t - cum_s) (q_t . k_s), s <= t, [t][s]
  float cum[kQ], ecum[kQ], beta[kQ], rq[kQ];
};

__device__ __forceinline__ float sum_sq8(const u32x4_t &v) {
  float s = 0.0f;
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const float f = bf16_elem(v, m);
    s = fmaf(f, f, s);
  }
  return s;
}
// sum over the WIDTH (8 or 16) consecutive lanes that share a row
template <int WIDTH>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int off = 1; off < WIDTH; off <<= 1) v += __shfl_xor(v, off);
  return v;
}

// T = (I + A)^-1 for the 64 x 64 unit lower-triangular I + A: am -> tm (fp32), tb (bf16).  Called by the
// whole workgroup (it contains barriers): wavefront 0 solves the four diagonal blocks, then the blocks
// at distance 1, 2, 3 below the diagonal are computed level by level, one block per wavefront.
__device__ __forceinline__ void invert_unit_lower(const float (*am)[kQ + 4], float (*tm)[kQ + 4], bf16_t (*tb)[kQ + 8],
                                                  int lane, int wave) {
  const int g = lane >> 4, c = lane & 15;
  // diagonal blocks: lane (g, c) solves column c of block g by forward substitution
  if (wave == 0) {
    float x[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float acc = r == c ? 1.0f : 0.0f;
#pragma unroll
      for (int m = 0; m < r; ++m) acc = fmaf(-am[16 * g + r][16 * g + m], x[m], acc);
      x[r] = acc;
      asm volatile("" ::: "memory");         // row by row: hoisting all 120 LDS reads costs as many registers
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      tm[16 * g + r][16 * g + c] = x[r];
      tb[16 * g + r][16 * g + c] = f32_to_bf16(x[r]);
#pragma unroll
      for (int j = 0; j < 4; ++j)            // blocks above the diagonal are zero
        if (j > g) tb[16 * g + r][16 * j + c] = 0;
    }
  }
  __syncthreads();
  // blocks below the diagonal, by distance d from it: T_ij = -T_ii sum_{m = j .. i-1} A_im T_mj, i = j + d
#pragma unroll
  for (int d = 1; d < 4; ++d) {
    const int j = wave, i = wave + d;
    if (i < 4) {
      f32x4_t m0 = {0.0f, 0.0f, 0.0f, 0.0f}, m1 = {0.0f, 0.0f, 0.0f, 0.0f};      // two chains of dependent MFMAs
      for (int m = j; m < i; ++m)
#pragma unroll
        for (int q = 0; q < 4; q += 2) {
          m0 = __builtin_amdgcn_mfma_f32_16x16x4f32(am[16 * i + c][16 * m + 4 * q + g], tm[16 * m + 4 * q + g][16 * j + c], m0, 0,
                                                     0, 0);
          m1 = __builtin_amdgcn_mfma_f32_16x16x4f32(am[16 * i + c][16 * m + 4 * q + 4 + g], tm[16 * m + 4 * q + 4 + g][16 * j + c],
                                                     m1, 0, 0, 0);
        }
      const f32x4_t macc = m0 + m1;
      // second product with the accumulators as the B operand: contraction slot (q, g) <-> k = 4 g + q
      f32x4_t res = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int q = 0; q < 4; ++q)
        res = __builtin_amdgcn_mfma_f32_16x16x4f32(tm[16 * i + c][16 * i + 4 * g + q], macc[q], res, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        tm[16 * i + 4 * g + r][16 * j + c] = -res[r];
        tb[16 * i + 4 * g + r][16 * j + c] = f32_to_bf16(-res[r]);
      }
    }
    __syncthreads();
  }
}

// Grid (n_heads, B).
//   qkv   bf16 [B*L, ld_qkv] after conv + SiLU: q of head h at q_col + NS h, k at k_col + NS h, v at v_col + 64 h
//   proj  bf16 [B*L, ld_p]: z of head h at columns 64 h, the beta logit at b_col + h, the decay logit at a_col + h
//   s_in / s_out f32 [B][H][NS][64] (S^T: [d_k][d_v]) or NULL;   y bf16 [B*L, ld_y]: RMSNorm_head(o) * norm_w * SiLU(z)
// Grid (n_heads, B * n_seg).  CARRY: the carry pass (no queries, no outputs; segments before the last):
//   carry_z f32 [B][H][n_seg][NS][64] <- Z^T, carry_m f32 [B][H][n_seg][NS][NS] <- [n][j] = Phi[j][n].
// Main pass with n_seg > 1: segment `seg` starts from s_start f32 [B][H][n_seg][NS][64].
template <int NS, bool CARRY>
__global__ __launch_bounds__(256, 1) void gdn_kernel(const bf16_t *__restrict__ qkv, int64_t ld_qkv, int q_col, int k_col,
                                                     int v_col, const bf16_t *__restrict__ proj, int64_t ld_p, int b_col,
                                                     int a_col, const float *__restrict__ dt_bias,
                                                     const float *__restrict__ A_log, const float *__restrict__ norm_w,
                                                     float eps, int64_t L, int n_seg, int64_t seg_len,
                                                     float *__restrict__ carry_z, float *__restrict__ carry_m,
                                                     const float *__restrict__ s_start, const float *s_in, float *s_out,
                                                     bf16_t *__restrict__ y, int64_t ld_y) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  GdnSmem<NS> &sm = *reinterpret_cast<GdnSmem<NS> *>(smem_raw);
  constexpr int kNB = NS / 16, kKS = NS / 32;
  constexpr int kG = CARRY ? 1 + NS / 64 : 1;      // groups of 64 "value" columns: the state, and in the carry pass Phi
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  const int h = blockIdx.x, n_heads = gridDim.x;
  const int64_t b = blockIdx.y / n_seg;
  const int seg = static_cast<int>(blockIdx.y % n_seg);
  if (CARRY && seg == n_seg - 1) return;            // nobody needs the last segment's carry
  const int64_t ts = seg * seg_len, te = ts + seg_len < L ? ts + seg_len : L;
  const float rate = __expf(A_log[h]), bias = dt_bias[h];
  const bf16_t *qkv_b = qkv + b * L * ld_qkv;
  const bf16_t *proj_b = proj + b * L * ld_p;
  const float q_scale = rsqrtf(static_cast<float>(NS));

  // state: sacc[0][nb][r] = S^T[d_k index 16 nb + 4 g + r][d_v index 16 wave + c]; carry pass: groups 1.. hold
  // the columns 64 (grp - 1) + 16 wave + c of the transition's transpose, starting from the identity
  f32x4_t sacc[kG][kNB];
  const int64_t s_stride = static_cast<int64_t>(NS) * kV;
  const int64_t unit = (b * n_heads + h) * n_seg + seg;
#pragma unroll
  for (int grp = 0; grp < kG; ++grp)
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        sacc[grp][nb][r] = (grp > 0 && 16 * nb + 4 * g + r == 64 * (grp - 1) + 16 * wave + c) ? 1.0f : 0.0f;
  if (!CARRY) {
    const float *sp = n_seg > 1 ? s_start + unit * s_stride : (s_in ? s_in + (b * n_heads + h) * s_stride : nullptr);
    if (sp) {
      sp += wave * 16 + c;
#pragma unroll
      for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) sacc[0][nb][r] = sp[(16 * nb + 4 * g + r) * kV];
    }
  }

  // roles while a chunk is parked: threads [0, NS) keys (8 x 8 blocks), the next 64 values; all: queries
  const bool is_k = tid < NS;
  const bool is_v = tid >= NS && tid < NS + 64;
  const int lt = is_k ? tid : tid - NS;
  const int n_co = is_k ? NS / 8 : kV / 8;
  const int so = lt / n_co, co = lt % n_co;
  const int so_phys = so ^ (co & 7);
  const int t_col = is_k ? k_col + h * NS + 8 * co : v_col + h * kV + 8 * co;
  const int e_row = tid >> 3, e_po = tid & 7;

  // A chunk's inputs are requested one chunk ahead (rows beyond the end: the last valid row, zeroed
  // when parked): what the parking needs right after the chunk before has been parked, the gate rows
  // after the chunk before has been stored.
  u32x4_t pv[8], pq[NS / 32], ez[2];
  unsigned short p_b = 0, p_a = 0;
  auto fetch_main = [&](int64_t t0) {
    if (t0 >= te) return;
    const bf16_t *row = proj_b + (t0 + lane < te ? t0 + lane : te - 1) * ld_p;
    p_b = row[b_col + h];
    p_a = row[a_col + h];
    if (is_k || is_v) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int64_t t = t0 + 8 * so + i;
        pv[i] = *reinterpret_cast<const u32x4_t *>(qkv_b + (t < te ? t : te - 1) * ld_qkv + t_col);
      }
    }
    if (!CARRY) {
#pragma unroll
      for (int i = 0; i < NS / 32; ++i) {
        const int piece = tid + 256 * i;
        const int64_t t = t0 + piece / (NS / 8);
        pq[i] = *reinterpret_cast<const u32x4_t *>(qkv_b + (t < te ? t : te - 1) * ld_qkv + q_col + h * NS + 8 * (piece % (NS / 8)));
      }
    }
  };
  auto fetch_out = [&](int64_t t0) {
    if (CARRY || t0 >= te) return;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int64_t t = t0 + e_row + 32 * i;
      ez[i] = *reinterpret_cast<const u32x4_t *>(proj_b + (t < te ? t : te - 1) * ld_p + h * kV + 8 * e_po);
    }
  };
  fetch_main(ts);
  fetch_out(ts);

  for (int64_t t0 = ts; t0 < te; t0 += kQ) {
    // The lane's coordinates go through an opaque copy every chunk: with them loop-invariant the compiler
    // hoists some two hundred addresses and mask predicates out of the loop and spills them.
    const int gq = opaque(g), cq = opaque(c);
    const int soq = opaque(so), coq = opaque(co), sopq = soq ^ (coq & 7), erq = opaque(e_row), epq = opaque(e_po);
    // per step: beta, log decay, cumulative log decay (every wavefront for itself, one step per lane)
    float beta = 0.0f, gl = 0.0f;
    if (t0 + lane < te) {
      beta = fast_rcp(1.0f + __expf(-bf16_to_f32(p_b)));
      gl = -rate * softplus_f32(bf16_to_f32(p_a) + bias);
    }
    const float cum = wave_inclusive_sum(gl);
    const float cum_last = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cum), 63));

    __syncthreads();                // the chunk before this one is done with the LDS
    if (is_k || is_v) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (t0 + 8 * soq + i >= te) pv[i] = u32x4_t{0u, 0u, 0u, 0u};
      if (is_k) {
        // row norms: the n_co lanes with this `soq` hold the eight steps' other column blocks
        const float w_lane = fast_exp2((cum_last - cum) * kLog2e);
        // a row at a time (normalised copy out, decay-weighted copy kept packed), then the packed rows are
        // transposed by byte permutes: few values live at once
        u32x4_t kw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float rk = rsqrtf(group_sum<NS / 8>(sum_sq8(pv[i])) + kL2Eps);
          *reinterpret_cast<u32x4_t *>(&sm.u.in.kn[8 * soq + i][8 * coq]) = scale8(pv[i], rk);
          kw[i] = scale8(pv[i], rk * __shfl(w_lane, 8 * soq + i));
        }
        park_8x8<kQ + 8>(kw, sm.kw_t, 8 * coq, 8 * sopq);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4_t *>(&sm.vt[8 * soq + i][8 * coq]) = pv[i];
      }
    }
    if (!CARRY) {
#pragma unroll
      for (int i = 0; i < NS / 32; ++i) {           // queries: 64 rows of NS / 8 pieces, raw; their norms
        const int piece = tid + 256 * i;
        const int row = piece / (NS / 8), oc = piece % (NS / 8);
        u32x4_t v = pq[i];
        if (t0 + row >= te) v = u32x4_t{0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4_t *>(&sm.u.in.qr[row][8 * oc]) = v;
        const float ss = group_sum<NS / 8>(sum_sq8(v));
        if (oc == 0) sm.rq[row] = rsqrtf(ss + kL2Eps) * q_scale;
      }
    }
    if (wave == 3) {
      sm.cum[lane] = cum;
      sm.ecum[lane] = fast_exp2(cum * kLog2e);
      sm.beta[lane] = beta;
    }
    __syncthreads();
    fetch_main(t0 + kQ);

    // ---- scores of this wavefront's 16 steps t = 16 wave + cq against all s (computed transposed),
    //      and the two products with the state the chunk starts from
    {
      const float cum_t = sm.cum[16 * wave + cq], beta_t = sm.beta[16 * wave + cq];
#pragma unroll
      for (int sb = 0; sb < 4; ++sb) {
        f32x4_t kk = {0.0f, 0.0f, 0.0f, 0.0f}, qk = {0.0f, 0.0f, 0.0f, 0.0f};
        if (sb <= wave) {
#pragma unroll
          for (int ks = 0; ks < kKS; ++ks) {
            const bf16x8_t fa = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.u.in.kn[16 * sb + cq][32 * ks + 8 * gq]));
            const bf16x8_t fk = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.u.in.kn[16 * wave + cq][32 * ks + 8 * gq]));
            kk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fk, kk, 0, 0, 0);
            if (!CARRY) {
              const bf16x8_t fq = as_frag(*reinterpret_cast<const u32x4_t *>(&sm.u.in.qr[16 * wave + cq][32 * ks + 8 * gq]));
              qk = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fq, qk, 0, 0, 0);
            }
          }
        }
        const f32x4_t cum_s = *reinterpret_cast<const f32x4_t *>(&sm.cum[16 * sb + 4 * gq]);
        f32x4_t av;
        float gv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int s = 16 * sb + 4 * gq + r, t = 16 * wave + cq;
          const float dec = s <= t ? fast_exp2((cum_t - cum_s[r]) * kLog2e) : 0.0f;
          av[r] = s < t ? beta_t * dec * kk[r] : 0.0f;
          gv[r] = dec * qk[r];
        }
        *reinterpret_cast<f32x4_t *>(&sm.a.am[16 * wave + cq][16 * sb + 4 * gq]) = av;
        if (!CARRY) {
          const u32x2_t packed = {pack_bf16x2(gv[0], gv[1]), pack_bf16x2(gv[2], gv[3])};
          *reinterpret_cast<u32x2_t *>(&sm.gs[16 * wave + cq][16 * sb + 4 * gq]) = packed;
        }
      }
    }
    bf16x8_t sop[kG][kKS];
#pragma unroll
    for (int grp = 0; grp < kG; ++grp)
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) sop[grp][ks] = frag_from_acc(sacc[grp][2 * ks], sacc[grp][2 * ks + 1]);
    f32x4_t rhs[kG][4], oacc[4];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
      f32x4_t pacc[kG];
#pragma unroll
      for (int grp = 0; grp < kG; ++grp) pacc[grp] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
      oacc[tb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int ks = 0; ks < kKS; ++ks) {
        const bf16x8_t fk = frag_perm<NS + 8>(sm.u.in.kn, 16 * tb + cq, 32 * ks, gq);
#pragma unroll
        for (int grp = 0; grp < kG; ++grp) pacc[grp] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fk, sop[grp][ks], pacc[grp], 0, 0, 0);
        if (!CARRY)
          oacc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag_perm<NS + 8>(sm.u.in.qr, 16 * tb + cq, 32 * ks, gq), sop[0][ks],
                                                             oacc[tb], 0, 0, 0);
      }
      const f32x4_t e = *reinterpret_cast<const f32x4_t *>(&sm.ecum[16 * tb + 4 * gq]);
      const f32x4_t bt = *reinterpret_cast<const f32x4_t *>(&sm.beta[16 * tb + 4 * gq]);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float vv = bf16_to_f32(sm.vt[16 * tb + 4 * gq + r][16 * wave + cq]);
        rhs[0][tb][r] = bt[r] * (vv - e[r] * pacc[0][r]);    // beta_t (v_t - gamma_t S_0 k_t)
#pragma unroll
        for (int grp = 1; grp < kG; ++grp) rhs[grp][tb][r] = -bt[r] * e[r] * pacc[grp][r];      // the same with v = 0
        oacc[tb][r] *= e[r];                                  // gamma_t S_0 q_t
      }
    }
    __syncthreads();                // A is complete; the step-major keys and queries are no longer read

    invert_unit_lower(sm.a.am, sm.u.tm, sm.tb, opaque(lane), wave);

    // ---- U = T rhs (rows t, this wavefront's 16 value channels); the contraction runs over steps,
    //      with rhs taken from the accumulators
    f32x4_t uacc[kG][4];
    {
      bf16x8_t rop[kG][2];
#pragma unroll
      for (int grp = 0; grp < kG; ++grp)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) rop[grp][k2] = frag_from_acc(rhs[grp][2 * k2], rhs[grp][2 * k2 + 1]);
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
#pragma unroll
        for (int grp = 0; grp < kG; ++grp) uacc[grp][tb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
          if (k2 == 0 || tb >= 2) {
            const bf16x8_t ft = frag_perm<kQ + 8>(sm.tb, 16 * tb + cq, 32 * k2, gq);
#pragma unroll
            for (int grp = 0; grp < kG; ++grp)
              uacc[grp][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ft, rop[grp][k2], uacc[grp][tb], 0, 0, 0);
          }
      }
    }
    bf16x8_t uop[kG][2];
#pragma unroll
    for (int grp = 0; grp < kG; ++grp)
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) uop[grp][k2] = frag_from_acc(uacc[grp][2 * k2], uacc[grp][2 * k2 + 1]);
    if (!CARRY) {
      // inside the chunk: O[t] += sum_{s <= t} exp(cum_t - cum_s) (q_t . k_s) u_s
#pragma unroll
      for (int tb = 0; tb < 4; ++tb)
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2)
          if (k2 == 0 || tb >= 2)
            oacc[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(frag_perm<kQ + 8>(sm.gs, 16 * tb + cq, 32 * k2, gq), uop[0][k2],
                                                               oacc[tb], 0, 0, 0);
    }
    // state at the chunk's end: S^T = gamma_64 S^T + sum_s (exp(cum_64 - cum_s) k_s) u_s^T
    {
      const float dec = fast_exp2(cum_last * kLog2e);
#pragma unroll
      for (int nb = 0; nb < kNB; ++nb) {
#pragma unroll
        for (int grp = 0; grp < kG; ++grp)
#pragma unroll
          for (int r = 0; r < 4; ++r) sacc[grp][nb][r] *= dec;
        const int row = 16 * nb + cq, sw = (row >> 3) & 7;
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          // steps 32 k2 + 4 gq .. +3 and 32 k2 + 16 + 4 gq .. +3 of the swizzled channel-major array
          const int p_lo = (4 * k2 + (gq >> 1)) ^ sw, p_hi = (4 * k2 + 2 + (gq >> 1)) ^ sw;
          const u32x2_t lo = *reinterpret_cast<const u32x2_t *>(&sm.kw_t[row][8 * p_lo + 4 * (gq & 1)]);
          const u32x2_t hi = *reinterpret_cast<const u32x2_t *>(&sm.kw_t[row][8 * p_hi + 4 * (gq & 1)]);
          const bf16x8_t fw = frag_from_halves(lo, hi);
#pragma unroll
          for (int grp = 0; grp < kG; ++grp)
            sacc[grp][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw, uop[grp][k2], sacc[grp][nb], 0, 0, 0);
        }
      }
    }
    if (CARRY) continue;
    // ---- output rows: query norm and scale, RMS norm over the head's 64 channels, SiLU(z) gate
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
      const f32x4_t rq = *reinterpret_cast<const f32x4_t *>(&sm.rq[16 * tb + 4 * gq]);
#pragma unroll
      for (int r = 0; r < 4; ++r) sm.a.y[16 * tb + 4 * gq + r][16 * wave + cq] = oacc[tb][r] * rq[r];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = erq + 32 * i;
      const int64_t t = t0 + row;
      const f32x4_t y0 = *reinterpret_cast<const f32x4_t *>(&sm.a.y[row][8 * epq]);
      const f32x4_t y1 = *reinterpret_cast<const f32x4_t *>(&sm.a.y[row][8 * epq + 4]);
      float ss = 0.0f;
#pragma unroll
      for (int m = 0; m < 4; ++m) ss = fmaf(y0[m], y0[m], fmaf(y1[m], y1[m], ss));
      const float rstd = rsqrtf(group_sum<8>(ss) * (1.0f / kV) + eps);
      const u32x4_t zv = ez[i];
      const f32x4_t w0 = *reinterpret_cast<const f32x4_t *>(norm_w + 8 * epq);
      const f32x4_t w1 = *reinterpret_cast<const f32x4_t *>(norm_w + 8 * epq + 4);
      float o[8];
#pragma unroll
      for (int m = 0; m < 8; ++m)
        o[m] = (m < 4 ? y0[m & 3] * w0[m & 3] : y1[m & 3] * w1[m & 3]) * rstd * silu_f32(bf16_elem(zv, m));
      const u32x4_t ov = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])};
      if (t < te) *reinterpret_cast<u32x4_t *>(y + (b * L + t) * ld_y + h * kV + 8 * epq) = ov;
    }
    fetch_out(t0 + kQ);
  }

  if (CARRY) {
    float *zp = carry_z + unit * s_stride + wave * 16 + c;
    float *mp = carry_m + unit * static_cast<int64_t>(NS) * NS + wave * 16 + c;
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        zp[(16 * nb + 4 * g + r) * kV] = sacc[0][nb][r];
#pragma unroll
        for (int grp = 1; grp < kG; ++grp) mp[(16 * nb + 4 * g + r) * NS + 64 * (grp - 1)] = sacc[grp][nb][r];
      }
  } else if (s_out && seg == n_seg - 1) {
    float *sp = s_out + (b * n_heads + h) * s_stride + wave * 16 + c;
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
      for (int r = 0; r < 4; ++r) sp[(16 * nb + 4 * g + r) * kV] = sacc[0][nb][r];
  }
}

// The state every segment starts from: start[0] = s_in (or 0), start[j + 1]^T = M_j start[j]^T + Z_j^T with the
// carry pass's arrays as stored (M_j[n][m] = Phi_j[m][n]).  Grid (n_heads, B); a thread owns NS / 4 columns of one row.
// Workgroup barrier for data that travels through LDS only: __syncthreads() also waits for the wave's
// outstanding global stores, a memory round trip behind every barrier that follows one (the fold stores a
// segment's start state right before it parks it)
__device__ __forceinline__ void fold_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int NS>
__global__ __launch_bounds__(256) void gdn_fold_kernel(const float *__restrict__ carry_z, const float *__restrict__ carry_m,
                                                       const float *__restrict__ s_in, float *__restrict__ s_start,
                                                       int n_seg) {
  constexpr int kCols = NS / 4, kPerRow = kV / kCols;       // columns per thread, threads per row
  __shared__ float cur[NS][kV + 1];
  const int tid = threadIdx.x, n = tid / kPerRow, v0 = (tid % kPerRow) * kCols;
  const int h = blockIdx.x, n_heads = gridDim.x;
  const int64_t bh = static_cast<int64_t>(blockIdx.y) * n_heads + h;
  const int64_t s_stride = static_cast<int64_t>(NS) * kV;
  float acc[kCols];
#pragma unroll
  for (int i = 0; i < kCols; ++i) acc[i] = s_in ? s_in[bh * s_stride + n * kV + v0 + i] : 0.0f;
  for (int j = 0; j < n_seg; ++j) {
    const int64_t unit = bh * n_seg + j;
#pragma unroll
    for (int i = 0; i < kCols; ++i) {
      s_start[unit * s_stride + n * kV + v0 + i] = acc[i];
      cur[n][v0 + i] = acc[i];
    }
    if (j == n_seg - 1) break;
    fold_barrier();
    const float *mrow = carry_m + unit * static_cast<int64_t>(NS) * NS + static_cast<int64_t>(n) * NS;
#pragma unroll
    for (int i = 0; i < kCols; ++i) acc[i] = carry_z[unit * s_stride + n * kV + v0 + i];
    // (the row of M in batches of 16 values, four 16-byte loads at a time: value by value the loop is a
    // chain of memory round trips)
    for (int m0 = 0; m0 < NS; m0 += 16) {
      float4 a4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) a4[q] = *reinterpret_cast<const float4 *>(mrow + m0 + 4 * q);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a[4] = {a4[q].x, a4[q].y, a4[q].z, a4[q].w};
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int i = 0; i < kCols; ++i) acc[i] = fmaf(a[r], cur[m0 + 4 * q + r][v0 + i], acc[i]);
      }
    }
    fold_barrier();
  }
}

// One step per sequence (L == 1): grid (n_heads, B); thread = (value channel v, quarter of the key channels).
// The state is read and written once, in rows of 64 consecutive value channels.
template <int NS>
__global__ __launch_bounds__(256) void gdn_step_kernel(const bf16_t *__restrict__ qkv, int64_t ld_qkv, int q_col, int k_col,
                                                       int v_col, const bf16_t *__restrict__ proj, int64_t ld_p, int b_col,
                                                       int a_col, const float *__restrict__ dt_bias,
                                                       const float *__restrict__ A_log, const float *__restrict__ norm_w,
                                                       float eps, const float *s_in, float *s_out, bf16_t *__restrict__ y,
                                                       int64_t ld_y) {
  __shared__ float kq[2][NS];          // normalised key, normalised and scaled query
  __shared__ float part[4][kV];
  __shared__ float red[2][4];
  const int tid = threadIdx.x, v = tid & 63, q4 = tid >> 6, lane = tid & 63;
  const int h = blockIdx.x, n_heads = gridDim.x;
  const int64_t b = blockIdx.y;
  const bf16_t *row = qkv + b * ld_qkv;
  const bf16_t *prow = proj + b * ld_p;
  // L2 norms of q and k: threads [0, NS) square a key element, threads [128, 128 + NS) a query element
  float kval = 0.0f, qval = 0.0f;
  if (tid < NS) kval = bf16_to_f32(row[k_col + h * NS + tid]);
  if (tid >= 128 && tid < 128 + NS) qval = bf16_to_f32(row[q_col + h * NS + tid - 128]);
  float sk = kval * kval, sq = qval * qval;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    sk += __shfl_xor(sk, off);
    sq += __shfl_xor(sq, off);
  }
  if (lane == 0) {
    red[0][q4] = sk;
    red[1][q4] = sq;
  }
  __syncthreads();
  const float rk = rsqrtf(red[0][0] + red[0][1] + red[0][2] + red[0][3] + kL2Eps);
  const float rq = rsqrtf(red[1][0] + red[1][1] + red[1][2] + red[1][3] + kL2Eps) * rsqrtf(static_cast<float>(NS));
  if (tid < NS) kq[0][tid] = kval * rk;
  if (tid >= 128 && tid < 128 + NS) kq[1][tid - 128] = qval * rq;
  __syncthreads();
  const float beta = fast_rcp(1.0f + __expf(-bf16_to_f32(prow[b_col + h])));
  const float alpha = __expf(-__expf(A_log[h]) * softplus_f32(bf16_to_f32(prow[a_col + h]) + dt_bias[h]));
  // this thread's state values: S^T[n][v] for its quarter of n
  constexpr int kPer = NS / 4;
  const int64_t base = (b * n_heads + h) * static_cast<int64_t>(NS) * kV + v;
  float st[kPer];
  float pred = 0.0f;
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    const int n = q4 * kPer + j;
    st[j] = alpha * (s_in ? s_in[base + static_cast<int64_t>(n) * kV] : 0.0f);
    pred = fmaf(st[j], kq[0][n], pred);
  }
  part[q4][v] = pred;
  __syncthreads();
  const float u = beta * (bf16_to_f32(row[v_col + h * kV + v]) - (part[0][v] + part[1][v] + part[2][v] + part[3][v]));
  __syncthreads();
  float o = 0.0f;
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    const int n = q4 * kPer + j;
    st[j] = fmaf(u, kq[0][n], st[j]);
    if (s_out) s_out[base + static_cast<int64_t>(n) * kV] = st[j];
    o = fmaf(st[j], kq[1][n], o);
  }
  part[q4][v] = o;
  __syncthreads();
  if (q4 == 0) {
    const float ov = part[0][v] + part[1][v] + part[2][v] + part[3][v];
    float ss = ov * ov;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    const float rstd = rsqrtf(ss * (1.0f / kV) + eps);
    y[b * ld_y + h * kV + v] = f32_to_bf16(ov * rstd * norm_w[v] * silu_f32(bf16_to_f32(prow[h * kV + v])));
  }
}

struct GdnPlanSeg {
  int n_seg;
  int64_t seg_len;
};
GdnPlanSeg gdn_plan(int64_t B, int64_t L, int n_heads) {
  // one workgroup for each of the 256 CUs; a segment is whole chunks and at least four of them
  const int64_t chunks = ceil_div(L, kQ);
  int64_t n_seg = ceil_div(256, B * n_heads);
  const int64_t max_seg = chunks / 4 > 0 ? chunks / 4 : 1;
  n_seg = n_seg < 1 ? 1 : (n_seg > max_seg ? max_seg : n_seg);
  GdnPlanSeg p;
  p.seg_len = ceil_div(chunks, n_seg) * kQ;
  p.n_seg = static_cast<int>(ceil_div(L, p.seg_len));
  return p;
}

template <int NS, bool CARRY>
hipError_t gdn_allow_lds() {
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
      e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gdn_kernel<NS, CARRY>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(sizeof(GdnSmem<NS>)));
      if (e != hipSuccess) return e;
      done[dev].store(true, std::memory_order_release);
    }
  }
  return hipSuccess;
}

template <int NS>
hipError_t gdn_dispatch(const bf16_t *qkv, int64_t ld_qkv, int q_col, int k_col, int v_col, const bf16_t *proj, int64_t ld_p,
                        int b_col, int a_col, const float *dt_bias, const float *A_log, const float *norm_w, float eps,
                        int64_t B, int64_t L, int n_heads, const float *s_in, float *s_out, float *carry, bf16_t *y,
                        int64_t ld_y, hipStream_t s) {
  if (L == 1) {
    hipLaunchKernelGGL((gdn_step_kernel<NS>), dim3(static_cast<unsigned>(n_heads), static_cast<unsigned>(B)), dim3(256), 0,
                       s, qkv, ld_qkv, q_col, k_col, v_col, proj, ld_p, b_col, a_col, dt_bias, A_log, norm_w, eps, s_in, s_out,
                       y, ld_y);
    return hipGetLastError();
  }
  const GdnPlanSeg p = gdn_plan(B, L, n_heads);
  const size_t units = static_cast<size_t>(B) * n_heads * p.n_seg;
  float *carry_z = carry, *carry_m = carry + units * NS * kV, *s_start = carry_m + units * NS * NS;
  const dim3 grid(static_cast<unsigned>(n_heads), static_cast<unsigned>(B * p.n_seg));
  hipError_t e;
  if (p.n_seg > 1) {
    if ((e = gdn_allow_lds<NS, true>()) != hipSuccess) return e;
    hipLaunchKernelGGL((gdn_kernel<NS, true>), grid, dim3(256), sizeof(GdnSmem<NS>), s, qkv, ld_qkv, q_col, k_col, v_col, proj,
                       ld_p, b_col, a_col, dt_bias, A_log, norm_w, eps, L, p.n_seg, p.seg_len, carry_z, carry_m, s_start, s_in,
                       s_out, y, ld_y);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL((gdn_fold_kernel<NS>), dim3(static_cast<unsigned>(n_heads), static_cast<unsigned>(B)), dim3(256), 0, s,
                       carry_z, carry_m, s_in, s_start, p.n_seg);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if ((e = gdn_allow_lds<NS, false>()) != hipSuccess) return e;
  hipLaunchKernelGGL((gdn_kernel<NS, false>), grid, dim3(256), sizeof(GdnSmem<NS>), s, qkv, ld_qkv, q_col, k_col, v_col, proj,
                     ld_p, b_col, a_col, dt_bias, A_log, norm_w, eps, L, p.n_seg, p.seg_len, carry_z, carry_m, s_start, s_in,
                     s_out, y, ld_y);
  return hipGetLastError();
}

}  // namespace

bool gdn_supported(int d_k, int d_v) { return d_v == kV && (d_k == 64 || d_k == 128); }

size_t gdn_carry_bytes(int64_t B, int64_t L, int n_heads, int d_k) {
  const GdnPlanSeg p = gdn_plan(B, L, n_heads);
  if (p.n_seg <= 1) return 0;
  return static_cast<size_t>(B) * n_heads * p.n_seg * (2 * static_cast<size_t>(d_k) * kV + static_cast<size_t>(d_k) * d_k) *
         sizeof(float);
}

hipError_t launch_gdn_scan(const void *qkv, int64_t ld_qkv, int q_col, int k_col, int v_col, const void *proj, int64_t ld_p,
                           int b_col, int a_col, const float *dt_bias, const float *A_log, const float *norm_w, float eps,
                           int64_t B, int64_t L, int n_heads, int d_k, const float *s_in, float *s_out, float *carry,
                           void *y, int64_t ld_y, hipStream_t s) {
  if (B * L <= 0) return hipSuccess;
  if (B * gdn_plan(B, L, n_heads).n_seg > 65535) return hipErrorInvalidValue;
  const bf16_t *qp = static_cast<const bf16_t *>(qkv), *pp = static_cast<const bf16_t *>(proj);
  if (d_k == 128)
    return gdn_dispatch<128>(qp, ld_qkv, q_col, k_col, v_col, pp, ld_p, b_col, a_col, dt_bias, A_log, norm_w, eps, B, L,
                             n_heads, s_in, s_out, carry, static_cast<bf16_t *>(y), ld_y, s);
  if (d_k == 64)
    return gdn_dispatch<64>(qp, ld_qkv, q_col, k_col, v_col, pp, ld_p, b_col, a_col, dt_bias, A_log, norm_w, eps, B, L, n_heads,
                            s_in, s_out, carry, static_cast<bf16_t *>(y), ld_y, s);
  return hipErrorInvalidValue;
}

}  // namespace rom
