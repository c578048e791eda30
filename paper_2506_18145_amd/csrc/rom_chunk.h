// Device helpers shared by the chunked recurrences on the matrix cores (rom_mamba2.hip, rom_gdn.hip):
// packed-bf16 access, the wavefront prefix sum, 8 x 8 block transposes into LDS, MFMA operand fragments.
// gfx950 only.
#pragma once

#include "rom_internal.h"

namespace rom {
namespace chunk {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kQ = 64;          // steps per chunk
constexpr float kLog2e = 1.44269504088896341f;

__device__ __forceinline__ float softplus_f32(float v) { return v > 20.0f ? v : log1pf(__expf(v)); }

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or_zero(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
// inclusive prefix sum over the 64 lanes (row shifts, then lane 15 / 31 broadcasts)
__device__ __forceinline__ float wave_inclusive_sum(float v) {
  v += dpp_or_zero<0x111, 0xF>(v);
  v += dpp_or_zero<0x112, 0xF>(v);
  v += dpp_or_zero<0x114, 0xF>(v);
  v += dpp_or_zero<0x118, 0xF>(v);
  v += dpp_or_zero<0x142, 0xA>(v);
  v += dpp_or_zero<0x143, 0xC>(v);
  return v;
}

// A copy the compiler cannot see through: values derived from it are recomputed where they are used
// instead of being hoisted out of a loop (and spilled) as loop invariants.
__device__ __forceinline__ int opaque(int v) {
  asm volatile("" : "+v"(v));
  return v;
}

__device__ __forceinline__ float bf16_elem(const u32x4_t &v, int m) {
  const unsigned int w = v[m >> 1];
  return __uint_as_float((m & 1) ? (w & 0xFFFF0000u) : (w << 16));
}
// eight packed bf16 values times f
__device__ __forceinline__ u32x4_t scale8(const u32x4_t &v, float f) {
  u32x4_t o;
#pragma unroll
  for (int a = 0; a < 4; ++a) o[a] = pack_bf16x2(f * bf16_elem(v, 2 * a), f * bf16_elem(v, 2 * a + 1));
  return o;
}
// Eight 16-byte pieces (eight consecutive columns of eight consecutive steps), step i scaled by f[i],
// to LDS column-major: for each of the eight columns the eight steps as one 16-byte row segment.
template <int PITCH>
__device__ __forceinline__ void park_scaled_8x8(const u32x4_t (&v)[8], const float (&f)[8], bf16_t (*dst)[PITCH], int col0,
                                                int step0) {
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    u32x4_t seg;
#pragma unroll
    for (int a = 0; a < 4; ++a)
      seg[a] = pack_bf16x2(f[2 * a] * bf16_elem(v[2 * a], m), f[2 * a + 1] * bf16_elem(v[2 * a + 1], m));
    *reinterpret_cast<u32x4_t *>(&dst[col0 + m][step0]) = seg;
  }
}

// eight 16-byte pieces (8 columns of 8 steps) -> column-major 16-byte segments: word a of column m's
// segment holds steps 2a, 2a+1, which v_perm_b32 picks out of word m/2 of the two step rows
template <int PITCH>
__device__ __forceinline__ void park_8x8(const u32x4_t (&v)[8], bf16_t (*dst)[PITCH], int col0, int step0) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {          // word w of a piece = columns 2w, 2w+1
    u32x4_t lo, hi;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const unsigned int p0 = v[2 * a][w], p1 = v[2 * a + 1][w];
      lo[a] = __builtin_amdgcn_perm(p1, p0, 0x05040100u);      // (p0.lo16, p1.lo16)
      hi[a] = __builtin_amdgcn_perm(p1, p0, 0x07060302u);      // (p0.hi16, p1.hi16)
    }
    *reinterpret_cast<u32x4_t *>(&dst[col0 + 2 * w][step0]) = lo;
    *reinterpret_cast<u32x4_t *>(&dst[col0 + 2 * w + 1][step0]) = hi;
  }
}

__device__ __forceinline__ bf16x8_t as_frag(const u32x4_t &v) { return __builtin_bit_cast(bf16x8_t, v); }
__device__ __forceinline__ bf16x8_t frag_from_halves(const u32x2_t &lo, const u32x2_t &hi) {
  const u32x4_t v = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8_t, v);
}
// two accumulator quads (rows 4g.. of two consecutive 16-row blocks) as the B operand of a 32-wide step
__device__ __forceinline__ bf16x8_t frag_from_acc(const f32x4_t &lo, const f32x4_t &hi) {
  const u32x4_t v = {pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]), pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])};
  return __builtin_bit_cast(bf16x8_t, v);
}
// the matching A operand: row `row` of a step-major bf16 array, columns base + 4g .. and base + 16 + 4g ..
template <int PITCH>
__device__ __forceinline__ bf16x8_t frag_perm(const bf16_t (*src)[PITCH], int row, int base, int g) {
  const u32x2_t lo = *reinterpret_cast<const u32x2_t *>(&src[row][base + 4 * g]);
  const u32x2_t hi = *reinterpret_cast<const u32x2_t *>(&src[row][base + 16 + 4 * g]);
  return frag_from_halves(lo, hi);
}

}  // namespace chunk
}  // namespace rom
