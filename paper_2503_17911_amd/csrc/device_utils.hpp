// Wave64 device helpers for gfx950: cross-lane reductions on DPP, the
// order-preserving key transform, and the code-row dot product.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ann {

__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }

// DPP controls (GFX9 encoding).
constexpr int kDppQuadXor1 = 0xB1;     // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;     // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}

__device__ __forceinline__ int xor_lane_i32(int v, int mask) {
  return __builtin_amdgcn_ds_bpermute((lane_id() ^ mask) << 2, v);
}

// Sum over aligned groups of W consecutive lanes; every lane of the group
// ends with the group's total.  W in {1,2,4,8,16,32,64}.
template <int W>
__device__ __forceinline__ int group_sum_i32(int v) {
  if constexpr (W >= 2) v += dpp_i32<kDppQuadXor1>(v);
  if constexpr (W >= 4) v += dpp_i32<kDppQuadXor2>(v);
  if constexpr (W >= 8) v += dpp_i32<kDppRowHalfMirror>(v);
  if constexpr (W >= 16) v += dpp_i32<kDppRowMirror>(v);
  if constexpr (W >= 32) v += xor_lane_i32(v, 16);
  if constexpr (W >= 64) v += xor_lane_i32(v, 32);
  return v;
}

// Inclusive prefix sum over the 64 lanes (row shifts inside each row of 16
// lanes, then the row totals are broadcast to the rows that follow).
__device__ __forceinline__ int wave_inclusive_scan_i32(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

__device__ __forceinline__ double xor_lane_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = xor_lane_i32(lo, mask);
  hi = xor_lane_i32(hi, mask);
  return __hiloint2double(hi, lo);
}

template <int W>
__device__ __forceinline__ double group_sum_f64(double v) {
#pragma unroll
  for (int m = 1; m < W; m <<= 1) v += xor_lane_f64(v, m);
  return v;
}

__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v = fmaxf(v, __int_as_float(xor_lane_i32(__float_as_int(v), m)));
  return v;
}

// fp32 -> uint32 such that unsigned order equals numeric order (no NaN).
__device__ __forceinline__ uint32_t order_u32(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unorder_f32(uint32_t u) {
  return __uint_as_float((u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u);
}

// Traversal key from the integer dot product (paper Section 5.2: squared L2 as
// stored norm minus twice the inner product; the per-query ||q||^2 is left out).
// Written with explicit roundings so that it is one multiply (exact), one
// subtract and one fused multiply-add, whatever the compiler's contraction mode.
__device__ __forceinline__ float key_from_idot(uint32_t metric, float s, float qlo, int idot, float norm_term) {
  float key;
  if (metric == ANN_L2) {
    float h = __fsub_rn(norm_term, __fmul_rn(2.0f, qlo));
    key = __fmaf_rn(__fmul_rn(-2.0f, s), (float)idot, h);
  } else {
    key = -__fmaf_rn(s, (float)idot, qlo);
  }
  uint32_t b = __float_as_uint(key);
  if ((b & 0x7FFFFFFFu) == 0) b = 0;  // -0 -> +0
  return __uint_as_float(b);
}

// The same for the 15-bit folded query, whose integer dot product arrives as
// two parts (query value = 128 * hi + lo): they are joined in 64 bits and
// converted to fp32 with one rounding.
__device__ __forceinline__ float key_from_idot15(uint32_t metric, float s, float qlo, int idot_hi, int idot_lo,
                                                 float norm_term) {
  const long long idot = (long long)idot_hi * 128 + (long long)idot_lo;
  const float f = __ll2float_rn(idot);
  float key;
  if (metric == ANN_L2) {
    float h = __fsub_rn(norm_term, __fmul_rn(2.0f, qlo));
    key = __fmaf_rn(__fmul_rn(-2.0f, s), f, h);
  } else {
    key = -__fmaf_rn(s, f, qlo);
  }
  uint32_t b = __float_as_uint(key);
  if ((b & 0x7FFFFFFFu) == 0) b = 0;
  return __uint_as_float(b);
}

// Partial integer dot product of one 16-byte code chunk with this lane's
// share of the folded query.
//   BITS == 8: the chunk holds 16 codes stored as (c ^ 0x80), i.e. c - 128 as
//              int8; tq[0..3] hold the 16 matching query bytes.
//   BITS == 4: the chunk holds 32 codes; tq[0..3] hold the query bytes of the
//              even dimensions (low nibbles), tq[4..7] those of the odd ones.
template <int BITS>
__device__ __forceinline__ int chunk_dot(const uint4 &c, const int *tq) {
  int acc = 0;
  if constexpr (BITS == 8) {
    acc = __builtin_amdgcn_sdot4(tq[0], (int)c.x, acc, false);
    acc = __builtin_amdgcn_sdot4(tq[1], (int)c.y, acc, false);
    acc = __builtin_amdgcn_sdot4(tq[2], (int)c.z, acc, false);
    acc = __builtin_amdgcn_sdot4(tq[3], (int)c.w, acc, false);
  } else {
    const uint32_t m = 0x0F0F0F0Fu;
    acc = __builtin_amdgcn_sdot4(tq[0], (int)(c.x & m), acc, false);
    acc = __builtin_amdgcn_sdot4(tq[4], (int)((c.x >> 4) & m), acc, false);
    acc = __builtin_amdgcn_sdot4(tq[1], (int)(c.y & m), acc, false);
    acc = __builtin_amdgcn_sdot4(tq[5], (int)((c.y >> 4) & m), acc, false);
    acc = __builtin_amdgcn_sdot4(tq[2], (int)(c.z & m), acc, false);
    acc = __builtin_amdgcn_sdot4(tq[6], (int)((c.z >> 4) & m), acc, false);
    acc = __builtin_amdgcn_sdot4(tq[3], (int)(c.w & m), acc, false);
    acc = __builtin_amdgcn_sdot4(tq[7], (int)((c.w >> 4) & m), acc, false);
  }
  return acc;
}

template <int BITS>
struct TqRegs {
  static constexpr int kWords = BITS == 8 ? 4 : 8;
};

}  // namespace ann
