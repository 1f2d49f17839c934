// Device-side helpers of libbct: 16-byte vector access, storage-dtype
// conversion and wavefront (64-lane) reductions for gfx950.
#ifndef BCT_DEVICE_H
#define BCT_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bct {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct F32 {
  typedef float elem;
  static constexpr int kElemsPerVec = 4;  // elements in one 16-byte vector
};
struct BF16 {
  typedef uint16_t elem;
  static constexpr int kElemsPerVec = 8;
};

// 16 bytes of storage -> E floats (exact widening).
template <typename DT>
__device__ __forceinline__ void unpack16(const u32x4 v, float* f);

template <>
__device__ __forceinline__ void unpack16<F32>(const u32x4 v, float* f) {
  f[0] = __uint_as_float(v.x);
  f[1] = __uint_as_float(v.y);
  f[2] = __uint_as_float(v.z);
  f[3] = __uint_as_float(v.w);
}
template <>
__device__ __forceinline__ void unpack16<BF16>(const u32x4 v, float* f) {
  f[0] = __uint_as_float(v.x << 16);
  f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16);
  f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16);
  f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16);
  f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

// Two floats -> two bf16 in one word, round-to-nearest-even (the hardware
// conversion of gfx950: v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 r;
  r.x = (__bf16)lo;
  r.y = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, r);
}

// E floats -> 16 bytes of storage, rounding to the storage dtype; the floats
// are overwritten with the stored (rounded) values so that a later read uses
// exactly what the cache now holds.
template <typename DT>
__device__ __forceinline__ u32x4 pack16_round(float* f);

template <>
__device__ __forceinline__ u32x4 pack16_round<F32>(float* f) {
  u32x4 v;
  v.x = __float_as_uint(f[0]);
  v.y = __float_as_uint(f[1]);
  v.z = __float_as_uint(f[2]);
  v.w = __float_as_uint(f[3]);
  return v;
}
template <>
__device__ __forceinline__ u32x4 pack16_round<BF16>(float* f) {
  u32x4 v;
  v.x = pack_bf16x2(f[0], f[1]);
  v.y = pack_bf16x2(f[2], f[3]);
  v.z = pack_bf16x2(f[4], f[5]);
  v.w = pack_bf16x2(f[6], f[7]);
  unpack16<BF16>(v, f);
  return v;
}

// One float -> storage element (used by the small epilogues).
__device__ __forceinline__ void store_elem(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_elem(uint16_t* p, size_t i, float v) {
  p[i] = __builtin_bit_cast(uint16_t, (__bf16)v);
}
__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, size_t i) {
  return __uint_as_float((uint32_t)p[i] << 16);
}

// The memory a workgroup of a unit_grid launch works on (see bct_internal.h).
__device__ __forceinline__ uint32_t block_unit() { return blockIdx.z * 32768u + blockIdx.y; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Butterfly reductions over the lanes whose ids differ in the bits of `mask`
// (a contiguous range of bits given as lowest and highest xor distance).
// The butterfly visits partners in a fixed order, so results are reproducible.
//
// A butterfly that starts at distance 1 takes its partners at distances 1, 2, 4 and 8 through the
// data-parallel-primitive path of the vector ALU (no trip through the LDS crossbar that a general
// lane exchange makes): distances 1 and 2 are quad permutations; at distance 4 every quad already
// holds one value, so the lane 7 - i of the half row (row_half_mirror) holds what lane i ^ 4 holds,
// and at distance 8 the lane 15 - i of the row (row_mirror) holds what lane i ^ 8 holds.  Same
// operands in the same order as the plain butterfly, so the same bits.
template <int CTRL>
__device__ __forceinline__ float dpp_partner(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int LO, int O>
__device__ __forceinline__ float xor_partner(float v) {
  if constexpr (LO == 1 && O == 1) return dpp_partner<0xB1>(v);        // quad_perm [1, 0, 3, 2]
  else if constexpr (LO == 1 && O == 2) return dpp_partner<0x4E>(v);   // quad_perm [2, 3, 0, 1]
  else if constexpr (LO == 1 && O == 4) return dpp_partner<0x141>(v);  // row_half_mirror
  else if constexpr (LO == 1 && O == 8) return dpp_partner<0x140>(v);  // row_mirror
  else return __shfl_xor(v, O, 64);
}
template <int LO, int HI>
__device__ __forceinline__ float xor_sum(float v) {
  v += xor_partner<LO, LO>(v);
  if constexpr (2 * LO <= HI) v += xor_partner<LO, 2 * LO>(v);
  if constexpr (4 * LO <= HI) v += xor_partner<LO, 4 * LO>(v);
  if constexpr (8 * LO <= HI) v += xor_partner<LO, 8 * LO>(v);
  if constexpr (16 * LO <= HI) v += xor_partner<LO, 16 * LO>(v);
  if constexpr (32 * LO <= HI) v += xor_partner<LO, 32 * LO>(v);
  return v;
}
template <int LO, int HI>
__device__ __forceinline__ float xor_max(float v) {
  v = fmaxf(v, xor_partner<LO, LO>(v));
  if constexpr (2 * LO <= HI) v = fmaxf(v, xor_partner<LO, 2 * LO>(v));
  if constexpr (4 * LO <= HI) v = fmaxf(v, xor_partner<LO, 4 * LO>(v));
  if constexpr (8 * LO <= HI) v = fmaxf(v, xor_partner<LO, 8 * LO>(v));
  if constexpr (16 * LO <= HI) v = fmaxf(v, xor_partner<LO, 16 * LO>(v));
  if constexpr (32 * LO <= HI) v = fmaxf(v, xor_partner<LO, 32 * LO>(v));
  return v;
}

// One wavefront merges the per-tile (max, sum of exp2(score - max)) pairs of a row, up to 128 of them (lane l
// takes tiles l and l + 64), into the row's (max, sum).  The operations and their order are those of
// normalise_kernel, so both give the same bits.
struct TileStats {
  float2 a, c;
};
__device__ __forceinline__ TileStats load_tile_stats(const float2* st, uint32_t n_tiles, uint32_t lane) {
  TileStats t = {make_float2(-INFINITY, 0.f), make_float2(-INFINITY, 0.f)};
  if (lane < n_tiles) t.a = st[lane];
  if (lane + 64 < n_tiles) t.c = st[lane + 64];
  return t;
}
__device__ __forceinline__ float2 merge_tile_stats(const TileStats& t) {
  const float mx = xor_max<1, 32>(fmaxf(t.a.x, t.c.x));
  float sm = t.a.y * fast_exp2(t.a.x - mx);
  sm += t.c.y * fast_exp2(t.c.x - mx);
  return make_float2(mx, xor_sum<1, 32>(sm));
}
__device__ __forceinline__ float2 merge_tile_stats(const float2* st, uint32_t n_tiles, uint32_t lane) {
  return merge_tile_stats(load_tile_stats(st, n_tiles, lane));
}
constexpr uint32_t kMaxMergedTiles = 128;

}  // namespace bct

#endif
