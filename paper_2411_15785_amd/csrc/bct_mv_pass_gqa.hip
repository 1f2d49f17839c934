// The MV pass for several query heads per KV head (bf16, d = 128, G > 2; gfx950).
//
// The update of MV is the same read-modify-write stream as in bct_mv_pass.hip.
// What changes is the read: with G query heads the output is
//     out[g,:] = sum_m rw[g][m] * MV_new[m,:]          (G x M) . (M x d)
// and on the vector ALU that is G FMAs per element of MV: at G = 4 the pass is
// bound by those FMAs (and by every one of the 16 lanes of a slot row computing
// all G softmax weights again), not by memory.  Here the contraction over the
// wavefront's 32 slots runs on v_mfma_f32_16x16x32_bf16:
//   B operand = MV_new (exactly the bf16 values just stored): lane (sub, sl)
//     holds columns 8 sub .. 8 sub + 7 of the slots 8 sl .. 8 sl + 7; an in-lane
//     8 x 8 transpose of 16-bit elements turns its 8 row registers into 8
//     operands, operand e = column 8 sub + e for the lane's 8 slots: column
//     index of the MFMA = sub, contraction entries 8 (l / 16) + u = the slots;
//   A operand = the softmax weights: lane (sub, sl) computes the weights of ONE
//     query head, g = sub, for its 8 slots (lanes sub >= G hold zeros), split
//     into hi + lo bf16 parts (two MFMAs) so that the weights keep fp32 grade;
//   accumulator e of lane (sub, sl): out[g = 4 sl + v][column 8 sub + e].
// The MFMA also sums over the four lane groups, so no lane exchange is needed.
#include "bct_device.h"
#include "bct_internal.h"

namespace bct {

namespace {

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <bool WRITE, int BS, bool NORM, int U>
__global__ __launch_bounds__(BS) void mv_pass_gqa_kernel(const DecodeParams p) {
  constexpr int D = 128, NB = U / 8, NW = BS / 64, SPB = NW * 4 * U;   // a wavefront covers 4 U slots
  constexpr uint32_t W = WRITE ? 1u : 0u;
  __shared__ float s_red[NW * kMaxG * D];

  const uint32_t split = blockIdx.x, unit = block_unit();
  if (unit >= p.B * p.Hkv) return;
  const uint32_t b = unit / p.Hkv, h = unit % p.Hkv;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int sub = lane % 16, sl = lane / 16;
  const uint32_t R = p.R, G = p.G, M = p.M;

  // M is a multiple of 64: the 32 slots of a wavefront are all inside the memory or all outside
  const uint32_t slot0 = split * SPB + wave * (4 * U) + sl * U;
  const bool active = slot0 < M;
  uint16_t* mv = (uint16_t*)p.mv + ((size_t)unit * M + slot0) * D + sub * 8;

  u32x4 raw[U];
#pragma unroll
  for (int u = 0; u < U; ++u) raw[u] = (u32x4){0u, 0u, 0u, 0u};
  if (active) {
#pragma unroll
    for (int u = 0; u < U; ++u) raw[u] = __builtin_nontemporal_load((const u32x4*)(mv + (size_t)u * D));
  }

  // (max, 1/sum) of the write row and of this lane's read row (query head g = sub)
  float2 nw = make_float2(0.f, 0.f), nr = make_float2(0.f, 0.f);
  if (NORM) {
    // all rows' pairs are requested before the first is reduced (rows past R repeat row 0 and are dropped)
    TileStats ts[kMaxRows];
#pragma unroll
    for (uint32_t r = 0; r < kMaxRows; ++r)
      ts[r] = load_tile_stats(p.stats + ((size_t)unit * R + (r < R ? r : 0u)) * p.n_tiles, p.n_tiles, lane);
#pragma unroll
    for (uint32_t r = 0; r < kMaxRows; ++r) {
      if (r < R) {
        const float2 ms = merge_tile_stats(ts[r]);
        const float mx = ms.x;
        float inv = 1.0f / ms.y;
        if (WRITE && r == 0) {
          if (p.gate) inv *= p.gate[(size_t)b * p.gate_bstride + h];
          nw = make_float2(mx, inv);
        }
        if (r == W + (uint32_t)sub && r >= W) nr = make_float2(mx, inv);
      }
    }
  } else {
    if (WRITE) nw = p.norm[(size_t)unit * R];
    if ((uint32_t)sub < G) nr = p.norm[(size_t)unit * R + W + sub];
  }

  const float* sc = p.scores + (size_t)unit * R * M + slot0;  // row r at sc + r * M
  float rw[U];
#pragma unroll
  for (int u = 0; u < U; ++u) rw[u] = 0.f;
  if (active && (uint32_t)sub < G) {
#pragma unroll
    for (int k = 0; k < U / 4; ++k) {
      const f32x4v a = *(const f32x4v*)(sc + (size_t)(W + sub) * M + 4 * k);
#pragma unroll
      for (int i = 0; i < 4; ++i) rw[4 * k + i] = fast_exp2(a[i] - nr.x) * nr.y;
    }
  }
  // hi + lo bf16 parts of the lane's weights, 8 slots per block: the A operands
  u32x4 ahi[NB], alo[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int w2 = 0; w2 < 4; ++w2) {
      const float r0 = rw[8 * nb + 2 * w2], r1 = rw[8 * nb + 2 * w2 + 1];
      const uint32_t hw = pack_bf16x2(r0, r1);
      ahi[nb][w2] = hw;
      alo[nb][w2] = pack_bf16x2(r0 - __uint_as_float(hw << 16), r1 - __uint_as_float(hw & 0xFFFF0000u));
    }

  if (WRITE && active) {
    float ww[U];
#pragma unroll
    for (int k = 0; k < U / 4; ++k) {
      const f32x4v a = *(const f32x4v*)(sc + 4 * k);
#pragma unroll
      for (int i = 0; i < 4; ++i) ww[4 * k + i] = fast_exp2(a[i] - nw.x) * nw.y;
    }
    float wvf[8];
    const uint16_t* wv = (const uint16_t*)p.wv + (size_t)b * p.kv_bstride + (size_t)h * D;
    unpack16<BF16>(*(const u32x4*)(wv + sub * 8), wvf);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[8];
      unpack16<BF16>(raw[u], x);
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(ww[u], wvf[e], x[e]);
      raw[u] = pack16_round<BF16>(x);
      __builtin_nontemporal_store(raw[u], (u32x4*)(mv + (size_t)u * D));
    }
  }

  // in-lane transpose of the 8 x 8 block of bf16 (slot u, column e) and the products
  f32x4v acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    f32x4v z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      u32x4 t;
#pragma unroll
      for (int w2 = 0; w2 < 4; ++w2) {
        const uint32_t lo = raw[8 * nb + 2 * w2][e / 2], hi = raw[8 * nb + 2 * w2 + 1][e / 2];
        t[w2] = (e % 2 == 0) ? ((lo & 0xFFFFu) | (hi << 16)) : ((lo >> 16) | (hi & 0xFFFF0000u));
      }
      const bf16x8 bv = __builtin_bit_cast(bf16x8, t);
      z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ahi[nb]), bv, z, 0, 0, 0);
      z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, alo[nb]), bv, z, 0, 0, 0);
    }
    acc[e] = z;
  }

  // accumulator e, element v of lane (sub, sl): query head 4 sl + v, column 8 sub + e
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const uint32_t g = 4 * sl + v;
    if (g < G) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s_red[(wave * kMaxG + g) * D + 8 * sub + e] = acc[e][v];
    }
  }
  __syncthreads();
  for (uint32_t i = tid; i < G * D; i += BS) {
    const uint32_t g = i / D, j = i % D;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) v += s_red[(w * kMaxG + g) * D + j];
    const uint32_t hq = h * G + g;
    if (p.S == 1) {
      store_elem((uint16_t*)p.out, (size_t)b * p.q_bstride + (size_t)hq * D + j, v);
    } else {
      p.partial[(((size_t)split * p.B + b) * p.Hq + hq) * D + j] = v;
    }
  }
}

}  // namespace

template <int BS, int U>
static void launch_gqa_bs(const DecodeParams& p, hipStream_t s) {
  const dim3 grid = unit_grid(p.S, (uint64_t)p.B * p.Hkv), block(BS);
  if (p.has_write) {
    if (p.fuse_norm) hipLaunchKernelGGL((mv_pass_gqa_kernel<true, BS, true, U>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((mv_pass_gqa_kernel<true, BS, false, U>), grid, block, 0, s, p);
  } else {
    if (p.fuse_norm) hipLaunchKernelGGL((mv_pass_gqa_kernel<false, BS, true, U>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((mv_pass_gqa_kernel<false, BS, false, U>), grid, block, 0, s, p);
  }
}

// bf16, d = 128, G > 2, a step with a read.  The launch shape is the plan's: 128 threads, 8 loads per lane
// (the kernel is written for any multiple of 8 loads; 16 measured slower, see plan_mv_pass).
hipError_t launch_stream_gqa(const DecodeParams& p, hipStream_t s) {
  if (p.d != 128 || p.G <= 2 || p.G > kMaxG || !p.has_read) return hipErrorInvalidConfiguration;
  if (p.mv_bs != 128 || p.mv_u != 8) return hipErrorInvalidConfiguration;
  launch_gqa_bs<128, 8>(p, s);
  return hipGetLastError();
}

}  // namespace bct
