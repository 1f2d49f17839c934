// The MV pass of a decode step (gfx950): the one read-modify-write stream over
// the value memory.  For every slot m of every memory (b, h):
//     MV[m,:] <- round(fma(ww[m], wv, MV[m,:]))            (section 3.2 step 4,
//                                                            section 3.4 equation,
//                                                            stored back: step 5)
//     out[g,:] += rw[g][m] * MV[m,:]  (the value just stored) (the layer's read)
// with ww = softmax of the write scores and rw[g] = softmax of the read scores
// (section 3.2 step 2), normalised with the per-row (max, 1/sum) that the
// normaliser kernel merged from the per-tile pairs of the scores pass.
//
// Shape of the launch: one workgroup = one (split, memory), and it makes NO
// loop over memory: every lane issues its U 16-byte loads up front, then does
// the arithmetic, then its U stores.  On MI355X a workgroup that walks a long
// contiguous range, alternating loads and stores, reaches ~5.4 TB/s on a plain
// in-place copy, while one-shot workgroups of 16 KB reach ~6.0-6.2 TB/s, so
// the split factor S is chosen to make the workgroups one-shot.
//
// Lane layout: LPS = d*sizeof(elem)/16 lanes hold one slot row (16 bytes each).
// The 64/LPS lane groups of a wavefront take U CONSECUTIVE slots each, so a
// lane's U softmax weights of one row are adjacent floats (one or two 16-byte
// loads), and one load instruction of the wavefront touches 64/LPS whole rows.
#include "bct_device.h"
#include "bct_internal.h"

namespace bct {

template <int U>
__device__ __forceinline__ void load_run(const float* p, float* w) {
  if constexpr (U % 4 == 0) {
#pragma unroll
    for (int i = 0; i < U / 4; ++i) {
      const f32x4 v = *(const f32x4*)(p + 4 * i);
      w[4 * i + 0] = v.x;
      w[4 * i + 1] = v.y;
      w[4 * i + 2] = v.z;
      w[4 * i + 3] = v.w;
    }
  } else {
    static_assert(U == 2, "U is 2, 4, 8 or 16");
    const float2 v = *(const float2*)p;
    w[0] = v.x;
    w[1] = v.y;
  }
}

// NORM: the workgroup merges the per-tile (max, sum) pairs of its memory's rows itself (at most 128
// tiles: two per lane, the same arithmetic as the normaliser kernel, so the same bits) while its MV
// loads are in flight, and the normaliser launch is dropped.
template <typename DT, int D, int GT, bool WRITE, bool READ, int BS, int U, bool NORM>
__global__ __launch_bounds__(BS) void mv_pass_kernel(const DecodeParams p) {
  typedef typename DT::elem elem;
  constexpr int E = DT::kElemsPerVec;
  constexpr int LPS = D / E;          // lanes per slot row
  constexpr int SPW = 64 / LPS;       // lane groups (slots per load instruction) per wavefront
  constexpr int NW = BS / 64;         // wavefronts per workgroup
  constexpr int SPB = NW * SPW * U;   // slots per workgroup

  __shared__ float s_red[READ ? NW * GT * D : 1];

  const uint32_t split = blockIdx.x, unit = block_unit();
  if (unit >= p.B * p.Hkv) return;
  const uint32_t b = unit / p.Hkv, h = unit % p.Hkv;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int sub = lane % LPS, sl = lane / LPS;
  const uint32_t R = p.R, G = p.G, M = p.M;

  // this lane's U consecutive slots; M is a multiple of 64 >= U, so a run is
  // either wholly inside the memory or wholly outside
  const uint32_t slot0 = split * SPB + (wave * SPW + sl) * U;
  const bool active = slot0 < M;
  elem* mv = (elem*)p.mv + ((size_t)unit * M + slot0) * D + sub * E;

  u32x4 raw[U];
  if (active) {
#pragma unroll
    for (int u = 0; u < U; ++u) raw[u] = __builtin_nontemporal_load((const u32x4*)(mv + (size_t)u * D));
  }

  float acc[GT][E];
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int e = 0; e < E; ++e) acc[g][e] = 0.f;

  // (max, 1/sum) of row r of this memory
  constexpr int NR = (WRITE ? 1 : 0) + (READ ? GT : 0);
  float2 nrm[NR];
  if (NORM) {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      if ((uint32_t)r < R) {
        const float2 ms = merge_tile_stats(p.stats + ((size_t)unit * R + r) * p.n_tiles, p.n_tiles, lane);
        const float mx = ms.x;
        float inv = 1.0f / ms.y;
        if (WRITE && r == 0 && p.gate) inv *= p.gate[(size_t)b * p.gate_bstride + h];
        nrm[r] = make_float2(mx, inv);
      }
    }
  } else {
#pragma unroll
    for (int r = 0; r < NR; ++r)
      if ((uint32_t)r < R) nrm[r] = p.norm[(size_t)unit * R + r];
  }

  if (active) {
    const float* sc = p.scores + (size_t)unit * R * M + slot0;  // row r at sc + r*M
    float ww[U];
    if (WRITE) {
      load_run<U>(sc, ww);
      const float2 n = nrm[0];
#pragma unroll
      for (int u = 0; u < U; ++u) ww[u] = fast_exp2(ww[u] - n.x) * n.y;
    }
    float rw[GT][U];
    if (READ) {
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        if ((uint32_t)g < G) {
          const int row = (WRITE ? 1 : 0) + g;
          load_run<U>(sc + (size_t)row * M, rw[g]);
          const float2 n = nrm[row];
#pragma unroll
          for (int u = 0; u < U; ++u) rw[g][u] = fast_exp2(rw[g][u] - n.x) * n.y;
        }
      }
    }
    float wvf[E];
    if (WRITE) {
      const elem* wv = (const elem*)p.wv + (size_t)b * p.kv_bstride + (size_t)h * D;
      unpack16<DT>(*(const u32x4*)(wv + sub * E), wvf);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float x[E];
      unpack16<DT>(raw[u], x);
      if (WRITE) {
#pragma unroll
        for (int e = 0; e < E; ++e) x[e] = __builtin_fmaf(ww[u], wvf[e], x[e]);
        raw[u] = pack16_round<DT>(x);  // x now holds the stored (rounded) values
      }
      if (READ) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
          if ((uint32_t)g < G) {
#pragma unroll
            for (int e = 0; e < E; ++e) acc[g][e] = __builtin_fmaf(rw[g][u], x[e], acc[g][e]);
          }
        }
      }
    }
    if (WRITE) {
#pragma unroll
      for (int u = 0; u < U; ++u) __builtin_nontemporal_store(raw[u], (u32x4*)(mv + (size_t)u * D));
    }
  }

  if (READ) {
    // sum over the lane groups of the wavefront (same column chunk `sub`),
    // then over the wavefronts through LDS, in a fixed order
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
      for (int e = 0; e < E; ++e) acc[g][e] = xor_sum<LPS, 32>(acc[g][e]);
    if (sl == 0) {
#pragma unroll
      for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < E; ++e) s_red[(wave * GT + g) * D + sub * E + e] = acc[g][e];
    }
    __syncthreads();
    for (uint32_t i = tid; i < G * D; i += BS) {
      const uint32_t g = i / D, j = i % D;
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) v += s_red[(w * GT + g) * D + j];
      const uint32_t hq = h * G + g;
      if (p.S == 1) {
        store_elem((elem*)p.out, (size_t)b * p.q_bstride + (size_t)hq * D + j, v);
      } else {
        p.partial[(((size_t)split * p.B + b) * p.Hq + hq) * D + j] = v;
      }
    }
  }
}

// ------------------------------------------------------------------ host side

// Workgroup shapes of the MV pass: (threads, 16-byte loads per lane); bytes per
// workgroup = threads * loads * 16.  Measured at B=32, H=32, M=4096, d=128 bf16
// (1 GiB of MV): 256x4 343 us, 256x2 343, 64x4 348, 128x8 359, 128x4 368,
// 512x16 376, 1024x8 379, 512x4 385, 256x8 395, 1024x4 404, 256x16 418,
// 512x8 424: small one-shot workgroups win, and the cost of summing their
// many partial outputs (one more launch) is ~5 us.  With four query heads per
// KV head the read accumulation is four times the arithmetic and registers
// and 512x8 is the fastest (394 us against 410 at B=64, Hkv=8, M=8192).
struct MvShape {
  uint32_t bs, u;
};
static constexpr MvShape kSmall = {256, 4};  // 16 KB per workgroup
static constexpr MvShape kWide = {512, 8};   // 64 KB per workgroup

// Mid-size caches, one query head per KV head: one workgroup per memory, 16 loads per lane (256, 512 or 1024
// threads for memories up to 64, 128, 256 KB).  No split of M, so no partial outputs and no merge launch;
// worth it while one or two rounds of such workgroups cover the chip and the launches saved still count.
// Measured inside a HIP graph, whole step, against the 16 KB shape (us):
//   bf16 d = 128, M = 1024: 192 memories 27.2 -> 23.1, 256: 32.8 -> 28.5 (config 2 of the benchmark), 384: 44.7 -> 46.1,
//                           512: 55.9 -> 54.1, 1024: 102 -> 109;  M = 512: 256: 17.5 -> 16.5, 512: 31.8 -> 26.5,
//                           1024: 55.8 -> 55.4, 2048: 102 -> 109;  M = 256: 512: 17.2 -> 15.8, 1024: 31.9 -> 26.6
//   fp32 d = 64,  M = 1024: 192: 30.9 -> 29.4, 256: 37.7 -> 36.1, 384: 53.8 -> 59.2;  M = 512: 512: 37.1 -> 33.6
//   fp32 d = 128, M = 512: 256: 39.9 -> 36.3, 384: 56.2 -> 59.2;  bf16 d = 64, M = 2048: 256: 34.2 -> 28.3
//   fewer than 192 memories lose (128 x M = 1024: 18.3 -> 19.6; 8: 10.2 -> 13.5): too few workgroups.
// Hence: at least 192 memories and at most 64 MB of MV in all.
static constexpr uint64_t kWholeMinBytes = 32u << 10, kWholeMaxBytes = 256u << 10;
static constexpr uint64_t kWholeMinUnits = 192, kWholeMaxTotal = 64ull << 20;

// bf16, d = 128, G > 2: the MFMA read (bct_mv_pass_gqa.hip), again 16 KB one-shot workgroups.  Measured at
// B = 64, Hkv = 8, G = 4, M = 8192 (MV pass alone): 128 threads 351 us, 256 threads 386 us, 512 threads 415 us,
// against 429 us for the vector-ALU read in its best shape (512 x 8); the smaller workgroups leave more
// partial outputs to sum (merge 21 us against 7 us).  16 loads per lane: 128 threads 397 us, 64 threads 357 us.
static constexpr MvShape kGqa = {128, 8};

void plan_mv_pass(DecodeParams& p, int dtype) {
  const bool gqa = p.G > 2 && dtype == 1 && p.d == 128;
  MvShape s = (p.G <= 2) ? kSmall : gqa ? kGqa : kWide;
  const uint64_t mem = (uint64_t)p.M * p.d * (dtype == 0 ? 4u : 2u), units = (uint64_t)p.B * p.Hkv;
  if (p.G <= 1 && mem > kWholeMinBytes && mem <= kWholeMaxBytes && units >= kWholeMinUnits && units * mem <= kWholeMaxTotal)
    s = MvShape{mem <= (64u << 10) ? 256u : mem <= (128u << 10) ? 512u : 1024u, 16u};
  p.mv_bs = s.bs;
  p.mv_u = s.u;
  const uint32_t row_bytes = p.d * (dtype == 0 ? 4u : 2u);
  const uint32_t spb = s.bs * s.u * 16u / row_bytes;  // slots per workgroup
  p.S = (p.M + spb - 1) / spb;
  // With at most two (max, sum) pairs per lane the workgroups of the MV pass merge them themselves.  In the
  // pass for several query heads that costs every workgroup a little (1 + G rows; 13 us over the 65536
  // workgroups of B = 64, Hkv = 8, M = 8192, where the normaliser launch takes 5), so a large grid leaves it
  // to the launch.
  const uint64_t wgs = (uint64_t)p.B * p.Hkv * p.S;
  p.fuse_norm = (p.n_tiles <= kMaxMergedTiles && (!gqa || wgs <= 16384)) ? 1u : 0u;
}

template <typename DT, int D, int GT, int BS, int U, bool NORM>
static void launch_mode_n(const DecodeParams& p, hipStream_t s) {
  const dim3 grid = unit_grid(p.S, (uint64_t)p.B * p.Hkv), block(BS);
  if (p.has_write && p.has_read)
    hipLaunchKernelGGL((mv_pass_kernel<DT, D, GT, true, true, BS, U, NORM>), grid, block, 0, s, p);
  else if (p.has_read)
    hipLaunchKernelGGL((mv_pass_kernel<DT, D, GT, false, true, BS, U, NORM>), grid, block, 0, s, p);
  else
    hipLaunchKernelGGL((mv_pass_kernel<DT, D, 1, true, false, BS, U, NORM>), grid, block, 0, s, p);
}

template <typename DT, int D, int GT, int BS, int U>
static void launch_mode(const DecodeParams& p, hipStream_t s) {
  if (p.fuse_norm) launch_mode_n<DT, D, GT, BS, U, true>(p, s);
  else launch_mode_n<DT, D, GT, BS, U, false>(p, s);
}

template <typename DT, int D>
static bool launch_shape(const DecodeParams& p, hipStream_t s) {
  const uint32_t G = p.G;
  if (p.mv_u == 16 && G <= 1 && p.fuse_norm) {   // one workgroup per memory (at most 2048 slots: the statistics always fit)
    if (p.mv_bs == 1024) launch_mode_n<DT, D, 1, 1024, 16, true>(p, s);
    else if (p.mv_bs == 512) launch_mode_n<DT, D, 1, 512, 16, true>(p, s);
    else if (p.mv_bs == 256) launch_mode_n<DT, D, 1, 256, 16, true>(p, s);
    else return false;
    return true;
  }
  if (p.mv_bs == kSmall.bs && p.mv_u == kSmall.u && G <= 2) {
    if (G <= 1) launch_mode<DT, D, 1, 256, 4>(p, s);
    else launch_mode<DT, D, 2, 256, 4>(p, s);
    return true;
  }
  if (p.mv_bs == kWide.bs && p.mv_u == kWide.u && G > 2) {
    if (!p.has_read) launch_mode<DT, D, 1, 512, 8>(p, s);
    else if (G <= 4) launch_mode<DT, D, 4, 512, 8>(p, s);
    else launch_mode<DT, D, 8, 512, 8>(p, s);
    return true;
  }
  if (p.mv_u == 8 && G > 2 && !p.has_read) {   // write-only step of a cache whose reads take the MFMA pass
    if (p.mv_bs == 256) launch_mode<DT, D, 1, 256, 8>(p, s);
    else if (p.mv_bs == 128) launch_mode<DT, D, 1, 128, 8>(p, s);
    else return false;
    return true;
  }
  return false;
}

hipError_t launch_stream(const DecodeParams& p, int dtype, hipStream_t s) {
  if (dtype == 1 && p.d == 128 && p.G > 2 && p.has_read) return launch_stream_gqa(p, s);
  bool ok;
  if (dtype == 0) ok = (p.d == 128) ? launch_shape<F32, 128>(p, s) : launch_shape<F32, 64>(p, s);
  else ok = (p.d == 128) ? launch_shape<BF16, 128>(p, s) : launch_shape<BF16, 64>(p, s);
  if (!ok) return hipErrorInvalidConfiguration;
  return hipGetLastError();
}

}  // namespace bct
