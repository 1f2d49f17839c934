// Decode-step kernels of libbct (gfx950).
//
// One decode step of one layer is three launches on the caller's stream:
//   1. scores : for every memory (b, h) and every row (the write query wq and
//               the G read queries q), the scaled dot products with all M keys
//               of MK, kept in the log2 domain, plus one (max, sum) pair per
//               slot tile.  (section 3.2 step 2 / Algorithm 1 "score"; the same
//               pass serves the read.)
//   2. stream : merges the (max, sum) pairs into the softmax normaliser, then
//               makes ONE pass over MV: load, ww[m] * wv + MV (one fp32 FMA),
//               round to storage, store, and accumulate the read output from
//               the value just stored.  (section 3.2 steps 2, 4, 5; section 3.4
//               equation.)  The normaliser must be known before any slot can be
//               written, which is why this is a second launch.
//   3. merge  : sums the split-M partial outputs in a fixed order (only if the
//               MV pass was split).
#include "bct_device.h"
#include "bct_internal.h"

namespace bct {

// ------------------------------------------------------------------ scores (generic)

// One workgroup = one (slot tile of 64, memory).  LPS lanes share a slot: each
// holds 16 bytes of the key row and of the query row.
template <typename DT, int D>
__global__ __launch_bounds__(256) void scores_generic_kernel(const DecodeParams p) {
  typedef typename DT::elem elem;
  constexpr int E = DT::kElemsPerVec;
  constexpr int LPS = D / E;       // lanes per slot
  constexpr int SPP = 256 / LPS;   // slots per pass of the workgroup
  constexpr int TILE = 64;
  static_assert(TILE % SPP == 0, "tile must be a whole number of passes");

  __shared__ float s_sc[kMaxRows][TILE];

  const uint32_t tile = blockIdx.x, unit = blockIdx.y;
  const uint32_t b = unit / p.Hkv, h = unit % p.Hkv;
  const int tid = threadIdx.x, sub = tid % LPS, sl = tid / LPS;
  const elem* mk = (const elem*)p.mk + (size_t)(p.mk_per_seq ? unit : h) * p.M * D;

  for (int pass = 0; pass < TILE / SPP; ++pass) {
    const uint32_t slot = tile * TILE + pass * SPP + sl;
    float kf[E];
    unpack16<DT>(*(const u32x4*)(mk + (size_t)slot * D + sub * E), kf);
    for (uint32_t r = 0; r < p.R; ++r) {
      const elem* x;
      float scale;
      if (p.has_write && r == 0) {
        x = (const elem*)p.wq + (size_t)b * p.kv_bstride + (size_t)h * D;
        scale = p.wscale_l2e;
      } else {
        x = (const elem*)p.q + (size_t)b * p.q_bstride + (size_t)(h * p.G + (r - p.has_write)) * D;
        scale = p.rscale_l2e;
      }
      float xf[E];
      unpack16<DT>(*(const u32x4*)(x + sub * E), xf);
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) dot = __builtin_fmaf(kf[e], xf[e], dot);
      dot = xor_sum<1, LPS / 2>(dot);
      if (sub == 0) {
        const float s = dot * scale;
        s_sc[r][pass * SPP + sl] = s;
        p.scores[((size_t)unit * p.R + r) * p.M + slot] = s;
      }
    }
  }
  __syncthreads();
  const int wave = tid / 64, lane = tid % 64;
  for (uint32_t r = wave; r < p.R; r += 4) {
    const float v = s_sc[r][lane];
    const float mx = xor_max<1, 32>(v);
    const float sm = xor_sum<1, 32>(fast_exp2(v - mx));
    if (lane == 0) p.stats[((size_t)unit * p.R + r) * p.n_tiles + tile] = make_float2(mx, sm);
  }
}

// ------------------------------------------------------------------ scores (bf16, shared keys, MFMA)

// With keys shared over the batch the scores of one KV head are a dense
// contraction: [B*R rows] x [d] x [M slots].  One wavefront owns 32*NT slots,
// keeps their key fragments in registers and walks the rows 32 at a time with
// v_mfma_f32_32x32x16_bf16 (A = query rows, B = key slots, fp32 accumulate).
// Lane l supplies row/slot (l % 32) and the 8 consecutive k at 8 * (l / 32);
// the accumulator holds column (l % 32), rows 8*(v/4) + 4*(l/32) + v%4.
template <int D, int NT>
__global__ __launch_bounds__(64) void scores_mfma_bf16_kernel(const DecodeParams p) {
  constexpr int KS = D / 16;
  const uint32_t tile = blockIdx.x, h = blockIdx.y;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const uint16_t* mk = (const uint16_t*)p.mk + (size_t)h * p.M * D;
  const uint32_t slot0 = tile * (32 * NT);

  u32x4 kf[NT][KS];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      kf[t][ks] = *(const u32x4*)(mk + (size_t)(slot0 + t * 32 + col) * D + ks * 16 + half * 8);

  const uint32_t rtot = p.B * p.R;
  for (uint32_t rb = blockIdx.z; rb * 32 < rtot; rb += gridDim.z) {
    const uint32_t rho = rb * 32 + col;
    u32x4 xf[KS];
    if (rho < rtot) {
      const uint32_t b = rho / p.R, r = rho % p.R;
      const uint16_t* x = (p.has_write && r == 0)
                              ? (const uint16_t*)p.wq + (size_t)b * p.kv_bstride + (size_t)h * D
                              : (const uint16_t*)p.q + (size_t)b * p.q_bstride +
                                    (size_t)(h * p.G + (r - p.has_write)) * D;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) xf[ks] = *(const u32x4*)(x + ks * 16 + half * 8);
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) xf[ks] = (u32x4){0u, 0u, 0u, 0u};
    }
    f32x16 c[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) c[t][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int t = 0; t < NT; ++t)
        c[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xf[ks]),
                                                       __builtin_bit_cast(bf16x8, kf[t][ks]), c[t], 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const uint32_t row = rb * 32 + (v / 4) * 8 + half * 4 + (v % 4);
      if (row < rtot) {
        const uint32_t b = row / p.R, r = row % p.R;
        const float scale = (p.has_write && r == 0) ? p.wscale_l2e : p.rscale_l2e;
        const size_t urow = (size_t)(b * p.Hkv + h) * p.R + r;
        float s[NT];
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          s[t] = c[t][v] * scale;
          p.scores[urow * p.M + slot0 + t * 32 + col] = s[t];
          mx = fmaxf(mx, s[t]);
        }
        mx = xor_max<1, 16>(mx);
        float sm = 0.f;
#pragma unroll
        for (int t = 0; t < NT; ++t) sm += fast_exp2(s[t] - mx);
        sm = xor_sum<1, 16>(sm);
        if (col == 0) p.stats[urow * p.n_tiles + tile] = make_float2(mx, sm);
      }
    }
  }
}

// ------------------------------------------------------------------ MV pass

// One workgroup = one (split, memory).  LPS lanes hold one slot row (16 bytes
// each); a wavefront covers 64/LPS slots per load and U loads per iteration,
// four wavefronts cover kStreamChunk = 64 slots per iteration.
template <typename DT, int D, int GT, bool WRITE, bool READ>
__global__ __launch_bounds__(256) void stream_kernel(const DecodeParams p) {
  typedef typename DT::elem elem;
  constexpr int E = DT::kElemsPerVec;
  constexpr int LPS = D / E;
  constexpr int SPW = 64 / LPS;  // slots per wavefront per load
  constexpr int U = LPS / 4;     // loads per lane per iteration
  static_assert(4 * SPW * U == (int)kStreamChunk, "a workgroup iteration covers 64 slots");

  __shared__ float s_gmax[kMaxRows], s_ginv[kMaxRows];
  __shared__ float s_red[READ ? 4 * GT * D : 1];

  const uint32_t split = blockIdx.x, unit = blockIdx.y;
  const uint32_t b = unit / p.Hkv, h = unit % p.Hkv;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int sub = lane % LPS, sl = lane / LPS;
  const uint32_t R = p.R, G = p.G, M = p.M;

  // softmax normalisers: merge the per-tile (max, sum) pairs of each row
  for (uint32_t r = wave; r < R; r += 4) {
    const float2* st = p.stats + ((size_t)unit * R + r) * p.n_tiles;
    float mx = -INFINITY;
    for (uint32_t i = lane; i < p.n_tiles; i += 64) mx = fmaxf(mx, st[i].x);
    mx = xor_max<1, 32>(mx);
    float sm = 0.f;
    for (uint32_t i = lane; i < p.n_tiles; i += 64) sm += st[i].y * fast_exp2(st[i].x - mx);
    sm = xor_sum<1, 32>(sm);
    if (lane == 0) {
      s_gmax[r] = mx;
      s_ginv[r] = 1.0f / sm;
    }
  }
  __syncthreads();

  float w_max = 0.f, w_inv = 0.f, r_max[GT], r_inv[GT];
  if (WRITE) {
    w_max = s_gmax[0];
    w_inv = s_ginv[0];
  }
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const bool on = READ && (uint32_t)g < G;
    r_max[g] = on ? s_gmax[(WRITE ? 1 : 0) + g] : 0.f;
    r_inv[g] = on ? s_ginv[(WRITE ? 1 : 0) + g] : 0.f;
  }

  float wvf[E];
  if (WRITE) {
    const elem* wv = (const elem*)p.wv + (size_t)b * p.kv_bstride + (size_t)h * D;
    unpack16<DT>(*(const u32x4*)(wv + sub * E), wvf);
  }
  float acc[GT][E];
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int e = 0; e < E; ++e) acc[g][e] = 0.f;

  elem* mv = (elem*)p.mv + (size_t)unit * M * D;
  const float* sc_w = p.scores + (size_t)unit * R * M;            // row 0 when WRITE
  const float* sc_r = sc_w + (WRITE ? (size_t)M : 0);             // read rows follow
  const uint32_t chunks = M / kStreamChunk;
  const uint32_t c0 = (uint32_t)(((uint64_t)chunks * split) / p.S);
  const uint32_t c1 = (uint32_t)(((uint64_t)chunks * (split + 1)) / p.S);

  for (uint32_t c = c0; c < c1; ++c) {
    const uint32_t base = c * kStreamChunk + wave * (SPW * U) + sl;
    u32x4 raw[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      raw[u] = __builtin_nontemporal_load((const u32x4*)(mv + (size_t)(base + u * SPW) * D + sub * E));
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t slot = base + u * SPW;
      float x[E];
      unpack16<DT>(raw[u], x);
      if (WRITE) {
        const float ww = fast_exp2(sc_w[slot] - w_max) * w_inv;
#pragma unroll
        for (int e = 0; e < E; ++e) x[e] = __builtin_fmaf(ww, wvf[e], x[e]);
        const u32x4 st = pack16_round<DT>(x);
        __builtin_nontemporal_store(st, (u32x4*)(mv + (size_t)slot * D + sub * E));
      }
      if (READ) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
          if ((uint32_t)g < G) {
            const float rw = fast_exp2(sc_r[(size_t)g * M + slot] - r_max[g]) * r_inv[g];
#pragma unroll
            for (int e = 0; e < E; ++e) acc[g][e] = __builtin_fmaf(rw, x[e], acc[g][e]);
          }
        }
      }
    }
  }

  if (READ) {
    // lanes with the same column chunk `sub` across the wavefront's slot groups
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
    for (uint32_t i = tid; i < G * D; i += 256) {
      const uint32_t g = i / D, j = i % D;
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) v += s_red[(w * GT + g) * D + j];
      const uint32_t hq = h * G + g;
      if (p.S == 1) {
        store_elem((elem*)p.out, (size_t)b * p.q_bstride + (size_t)hq * D + j, v);
      } else {
        p.partial[(((size_t)split * p.B + b) * p.Hq + hq) * D + j] = v;
      }
    }
  }
}

// out[b][hq][:] = round(sum over splits, ascending) of the partial outputs.
template <typename DT>
__global__ __launch_bounds__(256) void merge_kernel(const DecodeParams p) {
  typedef typename DT::elem elem;
  const size_t n = (size_t)p.B * p.Hq * p.d;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float v = 0.f;
  for (uint32_t s = 0; s < p.S; ++s) v += p.partial[(size_t)s * n + i];
  const size_t per_b = (size_t)p.Hq * p.d;
  store_elem((elem*)p.out, (i / per_b) * p.q_bstride + (i % per_b), v);
}

// ------------------------------------------------------------------ fill / copy

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* dst, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride)
    dst[i] = (u32x4){0u, 0u, 0u, 0u};
}

__global__ __launch_bounds__(256) void copy_kernel(u32x4* dst, const u32x4* src, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// ------------------------------------------------------------------ host side

static bool use_mfma_scores(const DecodeParams& p, int dtype) { return dtype == 1 && !p.mk_per_seq; }

void plan_decode(DecodeParams& p, int dtype) {
  if (use_mfma_scores(p, dtype)) {
    // the largest slot tile per wavefront that still gives about one
    // wavefront per SIMD (1024 on the chip)
    uint32_t nt = 1;
    if (p.M % 128 == 0 && (uint64_t)(p.M / 128) * p.Hkv >= 1024) nt = 4;
    else if ((uint64_t)(p.M / 64) * p.Hkv >= 1024) nt = 2;
    p.stat_tile = 32 * nt;
  } else {
    p.stat_tile = 64;
  }
  p.n_tiles = p.M / p.stat_tile;
  const uint32_t units = p.B * p.Hkv;
  const uint32_t chunks = p.M / kStreamChunk;
  uint32_t s = (2048 + units - 1) / units;
  uint32_t smax = chunks / 4;
  if (smax < 1) smax = 1;
  if (s > smax) s = smax;
  if (s > kMaxSplits) s = kMaxSplits;
  if (s < 1) s = 1;
  p.S = s;
}

template <int D, int NT>
static hipError_t launch_scores_mfma(const DecodeParams& p, hipStream_t s) {
  const uint32_t tiles = p.M / (32 * NT);
  const uint32_t rbs = (p.B * p.R + 31) / 32;
  uint32_t z = 1;
  const uint64_t waves = (uint64_t)tiles * p.Hkv;
  if (waves < 2048) z = (uint32_t)((2048 + waves - 1) / waves);
  if (z > rbs) z = rbs;
  hipLaunchKernelGGL((scores_mfma_bf16_kernel<D, NT>), dim3(tiles, p.Hkv, z), dim3(64), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_scores(const DecodeParams& p, int dtype, hipStream_t s) {
  if (use_mfma_scores(p, dtype)) {
    const uint32_t nt = p.stat_tile / 32;
    if (p.d == 128) {
      if (nt == 4) return launch_scores_mfma<128, 4>(p, s);
      if (nt == 2) return launch_scores_mfma<128, 2>(p, s);
      return launch_scores_mfma<128, 1>(p, s);
    }
    if (nt == 4) return launch_scores_mfma<64, 4>(p, s);
    if (nt == 2) return launch_scores_mfma<64, 2>(p, s);
    return launch_scores_mfma<64, 1>(p, s);
  }
  const dim3 grid(p.M / 64, p.B * p.Hkv);
  if (dtype == 0) {
    if (p.d == 128) hipLaunchKernelGGL((scores_generic_kernel<F32, 128>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((scores_generic_kernel<F32, 64>), grid, dim3(256), 0, s, p);
  } else {
    if (p.d == 128) hipLaunchKernelGGL((scores_generic_kernel<BF16, 128>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((scores_generic_kernel<BF16, 64>), grid, dim3(256), 0, s, p);
  }
  return hipGetLastError();
}

template <typename DT, int D, int GT>
static void launch_stream_mode(const DecodeParams& p, hipStream_t s) {
  const dim3 grid(p.S, p.B * p.Hkv), block(256);
  if (p.has_write && p.has_read) hipLaunchKernelGGL((stream_kernel<DT, D, GT, true, true>), grid, block, 0, s, p);
  else if (p.has_read) hipLaunchKernelGGL((stream_kernel<DT, D, GT, false, true>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((stream_kernel<DT, D, 1, true, false>), grid, block, 0, s, p);
}

template <typename DT, int D>
static void launch_stream_g(const DecodeParams& p, hipStream_t s) {
  if (p.G <= 1) launch_stream_mode<DT, D, 1>(p, s);
  else if (p.G <= 2) launch_stream_mode<DT, D, 2>(p, s);
  else if (p.G <= 4) launch_stream_mode<DT, D, 4>(p, s);
  else launch_stream_mode<DT, D, 8>(p, s);
}

hipError_t launch_stream(const DecodeParams& p, int dtype, hipStream_t s) {
  if (dtype == 0) {
    if (p.d == 128) launch_stream_g<F32, 128>(p, s);
    else launch_stream_g<F32, 64>(p, s);
  } else {
    if (p.d == 128) launch_stream_g<BF16, 128>(p, s);
    else launch_stream_g<BF16, 64>(p, s);
  }
  return hipGetLastError();
}

hipError_t launch_merge(const DecodeParams& p, int dtype, hipStream_t s) {
  if (!p.has_read || p.S == 1) return hipSuccess;
  const size_t n = (size_t)p.B * p.Hq * p.d;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (dtype == 0) hipLaunchKernelGGL((merge_kernel<F32>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((merge_kernel<BF16>), grid, block, 0, s, p);
  return hipGetLastError();
}

static unsigned grid_for(size_t n_vec) {
  size_t blocks = (n_vec + 255) / 256;
  const size_t cap = 256 * 16;  // 16 workgroups per CU keep the loop short and the chip full
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (unsigned)blocks;
}

hipError_t launch_fill_zero(void* dst, size_t n_bytes, hipStream_t s) {
  const size_t n_vec = n_bytes / 16;
  if (n_vec == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(n_vec)), dim3(256), 0, s, (u32x4*)dst, n_vec);
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t n_bytes, hipStream_t s) {
  const size_t n_vec = n_bytes / 16;
  if (n_vec == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_kernel, dim3(grid_for(n_vec)), dim3(256), 0, s, (u32x4*)dst, (const u32x4*)src, n_vec);
  return hipGetLastError();
}

}  // namespace bct
