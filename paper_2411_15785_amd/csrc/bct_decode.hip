// Decode-step kernels of libbct (gfx950).
//
// One decode step of one layer is four launches on the caller's stream:
//   1. scores : for every memory (b, h) and every row (the write query wq and
//               the G read queries q), the scaled dot products with all M keys
//               of MK, kept in the log2 domain, plus one (max, sum) pair per
//               slot tile.  (section 3.2 step 2 / Algorithm 1 "score"; the same
//               pass serves the read.)
//   2. normalise : merges the (max, sum) pairs into each row's softmax
//               normaliser.  Only for memories with more than 128 slot tiles
//               (and for large grids of the several-query-heads MV pass):
//               up to 128 pairs are two per lane, and every workgroup of the MV
//               pass merges them itself while its loads are in flight.
//   3. MV pass : ONE pass over MV: load, ww[m] * wv + MV (one fp32 FMA),
//               round to storage, store, and accumulate the read output from
//               the value just stored.  (section 3.2 steps 2, 4, 5; section 3.4
//               equation.)  The normaliser must be known before any slot can be
//               written, which is why this is a second launch.
//   4. merge  : sums the split-M partial outputs in a fixed order (only if the
//               MV pass was split).
#include "bct_device.h"
#include "bct_internal.h"

namespace bct {

// ------------------------------------------------------------------ scores (generic)

// One workgroup = one (slot tile of 64, memory): 16 KB of keys.  LPS lanes share a slot: each
// holds 16 bytes of the key row and of every query row.  All key loads of a lane are requested
// before the first product (one memory latency per workgroup, as in the MV pass); keys that belong to
// one sequence are read once per step and bypass the caches, shared keys stay cacheable.
template <typename DT, int D, int RT>
__global__ __launch_bounds__(256) void scores_generic_kernel(const DecodeParams p) {
  typedef typename DT::elem elem;
  constexpr int E = DT::kElemsPerVec;
  constexpr int LPS = D / E;       // lanes per slot
  constexpr int SPP = 256 / LPS;   // slots per pass of the workgroup
  constexpr int TILE = 64;
  constexpr int NP = TILE / SPP;   // passes: key rows per lane
  static_assert(TILE % SPP == 0, "tile must be a whole number of passes");

  __shared__ float s_sc[RT][TILE];

  const uint32_t tile = blockIdx.x, unit = block_unit();
  if (unit >= p.B * p.Hkv) return;
  const uint32_t b = unit / p.Hkv, h = unit % p.Hkv;
  const int tid = threadIdx.x, sub = tid % LPS, sl = tid / LPS;
  const uint32_t R = p.R;
  const elem* mk = (const elem*)p.mk + ((size_t)(p.mk_per_seq ? unit : h) * p.M + tile * TILE + sl) * D + sub * E;

  u32x4 kraw[NP];
  if (p.mk_per_seq) {
#pragma unroll
    for (int i = 0; i < NP; ++i) kraw[i] = __builtin_nontemporal_load((const u32x4*)(mk + (size_t)i * SPP * D));
  } else {
#pragma unroll
    for (int i = 0; i < NP; ++i) kraw[i] = *(const u32x4*)(mk + (size_t)i * SPP * D);
  }
  float xf[RT][E], scale[RT];
#pragma unroll
  for (uint32_t r = 0; r < RT; ++r) {
    if (r < R) {
      const elem* x = (p.has_write && r == 0)
                          ? (const elem*)p.wq + (size_t)b * p.kv_bstride + (size_t)h * D
                          : (const elem*)p.q + (size_t)b * p.q_bstride + (size_t)(h * p.G + (r - p.has_write)) * D;
      unpack16<DT>(*(const u32x4*)(x + sub * E), xf[r]);
      scale[r] = (p.has_write && r == 0) ? p.wscale_l2e : p.rscale_l2e;
    }
  }
  float* sc = p.scores + (size_t)unit * R * p.M + tile * TILE;
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    float kf[E];
    unpack16<DT>(kraw[i], kf);
#pragma unroll
    for (uint32_t r = 0; r < RT; ++r) {
      if (r < R) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) dot = __builtin_fmaf(kf[e], xf[r][e], dot);
        dot = xor_sum<1, LPS / 2>(dot);
        if (sub == 0) s_sc[r][i * SPP + sl] = dot * scale[r];
      }
    }
  }
  __syncthreads();
  // a wavefront per row: the tile's 64 scores leave as one 256-byte store, then the row's (max, sum)
  const int wave = tid / 64, lane = tid % 64;
  for (uint32_t r = wave; r < R; r += 4) {
    const float v = s_sc[r][lane];
    sc[(size_t)r * p.M + lane] = v;
    const float mx = xor_max<1, 32>(v);
    const float sm = xor_sum<1, 32>(fast_exp2(v - mx));
    if (lane == 0) p.stats[((size_t)unit * R + r) * p.n_tiles + tile] = make_float2(mx, sm);
  }
}

// ------------------------------------------------------------------ scores (bf16, shared keys, MFMA)

// With keys shared over the batch the scores of one KV head are a dense
// contraction: [M slots] x [d] x [B*R rows].  One wavefront owns 32*NT slots,
// keeps their key fragments in registers and walks the rows 32 at a time with
// v_mfma_f32_32x32x16_bf16 (A = key slots, B = query rows, fp32 accumulate).
// Lane l supplies slot/row (l % 32) and the 8 consecutive k at 8 * (l / 32).
// The accumulator of lane l holds query row (l % 32) and the slots
// 8*(v/4) + 4*(l/32) + v%4, v = 0..15: all slots of a row sit in two lanes, so
// the per-tile (max, sum) of a row is an in-lane reduction plus one exchange,
// and four consecutive slots go out as one 16-byte store.
template <int D, int NT>
__global__ __launch_bounds__(64) void scores_mfma_bf16_kernel(const DecodeParams p) {
  constexpr int KS = D / 16;
  const uint32_t tile = blockIdx.x, h = blockIdx.y;
  const int lane = threadIdx.x, col = lane % 32, half = lane / 32;
  const uint16_t* mk = (const uint16_t*)p.mk + (size_t)h * p.M * D;
  const uint32_t slot0 = tile * (32 * NT);
  const uint32_t rtot = p.B * p.R;

  // Order of the requests: the first block of operand rows, then the keys 32 slots at a time.  Loads
  // return in the order issued and the products below go through the keys in the same order, so the
  // scores of the first 32 slots are computed and on their way to memory while the other keys are
  // still arriving: the kernel's reads and its writes overlap, although every wavefront has its SIMD
  // to itself.  The operand rows of the next block of 32 are requested before the products of the
  // current one.
  auto load_rows = [&](uint32_t rb, u32x4 (&xf)[KS]) {
    const uint32_t rho = rb * 32 + col;
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
  };
  u32x4 xn[KS];
  if (blockIdx.z * 32 < rtot) load_rows(blockIdx.z, xn);

  u32x4 kf[NT][KS];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      kf[t][ks] = *(const u32x4*)(mk + (size_t)(slot0 + t * 32 + col) * D + ks * 16 + half * 8);

  for (uint32_t rb = blockIdx.z; rb * 32 < rtot; rb += gridDim.z) {
    const uint32_t rho = rb * 32 + col;   // this lane's query row
    const bool valid = rho < rtot;
    const uint32_t b = valid ? rho / p.R : 0u, r = valid ? rho % p.R : 0u;
    u32x4 xf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) xf[ks] = xn[ks];
    if ((rb + gridDim.z) * 32 < rtot) load_rows(rb + gridDim.z, xn);
    const float scale = (p.has_write && r == 0) ? p.wscale_l2e : p.rscale_l2e;
    const size_t urow = (size_t)(b * p.Hkv + h) * p.R + r;
    float* dst = p.scores + urow * p.M + slot0 + half * 4;
    // (max, sum of exp2(score - max)) of the row over the tile, 32 slots at a time
    float mx = -INFINITY, sm = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      f32x16 c;
#pragma unroll
      for (int v = 0; v < 16; ++v) c[v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[t][ks]),
                                                    __builtin_bit_cast(bf16x8, xf[ks]), c, 0, 0, 0);
      float mt = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        c[v] *= scale;
        mt = fmaxf(mt, c[v]);
      }
      if (valid) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x4 o = {c[q4 * 4 + 0], c[q4 * 4 + 1], c[q4 * 4 + 2], c[q4 * 4 + 3]};
          *(f32x4*)(dst + t * 32 + q4 * 8) = o;
        }
      }
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
      float st = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) st += fast_exp2(c[v] - mt);
      st += __shfl_xor(st, 32, 64);
      const float mn = fmaxf(mx, mt);
      sm = sm * fast_exp2(mx - mn) + st * fast_exp2(mt - mn);
      mx = mn;
    }
    if (valid && half == 0) p.stats[urow * p.n_tiles + tile] = make_float2(mx, sm);
  }
}

// Softmax normalisers: one wavefront per (memory, row) merges the per-tile
// (max, sum) pairs into the row's (max, 1 / sum of exp2(score - max)).  A step
// size, if given, multiplies the write row's 1 / sum: the MV pass then applies
// eta * ww at no cost of its own.
__global__ __launch_bounds__(256) void normalise_kernel(const DecodeParams p) {
  const uint32_t row = blockIdx.x * 4 + threadIdx.x / 64, lane = threadIdx.x % 64;
  if (row >= p.B * p.Hkv * p.R) return;
  const float2* st = p.stats + (size_t)row * p.n_tiles;
  float mx = -INFINITY;
  for (uint32_t i = lane; i < p.n_tiles; i += 64) mx = fmaxf(mx, st[i].x);
  mx = xor_max<1, 32>(mx);
  float sm = 0.f;
  for (uint32_t i = lane; i < p.n_tiles; i += 64) sm += st[i].y * fast_exp2(st[i].x - mx);
  sm = xor_sum<1, 32>(sm);
  if (lane == 0) {
    float inv = 1.0f / sm;
    if (p.gate && p.has_write && row % p.R == 0) {  // row 0 of a memory is its write row
      const uint32_t unit = row / p.R;
      inv *= p.gate[(size_t)(unit / p.Hkv) * p.gate_bstride + unit % p.Hkv];
    }
    p.norm[row] = make_float2(mx, inv);
  }
}

// out[b][hq][:] = round(sum over the S split-M partial outputs).  A workgroup
// covers 128 consecutive output elements: 8 groups of 32 lanes, each lane four
// elements (one 16-byte load per split); group k sums splits k, k+8, ... and
// the eight group sums are added in group order, so the result does not depend
// on timing.
template <typename DT>
__global__ __launch_bounds__(256) void merge_kernel(const DecodeParams p) {
  typedef typename DT::elem elem;
  __shared__ f32x4 s_part[8][32];
  const size_t n = (size_t)p.B * p.Hq * p.d;
  const int grp = threadIdx.x / 32, ln = threadIdx.x % 32;
  const size_t i = ((size_t)blockIdx.x * 32 + ln) * 4;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (i < n) {
#pragma unroll 4
    for (uint32_t s = grp; s < p.S; s += 8) acc += *(const f32x4*)(p.partial + (size_t)s * n + i);
  }
  s_part[grp][ln] = acc;
  __syncthreads();
  if (grp == 0 && i < n) {
    f32x4 v = s_part[0][ln];
#pragma unroll
    for (int k = 1; k < 8; ++k) v += s_part[k][ln];
    const size_t per_b = (size_t)p.Hq * p.d;
    const size_t o = (i / per_b) * p.q_bstride + (i % per_b);
    store_elem((elem*)p.out, o + 0, v.x);
    store_elem((elem*)p.out, o + 1, v.y);
    store_elem((elem*)p.out, o + 2, v.z);
    store_elem((elem*)p.out, o + 3, v.w);
  }
}

// ------------------------------------------------------------------ fill / copy

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* dst, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride)
    dst[i] = (u32x4){0u, 0u, 0u, 0u};
}

// A visit of a workgroup covers 16 KB: four 16-byte vectors per lane, all four loads issued before the
// first store, consecutive lanes on consecutive vectors (the access shape of the MV pass).
__global__ __launch_bounds__(256) void copy_kernel(u32x4* dst, const u32x4* src, size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * 1024;
  for (size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x; base < n_vec; base += stride) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (base + u * 256 < n_vec) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (base + u * 256 < n_vec) __builtin_nontemporal_store(v[u], dst + base + u * 256);
  }
}

// MV := amplitude * u, u uniform on the 2^24-point grid of [-1, 1): element i of the flat array takes
// the (i + 1)-th output of the splitmix64 generator started at `seed` (counter-based, so any thread
// can produce any element), its top 24 bits as a signed grid index.  Integer steps are exact, the
// two floating-point steps are single IEEE roundings: the values do not depend on the machine.
template <typename DT>
__global__ __launch_bounds__(256) void randomize_kernel(u32x4* dst, size_t n_vec, uint64_t seed, float amplitude) {
  constexpr int E = DT::kElemsPerVec;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride) {
    float f[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
      uint64_t z = seed + (uint64_t)(i * E + e + 1) * 0x9E3779B97F4A7C15ull;
      z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
      z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
      z ^= z >> 31;
      f[e] = (float)((int32_t)(z >> 40) - (1 << 23)) * (1.0f / 8388608.0f) * amplitude;
    }
    dst[i] = pack16_round<DT>(f);
  }
}

// ------------------------------------------------------------------ host side

static bool use_mfma_scores(const DecodeParams& p, int dtype) { return dtype == 1 && !p.mk_per_seq; }

void plan_decode(DecodeParams& p, int dtype) {
  if (use_mfma_scores(p, dtype)) {
    // the largest slot tile per wavefront that still gives one wavefront per
    // SIMD (1024 on the chip); measured at H=32, M=4096, 64 rows: 128 slots
    // 19 us, 64 slots 21 us, 32 slots 26 us (two launches' overhead included)
    uint32_t nt = 1;
    if (p.M % 128 == 0 && (uint64_t)(p.M / 128) * p.Hkv >= 1024) nt = 4;
    else if ((uint64_t)(p.M / 64) * p.Hkv >= 1024) nt = 2;
    p.stat_tile = 32 * nt;
  } else {
    p.stat_tile = 64;
  }
  p.n_tiles = p.M / p.stat_tile;
  plan_mv_pass(p, dtype);
  p.fused = (p.M <= kFusedMaxM && (uint64_t)p.B * p.Hkv <= kFusedMaxUnits) ? 1u : 0u;
}

template <int D, int NT>
static hipError_t launch_scores_mfma(const DecodeParams& p, hipStream_t s) {
  const uint32_t tiles = p.M / (32 * NT);
  const uint32_t rbs = (p.B * p.R + 31) / 32;
  uint32_t z = 1;
  const uint64_t waves = (uint64_t)tiles * p.Hkv;
  if (waves < 1024) z = (uint32_t)((1024 + waves - 1) / waves);
  if (z > rbs) z = rbs;
  hipLaunchKernelGGL((scores_mfma_bf16_kernel<D, NT>), dim3(tiles, p.Hkv, z), dim3(64), 0, s, p);
  return hipGetLastError();
}

// RT: the score rows of a memory the instantiation has registers for (write + read queries)
template <typename DT, int D>
static void launch_scores_generic(const DecodeParams& p, dim3 grid, hipStream_t s) {
  if (p.R <= 2) hipLaunchKernelGGL((scores_generic_kernel<DT, D, 2>), grid, dim3(256), 0, s, p);
  else if (p.R <= 3) hipLaunchKernelGGL((scores_generic_kernel<DT, D, 3>), grid, dim3(256), 0, s, p);
  else if (p.R <= 5) hipLaunchKernelGGL((scores_generic_kernel<DT, D, 5>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((scores_generic_kernel<DT, D, (int)kMaxRows>), grid, dim3(256), 0, s, p);
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
  const dim3 grid = unit_grid(p.M / 64, (uint64_t)p.B * p.Hkv);
  if (dtype == 0) {
    if (p.d == 128) launch_scores_generic<F32, 128>(p, grid, s);
    else launch_scores_generic<F32, 64>(p, grid, s);
  } else {
    if (p.d == 128) launch_scores_generic<BF16, 128>(p, grid, s);
    else launch_scores_generic<BF16, 64>(p, grid, s);
  }
  return hipGetLastError();
}

hipError_t launch_normalise(const DecodeParams& p, hipStream_t s) {
  if (p.fuse_norm) return hipSuccess;  // the MV pass does it
  const uint32_t rows = p.B * p.Hkv * p.R;
  hipLaunchKernelGGL(normalise_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_merge(const DecodeParams& p, int dtype, hipStream_t s) {
  if (!p.has_read || p.S == 1) return hipSuccess;
  const size_t n = (size_t)p.B * p.Hq * p.d;
  const dim3 grid((unsigned)((n + 127) / 128)), block(256);
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

hipError_t launch_randomize(void* dst, size_t n_bytes, int dtype, uint64_t seed, float amplitude, hipStream_t s) {
  const size_t n_vec = n_bytes / 16;
  if (n_vec == 0) return hipSuccess;
  if (dtype == 0)
    hipLaunchKernelGGL((randomize_kernel<F32>), dim3(grid_for(n_vec)), dim3(256), 0, s, (u32x4*)dst, n_vec, seed,
                       amplitude);
  else
    hipLaunchKernelGGL((randomize_kernel<BF16>), dim3(grid_for(n_vec)), dim3(256), 0, s, (u32x4*)dst, n_vec, seed,
                       amplitude);
  return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t n_bytes, hipStream_t s) {
  const size_t n_vec = n_bytes / 16;
  if (n_vec == 0) return hipSuccess;
  size_t blocks = (n_vec + 1023) / 1024;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (u32x4*)dst, (const u32x4*)src, n_vec);
  return hipGetLastError();
}

}  // namespace bct
