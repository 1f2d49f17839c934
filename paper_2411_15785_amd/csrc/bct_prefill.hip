// Chunked prefill of libbct for bf16 caches (gfx950, MFMA).
//
// A chunk of T tokens is T decode steps in token order with MV carried in fp32
// through the chunk.  Because MK is static, the write weights ww_t do not
// depend on MV, so the recurrence unrolls into dense contractions (section 3.5,
// "Optimized for Parallelism": the per-token updates are independent and can be
// accumulated concurrently):
//     WW = softmax_rows(write_scale * WQ . MK^T)   [T x M]
//     RW = softmax_rows(read_scale  * Q  . MK^T)   [T*G x M]
//     MV_end   = round(MV_start + WW^T . WV)                       (section 3.4 eq., summed over t)
//     out_t    = RW_t . (MV_start + sum_{s<=t} ww_s^T wv_s)         (read after the token's own write)
// Tokens are grouped in sub-chunks of 128.  For sub-chunk c,
//     out_c = RW_c . MV_c + tril(RW_c . WW_c^T) . WV_c,   MV_c = MV at the start of the sub-chunk,
// where the state kernel, which walks the sub-chunks in order with its MV tile
// in fp32 registers, leaves MV_c (rounded to bf16, as an MFMA operand has to be)
// in the workspace.  Launches: transpose (WV) -> stats (write rows) -> state -> read (all
// sub-chunks, the read rows normalised on the fly); a chunk that only reads: transpose (MV) -> stats
// (read rows) -> read.
//
// All matrix products use v_mfma_f32_32x32x16_bf16 with both operands read from
// LDS tiles whose rows run along the contraction index (C[i][j] += sum_k
// A[i][k] B[j][k]); the two operands whose memory layout runs the other way
// (MV over slots, WV over tokens) are transposed once per chunk into the
// workspace, and the MV snapshots are written transposed in the first place.  Rows are padded by 16 bytes so that the 32
// lanes of an operand read fall into different banks.  The accumulator of lane
// l holds column j = l % 32 and rows i = 8*(v/4) + 4*(l/32) + v%4; each product
// is oriented so that a lane's four consecutive v run along the NEXT product's
// contraction index and can be written to LDS as one 8-byte store.
//
// Precision: scores in fp32 from exact bf16 products; softmax weights are
// rounded to bf16 as MFMA operands for the reads; for the state they are split
// into hi + lo bf16 parts (two MFMAs) so that the stored MV carries fp32-grade
// weights like the decode step does.
#include "bct_device.h"
#include "bct_internal.h"

namespace bct {

namespace {

constexpr int kTC = 128;          // tokens per sub-chunk = rows per tile
constexpr float kNegBig = -1e30f;  // stands in for -inf in running maxima
constexpr float kNoRow = 1e30f;    // shift of a row that does not exist: exp2(score - kNoRow) = 0

__device__ __forceinline__ f32x16 mfma_bf16(const bf16x8 a, const bf16x8 b, const f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 frag(const uint16_t* tile, int ld, int row, int k) {
  return *(const bf16x8*)(tile + row * ld + k);
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int v = 0; v < 16; ++v) z[v] = 0.f;
  return z;
}
__device__ __forceinline__ uint16_t bf16_bits(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }
__device__ __forceinline__ float bf16_val(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Global -> LDS tile copies in two halves, so that the loads of the next tile
// can be in flight while the current one is used: fetch() issues all of a
// thread's 16-byte loads into registers, put() writes them to LDS.
// A tile is NROWS rows of NCOLS bf16; thread t handles 16-byte chunk t % CPR of
// rows t / CPR, t / CPR + RPP, ... of a workgroup of NT threads
template <int NROWS, int NCOLS, int NT = 256>
struct Tile {
  static constexpr int CPR = NCOLS / 8, RPP = NT / CPR, N = NROWS / RPP;
  static_assert(NROWS % RPP == 0, "whole passes");
  u32x4 v[N];
  uint32_t missing = 0;  // bit i: row i of this thread is a zero row

  // rowptr(r): address of row r, or nullptr for a zero row.  A missing row is a
  // load from `safe` (any valid 16-byte aligned address) whose result put()
  // replaces by zeros: the loads carry no branches, and nothing touches the
  // loaded registers until put(), so the loads stay in flight across the
  // products of the current tile.
  template <typename F>
  __device__ __forceinline__ void fetch_rows(const uint16_t* safe, F rowptr) {
    const int ch = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
    missing = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const uint16_t* src = rowptr(r0 + i * RPP);
      const bool ok = src != nullptr;
      v[i] = *(const u32x4*)((ok ? src : safe) + (ok ? ch * 8 : 0));
      missing |= ok ? 0u : (1u << i);
    }
  }
  // the same for data read once (past the caches, so that it does not push out what is reused)
  __device__ __forceinline__ void fetch_block_once(const uint16_t* src, size_t src_ld) {
    const int ch = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
#pragma unroll
    for (int i = 0; i < N; ++i)
      v[i] = __builtin_nontemporal_load((const u32x4*)(src + (size_t)(r0 + i * RPP) * src_ld + ch * 8));
    missing = 0;
  }
  // rows at src + r * src_ld, all present
  __device__ __forceinline__ void fetch_block(const uint16_t* src, size_t src_ld) {
    const int ch = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = *(const u32x4*)(src + (size_t)(r0 + i * RPP) * src_ld + ch * 8);
    missing = 0;
  }
  __device__ __forceinline__ void put(uint16_t* dst, int ld) const {
    const int ch = threadIdx.x % CPR, r0 = threadIdx.x / CPR;
#pragma unroll
    for (int i = 0; i < N; ++i)
      *(u32x4*)(dst + (r0 + i * RPP) * ld + ch * 8) = ((missing >> i) & 1u) ? (u32x4){0u, 0u, 0u, 0u} : v[i];
  }
};
template <int D, int NROWS, typename F>
__device__ __forceinline__ void rows_to_lds(uint16_t* dst, int ld, const uint16_t* safe, F rowptr) {
  Tile<NROWS, D> t;
  t.fetch_rows(safe, rowptr);
  t.put(dst, ld);
}
template <int NROWS, int NCOLS>
__device__ __forceinline__ void block_to_lds(uint16_t* dst, int ld, const uint16_t* src, size_t src_ld) {
  Tile<NROWS, NCOLS> t;
  t.fetch_block(src, src_ld);
  t.put(dst, ld);
}
__device__ __forceinline__ void store4_bf16(uint16_t* dst, float a, float b, float c, float d) {
  uint2 w;
  w.x = pack_bf16x2(a, b);
  w.y = pack_bf16x2(c, d);
  *(uint2*)dst = w;
}

__device__ __forceinline__ void merge_stat(float& m, float& s, float mo, float so) {
  const float mn = fmaxf(m, mo);
  s = s * fast_exp2(m - mn) + so * fast_exp2(mo - mn);
  m = mn;
}

}  // namespace

// ------------------------------------------------------------------ transposes

// MFMA operands must run along the contraction index, and two of them do not
// in memory: WV [token][column] is contracted over tokens and MV [slot][column]
// over slots.  This kernel writes the transposed copies once per chunk:
//   which = 0:  WVt[unit][column][token]  (tokens >= T zero-filled up to Tpad)
//   which = 1:  snap[0][unit][column][slot] = MV at the start of the chunk
// One workgroup transposes 64 rows through LDS.
template <int D>
__global__ __launch_bounds__(256) void prefill_transpose_kernel(const PrefillParams p, int which) {
  constexpr int LD = D + 8;
  __shared__ __attribute__((aligned(16))) uint16_t sT[64 * LD];
  const uint32_t unit = block_unit();
  if (unit >= p.B * p.Hkv) return;
  const uint32_t b = unit / p.Hkv, h = unit % p.Hkv;
  const uint32_t r0 = blockIdx.x * 64;
  const uint32_t rows = which == 0 ? p.Tpad : p.M;
  rows_to_lds<D, 64>(sT, LD, p.mv, [&](int r) -> const uint16_t* {
    if (which == 0) return r0 + r < p.T ? p.wv + (((size_t)b * p.T + r0 + r) * p.Hkv + h) * D : nullptr;
    return p.mv + ((size_t)unit * p.M + r0 + r) * D;
  });
  __syncthreads();
  uint16_t* dst = (which == 0 ? p.wvt : p.snap) + (size_t)unit * D * rows + r0;
  // A negative step size eta_t (section 3.5 reading: MV += eta_t ww^T wv) flips the sign of token t's row of
  // WV here, which is exact; the statistics kernel folds |eta_t| into the token's shift.  A thread's 8 rows
  // are the same in every pass of the loop below (256 is a multiple of 8).
  u32x4 flip = {0u, 0u, 0u, 0u};
  if (which == 0 && p.gate) {
    const uint32_t t8 = r0 + (threadIdx.x % 8) * 8;
    uint32_t sg[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
      sg[k] = (t8 + k < p.T && p.gate[((size_t)b * p.T + t8 + k) * p.Hkv + h] < 0.f) ? 0x8000u : 0u;
    flip = (u32x4){sg[0] | (sg[1] << 16), sg[2] | (sg[3] << 16), sg[4] | (sg[5] << 16), sg[6] | (sg[7] << 16)};
  }
  // thread -> (column j, 8 consecutive rows)
  for (int i = threadIdx.x; i < D * 8; i += 256) {
    const int j = i / 8, rr = (i % 8) * 8;
    u32x4 v;
    v.x = (uint32_t)sT[(rr + 0) * LD + j] | ((uint32_t)sT[(rr + 1) * LD + j] << 16);
    v.y = (uint32_t)sT[(rr + 2) * LD + j] | ((uint32_t)sT[(rr + 3) * LD + j] << 16);
    v.z = (uint32_t)sT[(rr + 4) * LD + j] | ((uint32_t)sT[(rr + 5) * LD + j] << 16);
    v.w = (uint32_t)sT[(rr + 6) * LD + j] | ((uint32_t)sT[(rr + 7) * LD + j] << 16);
    *(u32x4*)(dst + (size_t)j * rows + rr) = v ^ flip;
  }
}

// ------------------------------------------------------------------ stats

// Row statistics of the score matrix: for each write row (token t) and read
// row (token t, query head g) of a memory, the shift max + log2(sum of
// exp2(score - max)) over all M slots, so that a weight is exp2(score - shift)
// with no further multiplication (stored in .x of a float2; rows that do not
// exist use kNoRow, which makes every weight zero).  One workgroup = 128 rows;
// it walks the keys 128 slots at a time; each of its eight wavefronts scores
// 32 slots of the tile against 64 of the rows.
template <int D>
__global__ __launch_bounds__(512, 4) void prefill_stats_kernel(const PrefillParams p) {
  constexpr int LD = D + 8, KS = D / 16, NT = 512;
  // the query tile is only read into registers before the loop: the key tiles reuse its memory
  __shared__ __attribute__((aligned(16))) uint16_t sTile[128 * LD];
  __shared__ float2 sRed[4][kTC];
  uint16_t* const sX = sTile;
  uint16_t* const sK = sTile;

  // launch order: all sequences of one KV head, then the next head, so that the workgroups in flight
  // share one head's keys (1 MB at M = 4096) in each XCD's L2 instead of cycling through all heads
  const uint32_t uy = block_unit();
  if (uy >= p.B * p.Hkv) return;
  const uint32_t h = uy / p.B, b = uy % p.B, unit = b * p.Hkv + h;
  const uint32_t nw = p.has_write ? p.T : 0u, nr = (p.has_read && p.stats_read) ? p.T * p.G : 0u;
  const uint32_t row0 = blockIdx.x * kTC;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  // wavefront = (32 slots sg of the key tile, 64 rows rh of the row tile)
  const int sg = wave & 3, rh = wave >> 2;

  {
    Tile<kTC, D, NT> t;
    t.fetch_rows(p.mk, [&](int r) -> const uint16_t* {
      uint32_t row = row0 + r;
      if (row < nw) return p.wq + (((size_t)b * p.T + row) * p.Hkv + h) * D;
      row -= nw;
      if (row < nr) return p.q + (((size_t)b * p.T + row / p.G) * p.Hq + h * p.G + row % p.G) * D;
      return nullptr;
    });
    t.put(sX, LD);
  }
  const uint16_t* mk = p.mk + (size_t)(p.mk_per_seq ? unit : h) * p.M * D;

  float scale[2], m[2], s[2];
#pragma unroll
  for (int jt = 0; jt < 2; ++jt) {
    scale[jt] = (row0 + 64 * rh + 32 * jt + col < nw) ? p.wscale_l2e : p.rscale_l2e;
    m[jt] = kNegBig;
    s[jt] = 0.f;
  }
  // the query rows do not change over the loop: keep their operand fragments in registers.
  // A negative scale is moved into the row itself (negating bf16 is exact), so that below the
  // largest raw score is also the largest scaled one and the scaling can ride in the exponent's fma.
  __syncthreads();
  bf16x8 xb[2][KS];
#pragma unroll
  for (int jt = 0; jt < 2; ++jt) {
    const uint32_t flip = scale[jt] < 0.f ? 0x80008000u : 0u;
    scale[jt] = fabsf(scale[jt]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 v = __builtin_bit_cast(u32x4, frag(sX, LD, 64 * rh + 32 * jt + col, ks * 16 + half * 8));
      v ^= (u32x4){flip, flip, flip, flip};
      xb[jt][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }
  Tile<128, D, NT> tk;
  auto fetch_keys = [&](uint32_t m0) {
    tk.fetch_rows(p.mk, [&](int r) -> const uint16_t* { return (m0 + r < p.M) ? mk + (size_t)(m0 + r) * D : nullptr; });
  };
  fetch_keys(0);
  for (uint32_t m0 = 0; m0 < p.M; m0 += 128) {
    __syncthreads();
    tk.put(sK, LD);
    if (m0 + 128 < p.M) fetch_keys(m0 + 128);  // in flight during this tile's products
    __syncthreads();
    if (m0 + 32 * sg < p.M) {  // M is a multiple of 64: a wavefront's 32 slots are all in or all out
      f32x16 acc[2];
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) acc[jt] = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a = frag(sK, LD, 32 * sg + col, ks * 16 + half * 8);
#pragma unroll
        for (int jt = 0; jt < 2; ++jt) acc[jt] = mfma_bf16(a, xb[jt][ks], acc[jt]);
      }
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) {
        float tmax = acc[jt][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[jt][v]);
        const float mn = fmaxf(m[jt], tmax * scale[jt]);
        float add = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) add += fast_exp2(__builtin_fmaf(acc[jt][v], scale[jt], -mn));
        s[jt] = s[jt] * fast_exp2(m[jt] - mn) + add;
        m[jt] = mn;
      }
    }
  }
#pragma unroll
  for (int jt = 0; jt < 2; ++jt) {
    merge_stat(m[jt], s[jt], __shfl_xor(m[jt], 32, 64), __shfl_xor(s[jt], 32, 64));
    if (half == 0) sRed[sg][64 * rh + 32 * jt + col] = make_float2(m[jt], s[jt]);
  }
  __syncthreads();
  if (threadIdx.x < kTC) {
    float mm = sRed[0][threadIdx.x].x, ss = sRed[0][threadIdx.x].y;
#pragma unroll
    for (int w = 1; w < 4; ++w) merge_stat(mm, ss, sRed[w][threadIdx.x].x, sRed[w][threadIdx.x].y);
    uint32_t row = row0 + threadIdx.x;
    if (row < nw) {
      // a step size eta scales the token's write weights: exp2(score - shift) * |eta|
      // = exp2(score - (shift - log2 |eta|)); eta = 0 gives shift = +inf and weights 0
      // (|eta| here; the sign of eta rides on the token's row of WV^T, see prefill_transpose_kernel)
      const float le = p.gate ? __log2f(fabsf(p.gate[((size_t)b * p.T + row) * p.Hkv + h])) : 0.f;
      p.norm_w[(size_t)unit * p.T + row] = make_float2(mm + __log2f(ss) - le, 0.f);
    } else if (row - nw < nr) {
      p.norm_r[(size_t)unit * p.T * p.G + (row - nw)] = make_float2(mm + __log2f(ss), 0.f);
    }
  }
}

// ------------------------------------------------------------------ read of a chunk that does not write

// Output rows of one tile of 128 read rows (row rho of the tile = token rho / G, query head rho % G)
// when MV does not change over the chunk:  out = RW . MV,  with the rows' shifts from the statistics
// kernel.  The workgroup walks the M slots 64 at a time, recomputing the score tiles.  Eight wavefronts:
// for the scores each takes 32 rows x 32 slots of the tile, for the product 32 output rows x d/2 value
// columns.
template <int D>
__global__ __launch_bounds__(512) void prefill_read_only_kernel(const PrefillParams p) {
  constexpr int NT = 512;
  constexpr int LD = D + 8, KS = D / 16;
  constexpr int LP = 64 + 8;    // row length of tiles contracted over 64 slots
  __shared__ __attribute__((aligned(16))) uint16_t sXr[kTC * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sBuf[64 * LD + D * LP + kTC * LP];
  uint16_t* const sK = sBuf;
  uint16_t* const sVt = sK + 64 * LD;
  uint16_t* const sPr = sVt + D * LP;

  // launch order: all sequences of one KV head, then the next head, so that the workgroups in flight
  // share one head's keys (1 MB at M = 4096) in each XCD's L2 instead of cycling through all heads
  const uint32_t uy = block_unit();
  if (uy >= p.B * p.Hkv) return;
  const uint32_t h = uy / p.B, b = uy % p.B, unit = b * p.Hkv + h;
  const uint32_t G = p.G, T = p.T;
  const uint32_t c = p.c_begin + blockIdx.x / G, gp = blockIdx.x % G;
  const uint32_t t0 = c * kTC, rho0 = gp * kTC;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;

  {
    Tile<kTC, D, NT> t;
    t.fetch_rows(p.mk, [&](int r) -> const uint16_t* {
      const uint32_t rho = rho0 + r, tk = t0 + rho / G;
      return tk < T ? p.q + (((size_t)b * T + tk) * p.Hq + h * G + rho % G) * D : nullptr;
    });
    t.put(sXr, LD);
  }
  const uint16_t* mk = p.mk + (size_t)(p.mk_per_seq ? unit : h) * p.M * D;
  const uint16_t* mvt = p.snap + (size_t)unit * p.M * D;   // MV, transposed: [column][slot]

  // score step: wavefront = (slot half si, row group rj of 32); lane column = row
  const int si = wave & 1, rj = wave >> 1;
  float nrm_r;
  {
    const uint32_t rho = rho0 + 32 * rj + col, t = t0 + rho / G;
    nrm_r = t < T ? p.norm_r[(size_t)unit * T * G + (size_t)t * G + rho % G].x : kNoRow;
  }
  // product step: wavefront = (32 output rows, half of the value columns)
  constexpr int NOC = D / 64;                      // 32-column tiles per wavefront in the output product
  const int orow = 32 * (wave & 3), ocol = 32 * NOC * (wave >> 2);
  f32x16 oacc[NOC];
#pragma unroll
  for (int jt = 0; jt < NOC; ++jt) oacc[jt] = zero16();

  // the query rows do not change over the loop: keep their operand fragments in registers
  __syncthreads();
  bf16x8 xr[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) xr[ks] = frag(sXr, LD, 32 * rj + col, ks * 16 + half * 8);
  Tile<64, D, NT> tk;
  Tile<D, 64, NT> tv;
  tk.fetch_block(mk, D);
  tv.fetch_block(mvt, p.M);
  for (uint32_t m0 = 0; m0 < p.M; m0 += 64) {
    __syncthreads();
    tk.put(sK, LD);
    tv.put(sVt, LP);
    if (m0 + 64 < p.M) {  // next tiles, in flight during this tile's products
      tk.fetch_block(mk + (size_t)(m0 + 64) * D, D);
      tv.fetch_block(mvt + m0 + 64, p.M);
    }
    __syncthreads();
    {
      f32x16 sr = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) sr = mfma_bf16(frag(sK, LD, 32 * si + col, ks * 16 + half * 8), xr[ks], sr);
      const int r = 32 * rj + col;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float e[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) e[i] = fast_exp2(sr[4 * q4 + i] * p.rscale_l2e - nrm_r);
        store4_bf16(sPr + r * LP + 32 * si + 8 * q4 + 4 * half, e[0], e[1], e[2], e[3]);
      }
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int k = ks * 16 + half * 8;
      const bf16x8 a = frag(sPr, LP, orow + col, k);
#pragma unroll
      for (int jt = 0; jt < NOC; ++jt) oacc[jt] = mfma_bf16(a, frag(sVt, LP, ocol + 32 * jt + col, k), oacc[jt]);
    }
  }

#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const uint32_t r = orow + 8 * (v / 4) + 4 * half + (v % 4);
    const uint32_t rho = rho0 + r, t = t0 + rho / G;
    if (t < T) {
      uint16_t* o = p.out + (((size_t)b * T + t) * p.Hq + h * G + rho % G) * D;
#pragma unroll
      for (int jt = 0; jt < NOC; ++jt) o[ocol + 32 * jt + col] = bf16_bits(oacc[jt][v]);
    }
  }
}

// ------------------------------------------------------------------ read of a chunk that writes

// The read of a chunk that also writes, without a statistics pass over the read rows: the softmax of a
// read row is normalised at the end, out = (sum_m e_m MV_c[m] + sum_s A'[s] wv_s) / sum_m e_m with
// e_m = exp2(score_m - shift), and the shift follows the row's running maximum lazily - it moves only
// when a tile's maximum exceeds it by more than kTau (the weights then reach at most 2^kTau, far inside
// bf16 and fp32 range), which after the first tile is rare, so rescaling what has been accumulated is a
// seldom-taken, workgroup-uniform branch.  The write rows keep their shifts from the statistics kernel
// (the state kernel needs those before it can add anything to MV).
// Output rows of one tile of 128 read rows of sub-chunk c:
//     out = RW . MV_c  +  mask(RW . WW_c^T) . WV_c ,  mask: write token s <= the row's token.
// The workgroup walks the M slots 64 at a time, recomputing the score tiles.  Eight wavefronts.
// Score step: wavefront = (role, row group of 32): role 0 scores 32 read rows, role 1 32 write tokens,
// against all 64 slots of the tile, so a row's tile maximum and its sum are in two lanes.  Product step:
// 32 output rows x d/2 value columns and 32 write tokens x 64 read rows of the within-sub-chunk
// matrix; that keeps a lane under 256 registers, so two wavefronts share a SIMD.
template <int D>
__global__ __launch_bounds__(512) void prefill_read_online_kernel(const PrefillParams p) {
  constexpr int NT = 512;
  constexpr int LD = D + 8, KS = D / 16;
  constexpr int LP = 64 + 8;    // row length of tiles contracted over 64 slots
  constexpr int LA = kTC + 8;   // row length of tiles contracted over 128 tokens
  constexpr float kTau = 8.f;
  constexpr int kLoop = 64 * LD + D * LP + 2 * kTC * LP;  // sK, sVt, sPr, sPw
  constexpr int kTail = kTC * LA + D * LA;                // sA, sWVt
  constexpr int kRows = 2 * kTC * LD;                     // sXr, sXw
  constexpr int kSet = kLoop > kTail ? (kLoop > kRows ? kLoop : kRows) : (kTail > kRows ? kTail : kRows);
  // Two sets of the loop's tiles, used in turn, so that a wavefront can be a step ahead of the others
  // (one barrier per slot tile, see the loop).  The row tiles are only read into registers before the
  // loop and share the second set's memory; the tiles of the tail share the first set's.
  __shared__ __attribute__((aligned(16))) uint16_t sBuf[2][kSet];
  __shared__ float sScale[2][kTC];  // per read row: this tile's rescaling factor; at the end ([0]) 1 / sum
  __shared__ uint32_t sFlag[3];     // slot tile number % 3 -> some row's shift moved in that tile
  uint16_t* const sXr = sBuf[1];
  uint16_t* const sXw = sBuf[1] + kTC * LD;
  uint16_t* const sA = sBuf[0];
  uint16_t* const sWVt = sA + kTC * LA;

  // launch order: all sequences of one KV head, then the next head (shared keys stay in L2)
  const uint32_t uy = block_unit();
  if (uy >= p.B * p.Hkv) return;
  const uint32_t h = uy / p.B, b = uy % p.B, unit = b * p.Hkv + h;
  const uint32_t G = p.G, T = p.T;
  const uint32_t c = p.c_begin + blockIdx.x / G, gp = blockIdx.x % G;
  const uint32_t t0 = c * kTC, rho0 = gp * kTC;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const size_t units = (size_t)p.B * p.Hkv;

  {
    Tile<kTC, D, NT> t;
    t.fetch_rows(p.mk, [&](int r) -> const uint16_t* {
      const uint32_t rho = rho0 + r, tk = t0 + rho / G;
      return tk < T ? p.q + (((size_t)b * T + tk) * p.Hq + h * G + rho % G) * D : nullptr;
    });
    t.put(sXr, LD);
  }
  {
    Tile<kTC, D, NT> t;
    t.fetch_rows(p.mk, [&](int r) -> const uint16_t* {
      return t0 + r < T ? p.wq + (((size_t)b * T + t0 + r) * p.Hkv + h) * D : nullptr;
    });
    t.put(sXw, LD);
  }
  if (threadIdx.x < 3) sFlag[threadIdx.x] = 0u;
  const uint16_t* mk = p.mk + (size_t)(p.mk_per_seq ? unit : h) * p.M * D;
  const uint16_t* mvt = p.snap + ((size_t)c * units + unit) * p.M * D;   // MV_c, transposed: [column][slot]

  // score step: role 0 = read rows, role 1 = write tokens; row (token) 32 * rg + col of the tile
  const int role = wave >> 2, rg = wave & 3;
  const int srow = 32 * rg + col;
  float cs = role == 0 ? p.rscale_l2e : p.wscale_l2e;   // scale of this wavefront's rows (log2 domain)
  // role 0: the lazily followed running maximum of the row (scaled); role 1: the token's fixed shift
  float shift = kNegBig, zsum = 0.f;
  if (role == 1) shift = (t0 + srow < T) ? p.norm_w[(size_t)unit * T + t0 + srow].x : kNoRow;
  // product step: wavefront = (32 output rows, half of the value columns) and, for the
  // within-sub-chunk matrix, (32 write tokens, 64 read rows)
  constexpr int NOC = D / 64;
  const int orow = 32 * (wave & 3), ocol = 32 * NOC * (wave >> 2);
  const int as0 = 32 * (wave & 3), ar0 = 64 * (wave >> 2);
  f32x16 oacc[NOC], aacc[2];
#pragma unroll
  for (int jt = 0; jt < NOC; ++jt) oacc[jt] = zero16();
#pragma unroll
  for (int jt = 0; jt < 2; ++jt) aacc[jt] = zero16();

  // this wavefront's rows as operand fragments, kept in registers.  A negative read scale moves into the
  // row (negating bf16 is exact), so that the largest raw score is also the largest scaled one.
  __syncthreads();
  bf16x8 x[KS];
  {
    const uint32_t flip = (role == 0 && cs < 0.f) ? 0x80008000u : 0u;
    if (role == 0) cs = fabsf(cs);
    const uint16_t* sX = role == 0 ? sXr : sXw;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 v = __builtin_bit_cast(u32x4, frag(sX, LD, srow, ks * 16 + half * 8));
      v ^= (u32x4){flip, flip, flip, flip};
      x[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }
  // One barrier per slot tile.  Tile i uses set i % 2 of the buffers:
  //   before the barrier: the keys of tile i + 1 go to the other set (its keys were last read in the
  //     score step of tile i - 1, which every wavefront finished before the previous barrier); scores of
  //     tile i from this set's keys -> this set's weights (last read in the product step of tile i - 2);
  //   after the barrier: the values of tile i + 1 go to the other set (last read in the product step
  //     of tile i - 1, which every wavefront left before it arrived at this barrier); products of tile i.
  // So the wavefronts drift up to a step apart, and one's exponentials overlap another's products.
  Tile<64, D, NT> tk;
  Tile<D, 64, NT> tv;
  auto next_values = [&](uint32_t m) {
    if (G == 1) tv.fetch_block_once(mvt + m, p.M);   // nobody else reads this copy of MV
    else tv.fetch_block(mvt + m, p.M);
  };
  tk.fetch_block(mk, D);
  next_values(0);
  __syncthreads();             // the row fragments are in registers: the second set is free
  tk.put(sBuf[0], LD);
  tv.put(sBuf[0] + 64 * LD, LP);
  if (64 < p.M) {
    tk.fetch_block(mk + (size_t)64 * D, D);
    next_values(64);
  }
  uint32_t it = 0;
  for (uint32_t m0 = 0; m0 < p.M; m0 += 64, ++it) {
    uint16_t* const sK = sBuf[it & 1];
    uint16_t* const sVt = sK + 64 * LD;
    uint16_t* const sPr = sVt + D * LP;
    uint16_t* const sPw = sPr + kTC * LP;
    uint16_t* const sKn = sBuf[(it + 1) & 1];
    float* const sSc = sScale[it & 1];
    const uint32_t fl = it % 3;
    if (m0 + 64 < p.M) {
      tk.put(sKn, LD);
      if (m0 + 128 < p.M) tk.fetch_block(mk + (size_t)(m0 + 128) * D, D);
    }
    if (threadIdx.x == 0) sFlag[(it + 1) % 3] = 0u;   // last read in the product step of tile i - 2
    if (it == 0) __syncthreads();                     // the first tile's keys were staged just above
    {
      f32x16 s0 = zero16(), s1 = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s0 = mfma_bf16(frag(sK, LD, col, ks * 16 + half * 8), x[ks], s0);
        s1 = mfma_bf16(frag(sK, LD, 32 + col, ks * 16 + half * 8), x[ks], s1);
      }
      if (role == 0) {
        float tm = fmaxf(s0[0], s1[0]);
#pragma unroll
        for (int v = 1; v < 16; ++v) tm = fmaxf(tm, fmaxf(s0[v], s1[v]));
        tm = fmaxf(tm, __shfl_xor(tm, 32, 64)) * cs;
        float f = 1.f;
        if (tm > shift + kTau) {        // also the first tile (shift = kNegBig: f = 0, nothing accumulated yet)
          f = fast_exp2(shift - tm);
          shift = tm;
          zsum *= f;
          sFlag[fl] = 1u;
        }
        if (half == 0) sSc[srow] = f;
        float add = 0.f;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          float e0[4], e1[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            e0[i] = fast_exp2(__builtin_fmaf(s0[4 * q4 + i], cs, -shift));
            e1[i] = fast_exp2(__builtin_fmaf(s1[4 * q4 + i], cs, -shift));
            add += e0[i] + e1[i];
          }
          store4_bf16(sPr + srow * LP + 8 * q4 + 4 * half, e0[0], e0[1], e0[2], e0[3]);
          store4_bf16(sPr + srow * LP + 32 + 8 * q4 + 4 * half, e1[0], e1[1], e1[2], e1[3]);
        }
        zsum += add;
      } else {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          float e0[4], e1[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            e0[i] = fast_exp2(__builtin_fmaf(s0[4 * q4 + i], cs, -shift));
            e1[i] = fast_exp2(__builtin_fmaf(s1[4 * q4 + i], cs, -shift));
          }
          store4_bf16(sPw + srow * LP + 8 * q4 + 4 * half, e0[0], e0[1], e0[2], e0[3]);
          store4_bf16(sPw + srow * LP + 32 + 8 * q4 + 4 * half, e1[0], e1[1], e1[2], e1[3]);
        }
      }
    }
    __syncthreads();
    if (m0 + 64 < p.M) {
      tv.put(sKn + 64 * LD, LP);
      if (m0 + 128 < p.M) next_values(m0 + 128);
    }
    if (sFlag[fl]) {   // uniform over the workgroup: bring what has been accumulated to the new shifts
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float fr = sSc[orow + 8 * (v / 4) + 4 * half + (v % 4)];
#pragma unroll
        for (int jt = 0; jt < NOC; ++jt) oacc[jt][v] *= fr;
      }
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) {
        const float fc = sSc[ar0 + 32 * jt + col];
#pragma unroll
        for (int v = 0; v < 16; ++v) aacc[jt][v] *= fc;
      }
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int k = ks * 16 + half * 8;
      const bf16x8 a = frag(sPr, LP, orow + col, k);
#pragma unroll
      for (int jt = 0; jt < NOC; ++jt) oacc[jt] = mfma_bf16(a, frag(sVt, LP, ocol + 32 * jt + col, k), oacc[jt]);
      // rows of this product = write tokens s, columns = read rows
      const bf16x8 aw = frag(sPw, LP, as0 + col, k);
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) aacc[jt] = mfma_bf16(aw, frag(sPr, LP, ar0 + 32 * jt + col, k), aacc[jt]);
    }
  }

  __syncthreads();
  // 1 / (sum of the row's weights): the normaliser of everything accumulated for the row
  if (role == 0) {
    const float z = zsum + __shfl_xor(zsum, 32, 64);
    if (half == 0) sScale[0][srow] = 1.0f / z;
  }
  // A[row][s] = (s <= token of the row) ? sum_m e[row][m] ww[s][m] : 0
#pragma unroll
  for (int jt = 0; jt < 2; ++jt) {
    const int r = ar0 + 32 * jt + col;
    const int tl = (int)((rho0 + r) / G);  // the row's token within the sub-chunk
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int s0 = as0 + 8 * q4 + 4 * half;
      float e[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) e[i] = (s0 + i <= tl) ? aacc[jt][4 * q4 + i] : 0.f;
      store4_bf16(sA + r * LA + s0, e[0], e[1], e[2], e[3]);
    }
  }
  {
    Tile<D, kTC, NT> t;
    t.fetch_block(p.wvt + (size_t)unit * D * p.Tpad + t0, p.Tpad);
    t.put(sWVt, LA);
  }
  __syncthreads();
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const int k = ks * 16 + half * 8;
    const bf16x8 a = frag(sA, LA, orow + col, k);
#pragma unroll
    for (int jt = 0; jt < NOC; ++jt) oacc[jt] = mfma_bf16(a, frag(sWVt, LA, ocol + 32 * jt + col, k), oacc[jt]);
  }

#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const uint32_t r = orow + 8 * (v / 4) + 4 * half + (v % 4);
    const uint32_t rho = rho0 + r, t = t0 + rho / G;
    if (t < T) {
      const float inv = sScale[0][r];
      uint16_t* o = p.out + (((size_t)b * T + t) * p.Hq + h * G + rho % G) * D;
#pragma unroll
      for (int jt = 0; jt < NOC; ++jt) o[ocol + 32 * jt + col] = bf16_bits(oacc[jt][v] * inv);
    }
  }
}

// ------------------------------------------------------------------ state

// MV tile of 128 slots: acc = MV_start; tokens are walked 64 at a time; at the
// start of every sub-chunk c (if reads follow) round(acc) is left as MV_c;
// acc += WW^T . WV; finally MV = round(acc).  The write weights are recomputed
// per token tile and never leave the registers: a wavefront owns 32 slots and
// all d value columns.  Its score product has rows = tokens, columns = slots, so
// lane l ends up with the weights of slot l % 32 for the tokens
// 8 q + 4 (l / 32) + i (q, i = 0..3) of a 32-token step: per 16 tokens that is
// 4 + 4 values, which is an A operand (row = slot, 8 contraction entries per
// lane) of the state product once the B operand (WV^T) takes its tokens in the
// same order -- two 8-byte LDS reads instead of one 16-byte read.  Only the
// token tiles (write queries, WV^T, row statistics) go through LDS, two
// barriers per 64 tokens; between them the four wavefronts run on their own, so
// one's exponentials overlap another's products.  Each wavefront keeps the key
// fragments of its slots in registers (loaded straight from memory in operand
// layout).
template <int D>
__global__ __launch_bounds__(256, 2) void prefill_state_kernel(const PrefillParams p) {
  constexpr int LD = D + 8, KS = D / 16, NT = 256;
  constexpr int TT = 64;        // tokens per tile
  constexpr int LP = TT + 8;    // row length of the WV^T tile
  constexpr int NJ = D / 32;    // 32-column tiles of the state product
  constexpr int LS = 128 + 8;   // row length of the snapshot staging tile [column][slot]
  static_assert(TT * LD + D * LP >= 128 * LD, "the MV staging tile reuses the token tiles");
  __shared__ __attribute__((aligned(16))) uint16_t sTok[TT * LD + D * LP];
  // the snapshot has LDS of its own: it leaves after the token tile of the step has been staged (see the loop)
  __shared__ __attribute__((aligned(16))) uint16_t sSnapBuf[D * LS];
  __shared__ __attribute__((aligned(16))) float sNorm[TT];
  uint16_t* const sXw = sTok;
  uint16_t* const sWVt = sTok + TT * LD;
  uint16_t* const sSnap = sSnapBuf;   // [column][slot] snapshot on its way out
  uint16_t* const sStage = sTok;   // [slot][column] MV tile on its way in and out

  const uint32_t unit = block_unit();
  if (unit >= p.B * p.Hkv) return;
  const uint32_t b = unit / p.Hkv, h = unit % p.Hkv;
  const uint32_t m0 = blockIdx.x * 128, T = p.T;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const size_t units = (size_t)p.B * p.Hkv;
  const uint16_t* mk = p.mk + (size_t)(p.mk_per_seq ? unit : h) * p.M * D;
  uint16_t* mv = p.mv + ((size_t)unit * p.M + m0) * D;

  // M is a multiple of 64, so a wavefront's 32 slots are all inside the memory or all outside
  const int mslot = 32 * wave;
  const bool live = m0 + mslot < p.M;
  bf16x8 kb[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (live) v = *(const u32x4*)(mk + (size_t)(m0 + mslot + col) * D + ks * 16 + half * 8);
    kb[ks] = __builtin_bit_cast(bf16x8, v);
  }
  // state product: lane column = value column, accumulator rows = slots.  The MV tile comes in (and
  // at the end leaves) through LDS in whole rows; a lane picks its 16 x NJ elements from there.
  f32x16 macc[NJ];
  {
    Tile<128, D, NT> tm;
    tm.fetch_rows(p.mk, [&](int r) -> const uint16_t* { return m0 + r < p.M ? mv + (size_t)r * D : nullptr; });
    tm.put(sStage, LD);
  }
  __syncthreads();
#pragma unroll
  for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
    for (int v = 0; v < 16; ++v)
      macc[jt][v] = bf16_val(sStage[(mslot + 8 * (v / 4) + 4 * half + (v % 4)) * LD + 32 * jt + col]);

  const uint32_t ntile = (T + TT - 1) / TT;
  Tile<TT, D, NT> tx;
  Tile<D, TT, NT> tw;
  float tn = 0.f;
  // Tokens past the end of the chunk load the last token instead: their weights are zero (kNoRow) and
  // their WV^T columns are zero-filled, so whatever finite scores they get changes nothing.
  auto fetch_tokens = [&](uint32_t t0) {
    tx.fetch_rows(p.mk, [&](int r) -> const uint16_t* {
      return p.wq + (((size_t)b * T + min(t0 + r, T - 1)) * p.Hkv + h) * D;
    });
    tw.fetch_block(p.wvt + (size_t)unit * D * p.Tpad + t0, p.Tpad);
    if (threadIdx.x < TT) tn = p.norm_w[(size_t)unit * T + min(t0 + threadIdx.x, T - 1)].x;
  };
  fetch_tokens(0);
  for (uint32_t tt = 0; tt < ntile; ++tt) {
    const uint32_t t0 = tt * TT;
    // The token tile is staged first and the next one requested, and only then does a snapshot leave:
    // loads and stores share one counter, so a wait for loads that follows stores waits for the
    // stores as well - this way the snapshot's stores have the whole step to complete before the next
    // wait (for the next token tile) comes.
    __syncthreads();
    tx.put(sXw, LD);
    tw.put(sWVt, LP);
    if (threadIdx.x < TT) sNorm[threadIdx.x] = (t0 + threadIdx.x < T) ? tn : kNoRow;
    if (tt + 1 < ntile) fetch_tokens(t0 + TT);  // next tile, in flight during this one's products
    if (p.has_read && (t0 % kTC) == 0) {
      // MV at the start of sub-chunk c (c = 0: the tile just loaded, which saves a transposing pass over
      // MV of its own), transposed ([column][slot]) for the read kernel.  A lane holds
      // 4 consecutive slots of one column, and columns are M elements apart in memory, so the tile
      // goes through LDS and leaves in whole 256-byte rows.  (The previous snapshot left this buffer
      // two steps and several barriers ago.)
      if (live) {
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
            store4_bf16(sSnap + (32 * jt + col) * LS + mslot + 8 * q4 + 4 * half, macc[jt][4 * q4 + 0],
                        macc[jt][4 * q4 + 1], macc[jt][4 * q4 + 2], macc[jt][4 * q4 + 3]);
      }
      __syncthreads();
      uint16_t* sn = p.snap + ((size_t)(t0 / kTC) * units + unit) * p.M * D + m0;
      const int ch = threadIdx.x % 16;   // 16-byte chunk = 8 slots; M is a multiple of 64
      if (m0 + 8 * ch < p.M) {
#pragma unroll
        for (int r = threadIdx.x / 16; r < D; r += NT / 16)
          __builtin_nontemporal_store(*(const u32x4*)(sSnap + r * LS + 8 * ch), (u32x4*)(sn + (size_t)r * p.M + 8 * ch));
      }
    }
    __syncthreads();
#pragma unroll
    for (int st = 0; st < TT / 32; ++st) {
      const int tok0 = 32 * st;
      // scores: rows = tokens, columns = this wavefront's 32 slots
      f32x16 sc = zero16();
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) sc = mfma_bf16(frag(sXw, LD, tok0 + col, ks * 16 + half * 8), kb[ks], sc);
      // weights, split into hi + lo bf16 parts: words 0-1 of an operand from q4 = 2 ks, words 2-3 from 2 ks + 1
      u32x4 ah[2], al[2];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 sh = *(const f32x4*)(sNorm + tok0 + 8 * q4 + 4 * half);   // shifts of the lane's 4 tokens
        float w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = fast_exp2(sc[4 * q4 + i] * p.wscale_l2e - sh[i]);
        const uint32_t h0 = pack_bf16x2(w[0], w[1]), h1 = pack_bf16x2(w[2], w[3]);
        ah[q4 / 2][2 * (q4 % 2) + 0] = h0;
        ah[q4 / 2][2 * (q4 % 2) + 1] = h1;
        al[q4 / 2][2 * (q4 % 2) + 0] = pack_bf16x2(w[0] - __uint_as_float(h0 << 16), w[1] - __uint_as_float(h0 & 0xFFFF0000u));
        al[q4 / 2][2 * (q4 % 2) + 1] = pack_bf16x2(w[2] - __uint_as_float(h1 << 16), w[3] - __uint_as_float(h1 & 0xFFFF0000u));
      }
      // state product over the step's 32 tokens, 16 per MFMA, in the token order the weights came in:
      // entries 0-3 of a lane's operand are tokens 16 ks + 4 half + 0..3, entries 4-7 the same + 8.
      // All hi products of a token group before its lo products: no product waits for its predecessor.
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8 vh = __builtin_bit_cast(bf16x8, ah[ks]), vl = __builtin_bit_cast(bf16x8, al[ks]);
        bf16x8 bv[NJ];
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt) {
          const uint16_t* src = sWVt + (32 * jt + col) * LP + tok0 + 16 * ks + 4 * half;
          const uint2 b0 = *(const uint2*)src, b1 = *(const uint2*)(src + 8);
          bv[jt] = __builtin_bit_cast(bf16x8, (u32x4){b0.x, b0.y, b1.x, b1.y});
        }
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt) macc[jt] = mfma_bf16(vh, bv[jt], macc[jt]);
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt) macc[jt] = mfma_bf16(vl, bv[jt], macc[jt]);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
    for (int v = 0; v < 16; ++v)
      sStage[(mslot + 8 * (v / 4) + 4 * half + (v % 4)) * LD + 32 * jt + col] = bf16_bits(macc[jt][v]);
  __syncthreads();
  {
    constexpr int CPR = D / 8;
    const int ch = threadIdx.x % CPR;
#pragma unroll
    for (int r = threadIdx.x / CPR; r < 128; r += NT / CPR)
      if (m0 + r < p.M) __builtin_nontemporal_store(*(const u32x4*)(sStage + r * LD + 8 * ch), (u32x4*)(mv + (size_t)r * D + 8 * ch));
  }
}

// ------------------------------------------------------------------ host side

hipError_t launch_prefill_bf16(const PrefillParams& p0, hipStream_t s) {
  PrefillParams p = p0;
  const uint32_t units = p.B * p.Hkv;
  // a chunk that writes normalises its read rows on the fly (prefill_read_online_kernel): statistics of
  // the write rows only
  p.stats_read = (p.has_read && !p.has_write) ? 1u : 0u;
  const uint32_t rows = (p.has_write ? p.T : 0u) + (p.stats_read ? p.T * p.G : 0u);
  const uint32_t nb = (p.T + kTC - 1) / kTC;
  const bool d128 = p.d == 128;
  const dim3 block(256);
  hipError_t e;

  p.Tpad = nb * kTC;
  auto transpose = [&](int which) -> hipError_t {
    const dim3 g = unit_grid((which == 0 ? p.Tpad : p.M) / 64, units);
    if (d128) hipLaunchKernelGGL(prefill_transpose_kernel<128>, g, block, 0, s, p, which);
    else hipLaunchKernelGGL(prefill_transpose_kernel<64>, g, block, 0, s, p, which);
    return hipGetLastError();
  };
  if (p.has_write && (e = transpose(0)) != hipSuccess) return e;
  // with a write, the state kernel leaves MV_0 transposed as the first snapshot on its way through
  if (p.has_read && !p.has_write && (e = transpose(1)) != hipSuccess) return e;

  const dim3 gs = unit_grid((rows + kTC - 1) / kTC, units);
  if (d128) hipLaunchKernelGGL(prefill_stats_kernel<128>, gs, dim3(512), 0, s, p);
  else hipLaunchKernelGGL(prefill_stats_kernel<64>, gs, dim3(512), 0, s, p);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  auto read = [&](uint32_t c_begin, uint32_t c_count) -> hipError_t {
    p.c_begin = c_begin;
    const dim3 g = unit_grid(c_count * p.G, units);
    const dim3 rblock(512);
    if (p.has_write) {
      if (d128) hipLaunchKernelGGL((prefill_read_online_kernel<128>), g, rblock, 0, s, p);
      else hipLaunchKernelGGL((prefill_read_online_kernel<64>), g, rblock, 0, s, p);
    } else {
      if (d128) hipLaunchKernelGGL((prefill_read_only_kernel<128>), g, rblock, 0, s, p);
      else hipLaunchKernelGGL((prefill_read_only_kernel<64>), g, rblock, 0, s, p);
    }
    return hipGetLastError();
  };
  if (p.has_write) {
    const dim3 g = unit_grid((p.M + 127) / 128, units);
    if (d128) hipLaunchKernelGGL(prefill_state_kernel<128>, g, dim3(256), 0, s, p);
    else hipLaunchKernelGGL(prefill_state_kernel<64>, g, dim3(256), 0, s, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // every sub-chunk reads its starting state from the transposed copies in the workspace (with a write:
  // copy c is what the state kernel left when it reached sub-chunk c, MV_0 for c = 0; without a write:
  // the one copy of MV made above serves all of them), so one launch serves all sub-chunks
  if (p.has_read && (e = read(0, nb)) != hipSuccess) return e;
  return hipSuccess;
}

}  // namespace bct
