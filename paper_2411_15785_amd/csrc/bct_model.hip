// The dense glue of a Llama-shaped stack around the bounded-cache attention
// layer (gfx950): embedding lookup, RMS normalisation, skinny projections
// (the paper's W_wq and W_wv of section 3.2 step 1 among them), the SwiGLU MLP
// and the greedy arg-max, with their C entry points (include/bct_model.h).
//
// The projections multiply a handful of token rows (the decode batch) by a
// large weight matrix, so they are bound by streaming the weights from HBM
// once.  The weights are repacked once, when they are loaded, into 1 KB tiles
// in MFMA operand order, so that every wavefront load instruction reads one
// contiguous tile.  A workgroup owns 16 output features and all K inputs: its
// wavefronts split K, each keeps two 16 x 16 fp32 accumulators
// (v_mfma_f32_16x16x32_bf16; rows = token rows, columns = output features) for
// 32 token rows and reads the activations straight from memory (they stay in
// L2); the partial accumulators are summed through LDS in a fixed order.
#include "../../include/bct_model.h"

#include <stdio.h>

#include "bct_device.h"

namespace bct {

namespace {

// Workgroup shapes of the projections (wavefronts that split K, weight tiles a wavefront has in flight,
// feature tiles per workgroup) are template parameters chosen where the kernels are launched.

__device__ __forceinline__ float bf16f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f2bf16(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

// Row-major w [N][K] -> tiles of 16 features x 32 inputs, 1 KB each, tile (n / 16, k / 32) at index
// (n / 16) * (K / 32) + k / 32.  Inside a tile the 16 bytes of lane l = 16 * ((k % 32) / 8) + n % 16 hold
// the 8 consecutive inputs k % 8 = 0..7: the B operand of v_mfma_f32_16x16x32_bf16, so that one wavefront
// load instruction reads one whole tile, contiguously.
__global__ __launch_bounds__(256) void pack_weight_kernel(const uint16_t* __restrict__ w, u32x4* __restrict__ packed,
                                                          uint32_t N, uint32_t K) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte chunk of the packed array
  if (c >= (size_t)N * K / 8) return;
  const uint32_t KT = K / 32, l = (uint32_t)(c % 64);
  const size_t tile = c / 64;
  const uint32_t nt = (uint32_t)(tile / KT), kt = (uint32_t)(tile % KT);
  const uint32_t n = nt * 16 + l % 16, k = kt * 32 + (l / 16) * 8;
  packed[c] = *(const u32x4*)(w + (size_t)n * K + k);
}

// Tiled activations: rows in groups of 32, inputs in groups of 32; group (r / 32, k / 32) is 2 KB, two A
// operands of v_mfma_f32_16x16x32_bf16 (rows 0-15 and 16-31 of the group), each 64 lanes x 16 bytes with
// lane 16 * ((k % 32) / 8) + r % 16 holding the inputs k % 8 = 0..7.  Returns the 16-byte chunk index.
__device__ __forceinline__ size_t tiled_chunk(uint32_t r, uint32_t k, uint32_t K) {
  return ((((size_t)(r / 32) * (K / 32) + k / 32) * 2 + (r % 32) / 16) * 64) + 16 * ((k % 32) / 8) + r % 16;
}

__global__ __launch_bounds__(256) void pack_rows_kernel(const uint16_t* __restrict__ x, u32x4* __restrict__ packed,
                                                        uint32_t rows, uint32_t K) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte chunk of the row-major array
  if (c >= (size_t)rows * K / 8) return;
  const uint32_t r = (uint32_t)(c / (K / 8)), k = (uint32_t)(c % (K / 8)) * 8;
  packed[tiled_chunk(r, k, K)] = *(const u32x4*)(x + (size_t)r * K + k);
}

// Up to three row-major outputs side by side along N: output i takes the features [start[i], start[i + 1]).
struct LinearOut {
  uint16_t* ptr[3];
  uint32_t start[4];
};

// FT: feature tiles (of 16) per workgroup.  Every wavefront streams FT (x 2 for SwiGLU) weight tiles against
// each activation fragment it loads: the activations come from L2, where all workgroups ask for the same
// lines at the same time, and with one weight tile per fragment that traffic (2 KB per KB of weights)
// bounds the kernel at about 4 TB/s of weights; two tiles per fragment reach about 5.
template <bool SWIGLU, bool XT, int WAVES, int U, int FT>
__global__ __launch_bounds__(64 * WAVES) void linear_kernel(const uint16_t* __restrict__ x,
                                                            const u32x4* __restrict__ w,
                                                            const u32x4* __restrict__ w2, const uint16_t* residual,
                                                            LinearOut dst, uint32_t rows, uint32_t K,
                                                            uint32_t out_tiled) {
  constexpr int NW2 = SWIGLU ? 2 : 1;   // weight matrices
  constexpr int NS = FT * NW2;          // weight streams of a wavefront: stream s = feature tile s / NW2 of matrix s % NW2
  constexpr int NTHR = 64 * WAVES;
  __shared__ float sC[WAVES][32][17];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, jl = lane % 16, kg = lane / 16;
  const uint32_t nt0 = blockIdx.x * FT, r0 = blockIdx.y * 32, KT = K / 32;
  // this wavefront's share of the K tiles
  const uint32_t kt0 = (uint32_t)((uint64_t)wave * KT / WAVES), kt1 = (uint32_t)((uint64_t)(wave + 1) * KT / WAVES);
  const u32x4* wt[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) wt[s] = ((s % NW2) ? w2 : w) + ((size_t)(nt0 + s / NW2) * KT + kt0) * 64 + lane;
  // A operand: lane holds token row jl (+16 for the second row tile), inputs 8 * kg .. + 8 of the K tile.
  // Rows past the end load a valid row instead; their results are never stored.
  // Tiled activations: the two operands of K tile kt are the consecutive 1 KB tiles 2 * kt, 2 * kt + 1
  // of this row group (rows past the end are allocated, their content is never stored).
  // xstep: distance in bf16 elements between a lane's chunks of consecutive K tiles.
  const uint32_t ra = min(r0 + jl, rows - 1), rb = min(r0 + 16 + jl, rows - 1);
  const uint16_t* xa = XT ? x + (((size_t)blockIdx.y * KT + kt0) * 128 + lane) * 8
                          : x + (size_t)ra * K + (size_t)kt0 * 32 + kg * 8;
  const uint16_t* xb = XT ? xa + 64 * 8 : x + (size_t)rb * K + (size_t)kt0 * 32 + kg * 8;
  constexpr size_t xstep = XT ? 128 * 8 : 32;
  f32x4 acc[NS][2];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[s][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const uint32_t n_t = kt1 - kt0;
  // Rounds of U tiles: all loads of a round are issued before its first MFMA, so a round costs one memory
  // latency.  The last, partial round loads its missing tiles from the share's last tile (in bounds) and
  // zeroes their weights, which removes them from the sum.
  for (uint32_t t = 0; t < n_t; t += U) {
    const bool whole = t + U <= n_t;
    u32x4 b[U][NS], a0[U], a1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t i = whole ? t + u : min(t + u, n_t - 1);
#pragma unroll
      for (int s = 0; s < NS; ++s) b[u][s] = __builtin_nontemporal_load(wt[s] + i * 64);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t i = whole ? t + u : min(t + u, n_t - 1);
      a0[u] = *(const u32x4*)(xa + i * xstep);
      a1[u] = *(const u32x4*)(xb + i * xstep);
    }
    if (!whole) {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (t + u >= n_t) {
#pragma unroll
          for (int s = 0; s < NS; ++s) b[u][s] = u32x4{0u, 0u, 0u, 0u};
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bf16x8 va = __builtin_bit_cast(bf16x8, a0[u]), vb = __builtin_bit_cast(bf16x8, a1[u]);
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const bf16x8 vw = __builtin_bit_cast(bf16x8, b[u][s]);
        acc[s][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vw, acc[s][0], 0, 0, 0);
        acc[s][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vb, vw, acc[s][1], 0, 0, 0);
      }
    }
  }
  // accumulator element v of a lane: token row 4 * kg + v of the row tile, feature jl.  Per feature tile
  // the partials of all wavefronts go through LDS (one matrix at a time through the same buffer) and
  // every thread adds them in wave order for the outputs it owns (32 x 16 per tile).
  constexpr int OPT = (512 + NTHR - 1) / NTHR;   // outputs per thread and tile
#pragma unroll
  for (int f = 0; f < FT; ++f) {
    float sum[NW2][OPT];
#pragma unroll
    for (int pass = 0; pass < NW2; ++pass) {
      if (f || pass) __syncthreads();
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int v = 0; v < 4; ++v) sC[wave][16 * rt + 4 * kg + v][jl] = acc[f * NW2 + pass][rt][v];
      __syncthreads();
#pragma unroll
      for (int q = 0; q < OPT; ++q) {
        const uint32_t o = (threadIdx.x + q * NTHR) % 512, oi = o / 16, oj = o % 16;
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < WAVES; ++k) a += sC[k][oi][oj];
        sum[pass][q] = a;
      }
    }
#pragma unroll
    for (int q = 0; q < OPT; ++q) {
      const uint32_t o = threadIdx.x + q * NTHR, oi = (o % 512) / 16, oj = o % 16;
      if (o < 512 && r0 + oi < rows) {
        const uint32_t n = (nt0 + f) * 16 + oj;
        const int which = n >= dst.start[2] ? 2 : n >= dst.start[1] ? 1 : 0;
        const uint32_t width = dst.start[which + 1] - dst.start[which], col = n - dst.start[which];
        const size_t oo = (size_t)(r0 + oi) * width + col;
        const float g = sum[0][q];
        float y;
        if (SWIGLU) y = g / (1.0f + __expf(-g)) * sum[NW2 - 1][q];
        else y = residual ? g + bf16f(residual[oo]) : g;
        // a tiled output is the input of a projection whose K is this output's width
        dst.ptr[which][out_tiled ? tiled_chunk(r0 + oi, col, width) * 8 + col % 8 : oo] = f2bf16(y);
      }
    }
  }
}

// The same projections for MANY token rows (a prefill chunk: batch x T rows), where the product is a
// dense contraction bound by the matrix cores and no longer by streaming the weights.  A workgroup of
// 2 x WC wavefronts owns 32 * MI token rows x 64 * WC output features (SwiGLU: 32 * WC features of both
// matrices), each wavefront 16 * MI x 64 of it as MI x 4 accumulators of v_mfma_f32_16x16x32_bf16; built as
// 128 x 128 (MI 4, WC 2) and 256 x 256 (MI 8, WC 4).  Both operands are already stored in MFMA operand
// order (packed weights, tiled activations), so a K step of 32 inputs is a set of one-KB tiles that the
// workgroup copies to LDS unchanged (linear 16-byte accesses on both sides) and every wavefront reads back
// its MI row tiles and four feature tiles; the loads of the next K step are in flight in registers while the
// current one is multiplied (two LDS stages, one barrier per K step).
// Workgroups are numbered so that those resident on one XCD at a time (every eighth workgroup id) cover
// 8 row tiles x consecutive feature tiles: each operand panel is fetched into that XCD's L2 once for
// eight uses.  Output: the accumulators go through LDS (fp32) and leave as 16-byte row-contiguous chunks,
// with the residual added / the SwiGLU applied in fp32 before the one rounding to bf16.
template <bool SWIGLU, bool XT, int MI, int WC>
__global__ __launch_bounds__(128 * WC, 2) void linear_rows_kernel(const uint16_t* __restrict__ x,
                                                                  const u32x4* __restrict__ w,
                                                                  const u32x4* __restrict__ w2,
                                                                  const uint16_t* residual, LinearOut dst,
                                                                  uint32_t rows, uint32_t K, uint32_t NT,
                                                                  uint32_t out_tiled) {
  // 2 x WC wavefronts; a wavefront owns MI row tiles x 4 feature tiles (of 16 each)
  constexpr int NW = 2 * WC;                       // wavefronts
  constexpr int TA = 2 * MI, TB = 4 * WC;          // 1 KB tiles of a K step: activations, weights
  constexpr int NA = TA / NW, NB = TB / NW;        // of them per thread
  static_assert(TA % NW == 0 && TB % NW == 0, "tiles must divide among the wavefronts");
  constexpr uint32_t HB = 8;                       // row tiles of a band
  constexpr uint32_t BM = 32 * MI;                 // token rows of a workgroup
  constexpr uint32_t BNF = (SWIGLU ? 32 : 64) * WC;  // output features of a workgroup
  constexpr int ES = 68;                           // floats per row of the output staging (64 + pad)
  constexpr int ER = NW > 4 ? 16 : 32;             // rows of a wavefront staged at a time
  constexpr int kStage = (TA + TB) * 1024, kOut = NW * ER * ES * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * kStage > kOut ? 2 * kStage : kOut];
  u32x4(*sA)[TA][64] = (u32x4(*)[TA][64])smem;             // [stage][tile][lane]
  u32x4(*sB)[TB][64] = (u32x4(*)[TB][64])(smem + 2 * TA * 1024);
  float(*sE)[ER][ES] = (float(*)[ER][ES])smem;             // [wavefront][row][column], after the K loop

  const uint32_t RT = (rows + BM - 1) / BM, total = RT * NT, per = (total + 7) / 8;
  const uint32_t vid = (blockIdx.x % 8) * per + blockIdx.x / 8;
  if (vid >= total) return;
  const uint32_t nfull = RT / HB;
  uint32_t rt, nt;
  if (vid < nfull * HB * NT) {
    const uint32_t band = vid / (HB * NT), rem = vid % (HB * NT);
    nt = rem / HB;
    rt = band * HB + rem % HB;
  } else {
    const uint32_t rem = vid - nfull * HB * NT, cnt = RT - nfull * HB;
    nt = rem / cnt;
    rt = nfull * HB + rem % cnt;
  }
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, jl = lane % 16, kg = lane / 16;
  const int wr = wave / WC, wc = wave % WC;
  const uint32_t r0 = rt * BM, KT = K / 32;

  // this thread's chunks of a K step: tiles wave, wave + NW, ... of either operand
  const uint16_t* pa[NA];
  const u32x4* pb[NB];
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    const uint32_t tile = wave + NW * j;
    if (XT) {
      const uint32_t g = min(r0 / 32 + tile / 2, (rows + 31) / 32 - 1);   // row groups past the end: a valid one
      pa[j] = x + (((size_t)g * KT * 2 + tile % 2) * 64 + lane) * 8;
    } else {
      const uint32_t r = min(r0 + tile * 16 + jl, rows - 1);
      pa[j] = x + (size_t)r * K + kg * 8;
    }
  }
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const uint32_t tile = wave + NW * j;
    if (SWIGLU) pb[j] = ((tile % 2) ? w2 : w) + (size_t)(nt * (TB / 2) + tile / 2) * KT * 64 + lane;
    else pb[j] = w + (size_t)(nt * TB + tile) * KT * 64 + lane;
  }
  constexpr size_t astep = XT ? 128 * 8 : 32;

  f32x4 acc[MI][4];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  u32x4 ga[NA], gb[NB];
#pragma unroll
  for (int j = 0; j < NA; ++j) ga[j] = *(const u32x4*)pa[j];
#pragma unroll
  for (int j = 0; j < NB; ++j) gb[j] = *pb[j];
#pragma unroll
  for (int j = 0; j < NA; ++j) sA[0][wave + NW * j][lane] = ga[j];
#pragma unroll
  for (int j = 0; j < NB; ++j) sB[0][wave + NW * j][lane] = gb[j];
  __syncthreads();
  for (uint32_t kt = 0; kt < KT; ++kt) {
    const int st = kt & 1;
    const bool more = kt + 1 < KT;
    if (more) {
#pragma unroll
      for (int j = 0; j < NA; ++j) ga[j] = *(const u32x4*)(pa[j] + (size_t)(kt + 1) * astep);
#pragma unroll
      for (int j = 0; j < NB; ++j) gb[j] = pb[j][(size_t)(kt + 1) * 64];
    }
    bf16x8 a[MI], b[4];
#pragma unroll
    for (int i = 0; i < MI; ++i) a[i] = __builtin_bit_cast(bf16x8, sA[st][MI * wr + i][lane]);
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = __builtin_bit_cast(bf16x8, sB[st][4 * wc + i][lane]);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    if (more) {
#pragma unroll
      for (int j = 0; j < NA; ++j) sA[st ^ 1][wave + NW * j][lane] = ga[j];
#pragma unroll
      for (int j = 0; j < NB; ++j) sB[st ^ 1][wave + NW * j][lane] = gb[j];
    }
    __syncthreads();
  }

  // Output, ER rows of every wavefront at a time.  Accumulator element v of a lane: token row 4 * kg + v of
  // row tile i, column jl of B tile j.  Staging columns: plain, B tile j at 16 * j; SwiGLU, B tile
  // j = 2 * f + matrix at 32 * matrix + 16 * f (gate columns 0..31, up columns 32..63).
  constexpr int TPP = ER / 16;                     // row tiles per pass
#pragma unroll
  for (int hf = 0; hf < MI / TPP; ++hf) {
    if (hf) __syncthreads();
#pragma unroll
    for (int ii = 0; ii < TPP; ++ii)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = SWIGLU ? 32 * (j % 2) + 16 * (j / 2) + jl : 16 * j + jl;
#pragma unroll
        for (int v = 0; v < 4; ++v) sE[wave][16 * ii + 4 * kg + v][col] = acc[TPP * hf + ii][j][v];
      }
    __syncthreads();
    const int cc = lane % 8;
    if (!SWIGLU || cc < 4) {
#pragma unroll
      for (int ps = 0; ps < ER / 8; ++ps) {
        const int rr = ps * 8 + lane / 8;
        const uint32_t row = r0 + wr * (16 * MI) + hf * ER + rr;
        if (row < rows) {
          float y[8];
          *(f32x4*)&y[0] = *(const f32x4*)&sE[wave][rr][8 * cc];
          *(f32x4*)&y[4] = *(const f32x4*)&sE[wave][rr][8 * cc + 4];
          const uint32_t n = nt * BNF + (SWIGLU ? wc * 32 : wc * 64) + 8 * cc;
          const int which = n >= dst.start[2] ? 2 : n >= dst.start[1] ? 1 : 0;
          const uint32_t width = dst.start[which + 1] - dst.start[which], col = n - dst.start[which];
          const size_t oo = (size_t)row * width + col;
          if (SWIGLU) {
            float u[8];
            *(f32x4*)&u[0] = *(const f32x4*)&sE[wave][rr][32 + 8 * cc];
            *(f32x4*)&u[4] = *(const f32x4*)&sE[wave][rr][32 + 8 * cc + 4];
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = y[e] / (1.0f + __expf(-y[e])) * u[e];
          } else if (residual) {
            float rv[8];
            unpack16<BF16>(*(const u32x4*)(residual + oo), rv);
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] += rv[e];
          }
          const u32x4 o = pack16_round<BF16>(y);
          if (out_tiled) ((u32x4*)dst.ptr[which])[tiled_chunk(row, col, width)] = o;
          else *(u32x4*)(dst.ptr[which] + oo) = o;
        }
      }
    }
  }
}

// One workgroup per row; a thread keeps its (up to eight) 16-byte chunks of the row in registers between
// the sum of squares and the scaling, so the row is read once.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint16_t* x, const uint16_t* gain, uint16_t* out,
                                                      uint32_t rows, uint32_t dim, float eps, uint32_t out_tiled) {
  __shared__ float s_part[4];
  const uint32_t row = blockIdx.x;
  const uint16_t* xr = x + (size_t)row * dim;
  u32x4 v[8];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t c = (threadIdx.x + i * 256) * 8;
    if (c < dim) {
      v[i] = *(const u32x4*)(xr + c);
      float f[8];
      unpack16<BF16>(v[i], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) ss = __builtin_fmaf(f[e], f[e], ss);
    }
  }
  ss = xor_sum<1, 32>(ss);
  if (threadIdx.x % 64 == 0) s_part[threadIdx.x / 64] = ss;
  __syncthreads();
  ss = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
  const float r = 1.0f / sqrtf(ss / (float)dim + eps);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t c = (threadIdx.x + i * 256) * 8;
    if (c < dim) {
      float f[8], g[8];
      unpack16<BF16>(v[i], f);
      unpack16<BF16>(*(const u32x4*)(gain + c), g);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = f[e] * r * g[e];
      const u32x4 o = pack16_round<BF16>(f);
      if (out_tiled) ((u32x4*)out)[tiled_chunk(row, c, dim)] = o;
      else *(u32x4*)(out + (size_t)row * dim + c) = o;
    }
  }
}

__global__ __launch_bounds__(256) void embed_kernel(const int32_t* ids, const uint16_t* table, uint16_t* out,
                                                    uint32_t rows, uint32_t vocab, uint32_t dim) {
  const uint32_t cpr = dim / 8;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)rows * cpr) return;
  const uint32_t r = (uint32_t)(i / cpr), c = (uint32_t)(i % cpr);
  const int32_t id = ids[r];
  u32x4 v = {0u, 0u, 0u, 0u};
  if (id >= 0 && (uint32_t)id < vocab) v = *(const u32x4*)(table + (size_t)id * dim + c * 8);
  *(u32x4*)(out + (size_t)r * dim + c * 8) = v;
}

__global__ __launch_bounds__(256) void argmax_kernel(const uint16_t* logits, int32_t* ids, uint32_t N) {
  __shared__ float sv[256];
  __shared__ uint32_t si[256];
  const uint16_t* row = logits + (size_t)blockIdx.x * N;
  float best = -INFINITY;
  uint32_t bi = 0xFFFFFFFFu;
  auto take = [&](float v, uint32_t j) {
    if (v > best || bi == 0xFFFFFFFFu) {  // ascending j: a later equal value never replaces an earlier one
      best = v;
      bi = j;
    }
  };
  // 16-byte vectors (8 logits), four in flight per thread; rows start 16-byte aligned when N is a multiple of 8
  const uint32_t nvec = (N % 8 == 0) ? N / 8 : 0u;
  for (uint32_t v0 = threadIdx.x; v0 < nvec; v0 += 4 * 256) {
    u32x4 raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (v0 + u * 256 < nvec) raw[u] = *(const u32x4*)(row + (size_t)(v0 + u * 256) * 8);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (v0 + u * 256 < nvec) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t j = (v0 + u * 256) * 8 + 2 * e;
          take(__uint_as_float(raw[u][e] << 16), j);
          take(__uint_as_float(raw[u][e] & 0xFFFF0000u), j + 1);
        }
      }
    }
  }
  for (uint32_t j = nvec * 8 + threadIdx.x; j < N; j += 256) take(bf16f(row[j]), j);
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      const float ov = sv[threadIdx.x + s];
      const uint32_t oi = si[threadIdx.x + s];
      if (oi != 0xFFFFFFFFu && (si[threadIdx.x] == 0xFFFFFFFFu || ov > sv[threadIdx.x] ||
                                (ov == sv[threadIdx.x] && oi < si[threadIdx.x]))) {
        sv[threadIdx.x] = ov;
        si[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) ids[blockIdx.x] = (int32_t)si[0];
}

thread_local char g_merr[256] = "";

bct_status mfail(bct_status s, const char* msg) {
  snprintf(g_merr, sizeof(g_merr), "%s", msg);
  return s;
}
bct_status launched(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return BCT_OK;
  snprintf(g_merr, sizeof(g_merr), "%s launch failed: %s", what, hipGetErrorString(e));
  return BCT_ERR_HIP;
}
bool al16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

bct_status check_linear(const void* x, const void* w, const void* out, uint32_t rows, uint32_t K, uint32_t N) {
  if (!x || !w || !out || rows == 0 || K == 0 || N == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (K % 32 != 0 || N % 16 != 0) return mfail(BCT_ERR_UNSUPPORTED, "K must be a multiple of 32 and N of 16");
  if (!al16(x) || !al16(w) || !al16(out)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  return BCT_OK;
}

}  // namespace
}  // namespace bct

using namespace bct;

template <int WV, int UN, int FT>
static void launch_linear_w(const void* x, const void* w, const void* residual, const LinearOut& dst, uint32_t rows,
                            uint32_t K, uint32_t N, uint32_t flags, void* hip_stream) {
  const dim3 grid(N / (16 * FT), (rows + 31) / 32), block(64 * WV);
  if (flags & BCTM_X_TILED)
    hipLaunchKernelGGL((linear_kernel<false, true, WV, UN, FT>), grid, block, 0, (hipStream_t)hip_stream,
                       (const uint16_t*)x, (const u32x4*)w, (const u32x4*)nullptr, (const uint16_t*)residual, dst, rows,
                       K, 0u);
  else
    hipLaunchKernelGGL((linear_kernel<false, false, WV, UN, FT>), grid, block, 0, (hipStream_t)hip_stream,
                       (const uint16_t*)x, (const u32x4*)w, (const u32x4*)nullptr, (const uint16_t*)residual, dst, rows,
                       K, 0u);
}

// The kernel of a projection shape.  Many rows (from 128 on): the matrix-core kernel, for feature counts its
// 128-feature (SwiGLU: 64) workgroup tiles cover exactly; 256 x 256 workgroups halve the LDS and L1 traffic
// per flop (measured +5..10 % at 16384 rows) but pad the rows to 256 and need a feature count they divide.
// Few rows: the streaming kernel; measured at 32 rows (weights in TB/s): K = 4096, N = 4096 / 12288: 16
// wavefronts, one feature tile 3.6 / 4.0 against 2.8 / 3.8 for two tiles (too few workgroups); N = 32000:
// two tiles 5.0 against 4.3.
static uint32_t linear_kernel_of(uint32_t rows, uint32_t N, bool swiglu) {
  if (rows >= 128 && N % (swiglu ? 64u : 128u) == 0)
    return (rows >= 1024 && N % (swiglu ? 128u : 256u) == 0) ? BCTM_KERNEL_TILE256 : BCTM_KERNEL_TILE128;
  if (!swiglu && N >= 16384 && N % 32 == 0) return BCTM_KERNEL_STREAMING_WIDE;
  // three feature tiles per workgroup when that still leaves a workgroup for every compute unit: 12288
  // features (W_q | W_wq | W_wv at 4096 each) are exactly 256 workgroups, 19.5 us against 24.3
  if (!swiglu && N % 48 == 0 && N / 48 >= 256) return BCTM_KERNEL_STREAMING_TRIPLE;
  return BCTM_KERNEL_STREAMING;
}

template <bool SWIGLU, int MI, int WC>
static void launch_rows_shape(const void* x, const void* w, const void* w2, const void* residual,
                              const LinearOut& dst, uint32_t rows, uint32_t K, uint32_t N, uint32_t flags,
                              void* hip_stream) {
  const uint32_t NT = N / ((SWIGLU ? 32u : 64u) * WC), RT = (rows + 32 * MI - 1) / (32 * MI);
  const dim3 grid(8 * ((RT * NT + 7) / 8)), block(128 * WC);
  const uint32_t ot = flags & BCTM_OUT_TILED ? 1u : 0u;
  if (flags & BCTM_X_TILED)
    hipLaunchKernelGGL((linear_rows_kernel<SWIGLU, true, MI, WC>), grid, block, 0, (hipStream_t)hip_stream,
                       (const uint16_t*)x, (const u32x4*)w, (const u32x4*)w2, (const uint16_t*)residual, dst, rows, K,
                       NT, ot);
  else
    hipLaunchKernelGGL((linear_rows_kernel<SWIGLU, false, MI, WC>), grid, block, 0, (hipStream_t)hip_stream,
                       (const uint16_t*)x, (const u32x4*)w, (const u32x4*)w2, (const uint16_t*)residual, dst, rows, K,
                       NT, ot);
}

template <bool SWIGLU>
static void launch_rows(uint32_t kernel, const void* x, const void* w, const void* w2, const void* residual,
                        const LinearOut& dst, uint32_t rows, uint32_t K, uint32_t N, uint32_t flags,
                        void* hip_stream) {
  if (kernel == BCTM_KERNEL_TILE256)
    launch_rows_shape<SWIGLU, 8, 4>(x, w, w2, residual, dst, rows, K, N, flags, hip_stream);
  else
    launch_rows_shape<SWIGLU, 4, 2>(x, w, w2, residual, dst, rows, K, N, flags, hip_stream);
}

template <int WV, int UN, int FT>
static void launch_swiglu_w(const void* x, const void* wg, const void* wu, const LinearOut& dst, uint32_t rows,
                            uint32_t K, uint32_t N, uint32_t flags, void* hip_stream) {
  const dim3 grid(N / (16 * FT), (rows + 31) / 32), block(64 * WV);
  const uint32_t ot = flags & BCTM_OUT_TILED ? 1u : 0u;
  if (flags & BCTM_X_TILED)
    hipLaunchKernelGGL((linear_kernel<true, true, WV, UN, FT>), grid, block, 0, (hipStream_t)hip_stream,
                       (const uint16_t*)x, (const u32x4*)wg, (const u32x4*)wu, (const uint16_t*)nullptr, dst, rows, K, ot);
  else
    hipLaunchKernelGGL((linear_kernel<true, false, WV, UN, FT>), grid, block, 0, (hipStream_t)hip_stream,
                       (const uint16_t*)x, (const u32x4*)wg, (const u32x4*)wu, (const uint16_t*)nullptr, dst, rows, K, ot);
}

extern "C" {

bct_status bctm_embed(const int32_t* ids, const void* table, void* out, uint32_t rows, uint32_t vocab, uint32_t dim,
                      void* hip_stream) {
  if (!ids || !table || !out || rows == 0 || vocab == 0 || dim == 0)
    return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (dim % 8 != 0) return mfail(BCT_ERR_UNSUPPORTED, "dim must be a multiple of 8");
  if (!al16(table) || !al16(out)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  const size_t n = (size_t)rows * (dim / 8);
  hipLaunchKernelGGL(embed_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream, ids,
                     (const uint16_t*)table, (uint16_t*)out, rows, vocab, dim);
  return launched("embed");
}

bct_status bctm_rmsnorm(const void* x, const void* gain, void* out, uint32_t rows, uint32_t dim, float eps,
                        uint32_t flags, void* hip_stream) {
  if (!x || !gain || !out || rows == 0 || dim == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (flags & ~BCTM_OUT_TILED) return mfail(BCT_ERR_INVALID_ARG, "rmsnorm takes only BCTM_OUT_TILED");
  if (dim % 8 != 0 || dim > 16384) return mfail(BCT_ERR_UNSUPPORTED, "dim must be a multiple of 8, at most 16384");
  if ((flags & BCTM_OUT_TILED) && dim % 32 != 0)
    return mfail(BCT_ERR_UNSUPPORTED, "tiled activations need a multiple of 32 columns");
  if ((flags & BCTM_OUT_TILED) && x == out) return mfail(BCT_ERR_INVALID_ARG, "a tiled output cannot overwrite x");
  if (!al16(x) || !al16(gain) || !al16(out)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(256), 0, (hipStream_t)hip_stream, (const uint16_t*)x,
                     (const uint16_t*)gain, (uint16_t*)out, rows, dim, eps, flags & BCTM_OUT_TILED);
  return launched("rmsnorm");
}

bct_status bctm_pack_rows(const void* x, void* tiled, uint32_t rows, uint32_t K, void* hip_stream) {
  if (!x || !tiled || rows == 0 || K == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (x == tiled) return mfail(BCT_ERR_INVALID_ARG, "packing in place is not possible");
  if (K % 32 != 0) return mfail(BCT_ERR_UNSUPPORTED, "tiled activations need a multiple of 32 columns");
  if (!al16(x) || !al16(tiled)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  const size_t chunks = (size_t)rows * K / 8;
  if ((chunks + 255) / 256 > 0x7FFFFFFFu) return mfail(BCT_ERR_UNSUPPORTED, "matrix too large");
  hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream,
                     (const uint16_t*)x, (u32x4*)tiled, rows, K);
  return launched("pack_rows");
}

bct_status bctm_pack_weight(const void* w, void* packed, uint32_t N, uint32_t K, void* hip_stream) {
  if (!w || !packed || N == 0 || K == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (w == packed) return mfail(BCT_ERR_INVALID_ARG, "packing in place is not possible");
  if (K % 32 != 0 || N % 16 != 0) return mfail(BCT_ERR_UNSUPPORTED, "K must be a multiple of 32 and N of 16");
  if (!al16(w) || !al16(packed)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  const size_t chunks = (size_t)N * K / 8;
  if ((chunks + 255) / 256 > 0x7FFFFFFFu) return mfail(BCT_ERR_UNSUPPORTED, "matrix too large");
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream,
                     (const uint16_t*)w, (u32x4*)packed, N, K);
  return launched("pack_weight");
}

static bct_status launch_linear(const void* x, const void* w, const void* residual, const LinearOut& dst,
                                uint32_t rows, uint32_t K, uint32_t N, uint32_t flags, void* hip_stream) {
  const uint32_t kernel = linear_kernel_of(rows, N, false);
  if (kernel == BCTM_KERNEL_TILE128 || kernel == BCTM_KERNEL_TILE256)
    launch_rows<false>(kernel, x, w, nullptr, residual, dst, rows, K, N, flags, hip_stream);
  else if (kernel == BCTM_KERNEL_STREAMING_WIDE) launch_linear_w<8, 4, 2>(x, w, residual, dst, rows, K, N, flags, hip_stream);
  else if (kernel == BCTM_KERNEL_STREAMING_TRIPLE) launch_linear_w<8, 4, 3>(x, w, residual, dst, rows, K, N, flags, hip_stream);
  else launch_linear_w<16, 8, 1>(x, w, residual, dst, rows, K, N, flags, hip_stream);
  return launched("linear");
}

bct_status bctm_linear(const void* x, const void* w, const void* residual, void* out, uint32_t rows, uint32_t K,
                       uint32_t N, uint32_t flags, void* hip_stream) {
  const bct_status st = check_linear(x, w, out, rows, K, N);
  if (st != BCT_OK) return st;
  if (flags & ~BCTM_X_TILED) return mfail(BCT_ERR_INVALID_ARG, "linear takes only BCTM_X_TILED");
  if (x == out) return mfail(BCT_ERR_INVALID_ARG, "out must not be x");
  if (!al16(residual)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  const LinearOut dst = {{(uint16_t*)out, nullptr, nullptr}, {0u, N, N, N}};
  return launch_linear(x, w, residual, dst, rows, K, N, flags, hip_stream);
}

bct_status bctm_linear_split(const void* x, const void* w, void* out0, uint32_t N0, void* out1, uint32_t N1,
                             void* out2, uint32_t N2, uint32_t rows, uint32_t K, uint32_t flags, void* hip_stream) {
  if (N0 == 0 || N1 == 0) return mfail(BCT_ERR_INVALID_ARG, "the first two outputs must not be empty");
  if ((uint64_t)N0 + N1 + N2 > 0xFFFFFFF0ull) return mfail(BCT_ERR_UNSUPPORTED, "too many features");
  const uint32_t N = N0 + N1 + N2;
  const bct_status st = check_linear(x, w, out0, rows, K, N);
  if (st != BCT_OK) return st;
  if (flags & ~BCTM_X_TILED) return mfail(BCT_ERR_INVALID_ARG, "linear takes only BCTM_X_TILED");
  if (!out1 || (N2 && !out2)) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (N0 % 16 != 0 || N1 % 16 != 0 || N2 % 16 != 0)
    return mfail(BCT_ERR_UNSUPPORTED, "every output width must be a multiple of 16");
  if (x == out0 || x == out1 || x == out2) return mfail(BCT_ERR_INVALID_ARG, "out must not be x");
  if (!al16(out1) || !al16(out2)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  const LinearOut dst = {{(uint16_t*)out0, (uint16_t*)out1, (uint16_t*)out2}, {0u, N0, N0 + N1, N}};
  return launch_linear(x, w, nullptr, dst, rows, K, N, flags, hip_stream);
}

bct_status bctm_swiglu(const void* x, const void* w_gate, const void* w_up, void* out, uint32_t rows, uint32_t K,
                       uint32_t N, uint32_t flags, void* hip_stream) {
  const bct_status st = check_linear(x, w_gate, out, rows, K, N);
  if (st != BCT_OK) return st;
  if (flags & ~(BCTM_X_TILED | BCTM_OUT_TILED)) return mfail(BCT_ERR_INVALID_ARG, "unknown flag");
  if (!w_up) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (x == out) return mfail(BCT_ERR_INVALID_ARG, "out must not be x");
  if ((flags & BCTM_OUT_TILED) && N % 32 != 0)
    return mfail(BCT_ERR_UNSUPPORTED, "tiled activations need a multiple of 32 columns");
  if (!al16(w_up)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  const LinearOut dst = {{(uint16_t*)out, nullptr, nullptr}, {0u, N, N, N}};
  const uint32_t kernel = linear_kernel_of(rows, N, true);
  if (kernel == BCTM_KERNEL_TILE128 || kernel == BCTM_KERNEL_TILE256) launch_rows<true>(kernel, x, w_gate, w_up, nullptr, dst, rows, K, N, flags, hip_stream);
  else launch_swiglu_w<4, 8, 1>(x, w_gate, w_up, dst, rows, K, N, flags, hip_stream);   // 36 us at 4096 -> 11008 (8 wavefronts: 38)
  return launched("swiglu");
}

bct_status bctm_linear_plan(uint32_t rows, uint32_t K, uint32_t N, uint32_t swiglu, uint32_t* kernel) {
  if (!kernel || rows == 0 || K == 0 || N == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (K % 32 != 0 || N % 16 != 0) return mfail(BCT_ERR_UNSUPPORTED, "K must be a multiple of 32 and N of 16");
  *kernel = linear_kernel_of(rows, N, swiglu != 0);
  return BCT_OK;
}

bct_status bctm_argmax(const void* logits, int32_t* ids, uint32_t rows, uint32_t N, void* hip_stream) {
  if (!logits || !ids || rows == 0 || N == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(256), 0, (hipStream_t)hip_stream, (const uint16_t*)logits, ids, N);
  return launched("argmax");
}

const char* bctm_last_error(void) { return g_merr; }

}  // extern "C"
