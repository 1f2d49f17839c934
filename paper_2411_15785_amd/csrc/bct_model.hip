// The dense glue of a Llama-shaped stack around the bounded-cache attention
// layer (gfx950): embedding lookup, RMS normalisation, skinny projections
// (the paper's W_wq and W_wv of section 3.2 step 1 among them), the SwiGLU MLP
// and the greedy arg-max, with their C entry points (include/bct_model.h).
//
// The projections multiply a handful of token rows (the decode batch) by a
// large weight matrix, so they are bound by streaming the weights from HBM
// once.  A workgroup owns 32 output features and all K inputs: its eight
// wavefronts split K, each keeps a 32 x 32 fp32 accumulator
// (v_mfma_f32_32x32x16_bf16, rows = token rows, columns = output features) and
// reads its operands straight from memory in operand layout (lane l: row or
// feature l % 32, the 8 consecutive k at 8 * (l / 32)); the eight partial
// accumulators are summed through LDS in a fixed order.
#include "../../include/bct_model.h"

#include <stdio.h>

#include "bct_device.h"

namespace bct {

namespace {

constexpr int kLinWaves = 8;

__device__ __forceinline__ float bf16f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f2bf16(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

template <bool SWIGLU>
__global__ __launch_bounds__(64 * kLinWaves) void linear_kernel(const uint16_t* __restrict__ x,
                                                                const uint16_t* __restrict__ w,
                                                                const uint16_t* __restrict__ w2,
                                                                const uint16_t* residual, uint16_t* out,
                                                                uint32_t rows, uint32_t K, uint32_t N) {
  __shared__ float sC[kLinWaves][32][33];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64, col = lane % 32, half = lane / 32;
  const uint32_t n0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const uint32_t kper = K / kLinWaves, k0 = wave * kper;  // K is a multiple of 64: kper a multiple of 8
  const bool row_ok = r0 + col < rows;
  const uint16_t* xp = x + (size_t)(row_ok ? r0 + col : 0) * K + k0 + half * 8;
  const uint16_t* wp = w + (size_t)(n0 + col) * K + k0 + half * 8;
  const uint16_t* wp2 = SWIGLU ? w2 + (size_t)(n0 + col) * K + k0 + half * 8 : nullptr;
  f32x16 acc, acc2;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = acc2[v] = 0.f;
  auto step = [&](uint32_t s, bool in) {
    u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u}, b2 = {0u, 0u, 0u, 0u};
    if (in) {
      b = __builtin_nontemporal_load((const u32x4*)(wp + s * 16));
      if (SWIGLU) b2 = __builtin_nontemporal_load((const u32x4*)(wp2 + s * 16));
      if (row_ok) a = *(const u32x4*)(xp + s * 16);
    }
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc,
                                                  0, 0, 0);
    if (SWIGLU)
      acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b2),
                                                     acc2, 0, 0, 0);
  };
  // kper / 16 whole steps of 16 k; kper is a multiple of 8, so a remainder of 8
  // is one more step in which only the lower half-wavefront has data
  const uint32_t full = kper / 16;
#pragma unroll 8
  for (uint32_t s = 0; s < full; ++s) step(s, true);
  if (kper % 16) step(full, half == 0);
  // accumulator: lane column = feature n0 + col, rows = token rows 8*(v/4) + 4*half + v%4.
  // Each thread then owns two of the 32 x 32 outputs and adds the eight partials in wave order;
  // the SwiGLU variant sends its second accumulator through the same buffer afterwards.
  float sum[2][2];
#pragma unroll
  for (int pass = 0; pass < (SWIGLU ? 2 : 1); ++pass) {
    if (pass) __syncthreads();
#pragma unroll
    for (int v = 0; v < 16; ++v) sC[wave][8 * (v / 4) + 4 * half + (v % 4)][col] = pass ? acc2[v] : acc[v];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const uint32_t t = threadIdx.x + e * 64 * kLinWaves, i = t / 32, j = t % 32;
      float a = 0.f;
#pragma unroll
      for (int k = 0; k < kLinWaves; ++k) a += sC[k][i][j];
      sum[pass][e] = a;
    }
  }
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const uint32_t t = threadIdx.x + e * 64 * kLinWaves, i = t / 32, j = t % 32;
    if (r0 + i >= rows) continue;
    const size_t o = (size_t)(r0 + i) * N + n0 + j;
    const float g = sum[0][e];
    float y;
    if (SWIGLU) y = g / (1.0f + __expf(-g)) * sum[1][e];
    else y = residual ? g + bf16f(residual[o]) : g;
    out[o] = f2bf16(y);
  }
}

__global__ __launch_bounds__(256) void rmsnorm_kernel(const uint16_t* x, const uint16_t* gain, uint16_t* out,
                                                      uint32_t rows, uint32_t dim, float eps) {
  const uint32_t row = blockIdx.x * 4 + threadIdx.x / 64, lane = threadIdx.x % 64;
  if (row >= rows) return;
  const uint16_t* xr = x + (size_t)row * dim;
  float ss = 0.f;
  for (uint32_t c = lane * 8; c < dim; c += 512) {
    float f[8];
    unpack16<BF16>(*(const u32x4*)(xr + c), f);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss = __builtin_fmaf(f[e], f[e], ss);
  }
  ss = xor_sum<1, 32>(ss);
  const float r = 1.0f / sqrtf(ss / (float)dim + eps);
  for (uint32_t c = lane * 8; c < dim; c += 512) {
    float f[8], g[8];
    unpack16<BF16>(*(const u32x4*)(xr + c), f);
    unpack16<BF16>(*(const u32x4*)(gain + c), g);
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = f[e] * r * g[e];
    *(u32x4*)(out + (size_t)row * dim + c) = pack16_round<BF16>(f);
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
  for (uint32_t j = threadIdx.x; j < N; j += 256) {
    const float v = bf16f(row[j]);
    if (v > best || bi == 0xFFFFFFFFu) {  // ascending j: a later equal value never replaces an earlier one
      best = v;
      bi = j;
    }
  }
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
  if (K % 64 != 0 || N % 32 != 0) return mfail(BCT_ERR_UNSUPPORTED, "K must be a multiple of 64 and N of 32");
  if (!al16(x) || !al16(w) || !al16(out)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  return BCT_OK;
}

}  // namespace
}  // namespace bct

using namespace bct;

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
                        void* hip_stream) {
  if (!x || !gain || !out || rows == 0 || dim == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (dim % 8 != 0 || dim > 16384) return mfail(BCT_ERR_UNSUPPORTED, "dim must be a multiple of 8, at most 16384");
  if (!al16(x) || !al16(gain) || !al16(out)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  hipLaunchKernelGGL(rmsnorm_kernel, dim3((rows + 3) / 4), dim3(256), 0, (hipStream_t)hip_stream, (const uint16_t*)x,
                     (const uint16_t*)gain, (uint16_t*)out, rows, dim, eps);
  return launched("rmsnorm");
}

bct_status bctm_linear(const void* x, const void* w, const void* residual, void* out, uint32_t rows, uint32_t K,
                       uint32_t N, void* hip_stream) {
  const bct_status st = check_linear(x, w, out, rows, K, N);
  if (st != BCT_OK) return st;
  if (!al16(residual)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  hipLaunchKernelGGL((linear_kernel<false>), dim3(N / 32, (rows + 31) / 32), dim3(64 * kLinWaves), 0,
                     (hipStream_t)hip_stream, (const uint16_t*)x, (const uint16_t*)w, (const uint16_t*)nullptr,
                     (const uint16_t*)residual, (uint16_t*)out, rows, K, N);
  return launched("linear");
}

bct_status bctm_swiglu(const void* x, const void* w_gate, const void* w_up, void* out, uint32_t rows, uint32_t K,
                       uint32_t N, void* hip_stream) {
  const bct_status st = check_linear(x, w_gate, out, rows, K, N);
  if (st != BCT_OK) return st;
  if (!w_up) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  if (!al16(w_up)) return mfail(BCT_ERR_MISALIGNED, "pointers must be 16-byte aligned");
  hipLaunchKernelGGL((linear_kernel<true>), dim3(N / 32, (rows + 31) / 32), dim3(64 * kLinWaves), 0,
                     (hipStream_t)hip_stream, (const uint16_t*)x, (const uint16_t*)w_gate, (const uint16_t*)w_up,
                     (const uint16_t*)nullptr, (uint16_t*)out, rows, K, N);
  return launched("swiglu");
}

bct_status bctm_argmax(const void* logits, int32_t* ids, uint32_t rows, uint32_t N, void* hip_stream) {
  if (!logits || !ids || rows == 0 || N == 0) return mfail(BCT_ERR_INVALID_ARG, "NULL pointer or zero size");
  hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(256), 0, (hipStream_t)hip_stream, (const uint16_t*)logits, ids, N);
  return launched("argmax");
}

const char* bctm_last_error(void) { return g_merr; }

}  // extern "C"
