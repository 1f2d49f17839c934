// The decode step of a SMALL cache as one launch (gfx950).
//
// The four-launch step (scores, normalise, MV pass, merge) is built to stream
// gigabytes; on a cache of a few megabytes its time is four launch latencies.
// Here one workgroup owns one memory (b, h) from start to finish, so the
// dependency "the softmax normaliser of all M slots before any slot is
// written" (section 3.2 steps 2 and 4) is a workgroup barrier instead of a
// launch boundary:
//   A. scores of the write query and the G read queries against all M keys
//      (log2 domain) into LDS;
//   B. per row: max and sum over the M slots, then the scores are replaced in
//      place by the softmax weights (the write row times the token's step
//      size, if one is given);
//   C. one pass over MV: load, fma(ww[m], wv, MV[m,:]), round, store, and
//      accumulate rw[g][m] times the value just stored (section 3.4 equation,
//      then the read);
//   D. the G output rows are summed over the lanes and wavefronts in a fixed
//      order and stored.
// Chosen by plan_decode for M <= kFusedMaxM and at most kFusedMaxUnits memories
// (one resident round of workgroups); BCT_STEP_STREAMING in the descriptor's flags turns it off.
#include "bct_device.h"
#include "bct_internal.h"

namespace bct {

template <typename DT, int D, int GT>
__global__ __launch_bounds__(256) void decode_fused_kernel(const DecodeParams p) {
  typedef typename DT::elem elem;
  constexpr int E = DT::kElemsPerVec;
  constexpr int LPS = D / E;       // lanes per slot row (16 bytes each)
  constexpr int SPP = 256 / LPS;   // slots per pass of the workgroup
  constexpr int UC = 4;            // slots a lane has in flight in step C

  __shared__ __attribute__((aligned(16))) float s_w[kMaxRows][kFusedMaxM];
  __shared__ float2 s_norm[kMaxRows];
  __shared__ float s_red[4 * GT * D];

  const uint32_t unit = blockIdx.x, b = unit / p.Hkv, h = unit % p.Hkv;
  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
  const int sub = tid % LPS, sl = tid / LPS;
  const uint32_t R = p.R, G = p.G, M = p.M, W = p.has_write;

  // ---- A: scores.  The query rows stay in registers (this lane's 16 bytes of each).
  {
    const elem* mk = (const elem*)p.mk + (size_t)(p.mk_per_seq ? unit : h) * M * D + sub * E;
    float xf[kMaxRows][E], scale[kMaxRows];
#pragma unroll
    for (uint32_t r = 0; r < kMaxRows; ++r) {
      if (r < R) {
        const elem* x = (W && r == 0) ? (const elem*)p.wq + (size_t)b * p.kv_bstride + (size_t)h * D
                                      : (const elem*)p.q + (size_t)b * p.q_bstride + (size_t)(h * G + (r - W)) * D;
        unpack16<DT>(*(const u32x4*)(x + sub * E), xf[r]);
        scale[r] = (W && r == 0) ? p.wscale_l2e : p.rscale_l2e;
      }
    }
    // UC key rows in flight per lane.  A pass of the workgroup covers SPP consecutive slots starting at a
    // multiple of SPP, and SPP divides 64 which divides M: a pass is wholly inside the memory or wholly
    // outside, so the bounds tests below are uniform over the workgroup (the lane exchanges inside are safe)
    for (uint32_t s0 = sl; s0 < M; s0 += SPP * UC) {
      u32x4 kraw[UC];
#pragma unroll
      for (int u = 0; u < UC; ++u)
        if (s0 + u * SPP < M) kraw[u] = *(const u32x4*)(mk + (size_t)(s0 + u * SPP) * D);
#pragma unroll
      for (int u = 0; u < UC; ++u) {
        const uint32_t slot = s0 + u * SPP;
        if (slot < M) {
          float kf[E];
          unpack16<DT>(kraw[u], kf);
#pragma unroll
          for (uint32_t r = 0; r < kMaxRows; ++r) {
            if (r < R) {
              float dot = 0.f;
#pragma unroll
              for (int e = 0; e < E; ++e) dot = __builtin_fmaf(kf[e], xf[r][e], dot);
              dot = xor_sum<1, LPS / 2>(dot);
              if (sub == 0) s_w[r][slot] = dot * scale[r];
            }
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- B: normalisers (one wavefront per row), then weights in place
  for (uint32_t r = wave; r < R; r += 4) {
    float mx = -INFINITY;
    for (uint32_t m = lane; m < M; m += 64) mx = fmaxf(mx, s_w[r][m]);
    mx = xor_max<1, 32>(mx);
    float sm = 0.f;
    for (uint32_t m = lane; m < M; m += 64) sm += fast_exp2(s_w[r][m] - mx);
    sm = xor_sum<1, 32>(sm);
    if (lane == 0) {
      float inv = 1.0f / sm;
      if (p.gate && W && r == 0) inv *= p.gate[(size_t)b * p.gate_bstride + h];
      s_norm[r] = make_float2(mx, inv);
    }
  }
  __syncthreads();
  for (uint32_t i = tid; i < R * M; i += 256) {
    const uint32_t r = i / M, m = i % M;
    const float2 n = s_norm[r];
    s_w[r][m] = fast_exp2(s_w[r][m] - n.x) * n.y;
  }
  __syncthreads();

  // ---- C: the MV pass, UC slots per lane at a time (SPP * UC divides M or the tail is masked)
  elem* mv = (elem*)p.mv + (size_t)unit * M * D + sub * E;
  float wvf[E];
  if (W) {
    const elem* wv = (const elem*)p.wv + (size_t)b * p.kv_bstride + (size_t)h * D;
    unpack16<DT>(*(const u32x4*)(wv + sub * E), wvf);
  }
  float acc[GT][E];
#pragma unroll
  for (int g = 0; g < GT; ++g)
#pragma unroll
    for (int e = 0; e < E; ++e) acc[g][e] = 0.f;
  for (uint32_t s0 = sl; s0 < M; s0 += SPP * UC) {
    u32x4 raw[UC];
#pragma unroll
    for (int u = 0; u < UC; ++u) {
      const uint32_t slot = s0 + u * SPP;
      if (slot < M) raw[u] = *(const u32x4*)(mv + (size_t)slot * D);
    }
#pragma unroll
    for (int u = 0; u < UC; ++u) {
      const uint32_t slot = s0 + u * SPP;
      if (slot < M) {
        float x[E];
        unpack16<DT>(raw[u], x);
        if (W) {
          const float ww = s_w[0][slot];
#pragma unroll
          for (int e = 0; e < E; ++e) x[e] = __builtin_fmaf(ww, wvf[e], x[e]);
          *(u32x4*)(mv + (size_t)slot * D) = pack16_round<DT>(x);  // x now holds the stored values
        }
        if (p.has_read) {
#pragma unroll
          for (int g = 0; g < GT; ++g) {
            if ((uint32_t)g < G) {
              const float rw = s_w[W + g][slot];
#pragma unroll
              for (int e = 0; e < E; ++e) acc[g][e] = __builtin_fmaf(rw, x[e], acc[g][e]);
            }
          }
        }
      }
    }
  }

  // ---- D: output rows
  if (p.has_read) {
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
      for (int e = 0; e < E; ++e) acc[g][e] = xor_sum<LPS, 32>(acc[g][e]);
    if (lane / LPS == 0) {
#pragma unroll
      for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < E; ++e) s_red[(wave * GT + g) * D + sub * E + e] = acc[g][e];
    }
    __syncthreads();
    for (uint32_t i = tid; i < G * D; i += 256) {
      const uint32_t g = i / D, j = i % D;
      const float v = (s_red[(0 * GT + g) * D + j] + s_red[(1 * GT + g) * D + j]) +
                      (s_red[(2 * GT + g) * D + j] + s_red[(3 * GT + g) * D + j]);
      store_elem((elem*)p.out, (size_t)b * p.q_bstride + (size_t)(h * G + g) * D + j, v);
    }
  }
}

template <typename DT, int D>
static void launch_fused_g(const DecodeParams& p, hipStream_t s) {
  const dim3 grid(p.B * p.Hkv), block(256);
  const uint32_t G = p.has_read ? p.G : 1u;
  if (G <= 1) hipLaunchKernelGGL((decode_fused_kernel<DT, D, 1>), grid, block, 0, s, p);
  else if (G <= 2) hipLaunchKernelGGL((decode_fused_kernel<DT, D, 2>), grid, block, 0, s, p);
  else if (G <= 4) hipLaunchKernelGGL((decode_fused_kernel<DT, D, 4>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((decode_fused_kernel<DT, D, 8>), grid, block, 0, s, p);
}

hipError_t launch_fused(const DecodeParams& p, int dtype, hipStream_t s) {
  if (p.M > kFusedMaxM || p.G > kMaxG) return hipErrorInvalidConfiguration;
  if (dtype == 0) {
    if (p.d == 128) launch_fused_g<F32, 128>(p, s);
    else launch_fused_g<F32, 64>(p, s);
  } else {
    if (p.d == 128) launch_fused_g<BF16, 128>(p, s);
    else launch_fused_g<BF16, 64>(p, s);
  }
  return hipGetLastError();
}

}  // namespace bct
