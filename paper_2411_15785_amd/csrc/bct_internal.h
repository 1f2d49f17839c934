// Host-side plan and launcher declarations shared by the C ABI layer and the
// kernel files of libbct.  Nothing here is visible to callers of the library.
#ifndef BCT_INTERNAL_H
#define BCT_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace bct {

constexpr uint32_t kMaxG = 8;          // query heads per KV head
constexpr uint32_t kMaxRows = 1 + kMaxG;  // score rows per memory: write + G reads
constexpr uint32_t kMinStatTile = 32;  // smallest slot tile with its own (max, sum) partial
// A cache this small is stepped by one launch, one workgroup per memory: up to this many
// slots and this many memories (one resident round of workgroups).  Measured inside a HIP graph
// (bf16 d = 128 / fp32 d = 64, 4 to 512 memories): M = 64: 6.5-7.9 us against 7.0-10.9 us for
// the four launches, M = 128: equal or better, M = 256: 15-21 us against 9-23 us (a single
// workgroup has too few loads in flight to stream a larger memory), so the limit is 128.
// Launched eagerly the one launch also saves three launch overheads (config 1: 11 us against 25).
constexpr uint32_t kFusedMaxM = 128;
constexpr uint32_t kFusedMaxUnits = 512;

// One decode step of one layer: everything its launches need.
struct DecodeParams {
  const void* mk;   // [Hkv][M][d] or [B][Hkv][M][d]
  void* mv;         // [B][Hkv][M][d], updated in place
  const void* q;    // [B][Hq][d] or null
  const void* wq;   // [B][Hkv][d] or null
  const void* wv;   // [B][Hkv][d] or null
  void* out;        // [B][Hq][d] or null
  float* scores;    // [B*Hkv][R][M], log2-domain scaled scores
  float2* stats;    // [B*Hkv][R][n_tiles] (max, sum of exp2(score - max)) per slot tile
  float2* norm;     // [B*Hkv][R] (max, 1 / sum of exp2(score - max)) per row
  float* partial;   // [S][B][Hq][d] split-M partial outputs
  uint32_t B, Hq, Hkv, G, M, d;
  uint32_t R;        // rows per memory this step: has_write + (has_read ? G : 0)
  uint32_t has_write, has_read;
  uint32_t mk_per_seq;
  uint32_t stat_tile;  // slots per (max, sum) partial
  uint32_t n_tiles;    // M / stat_tile
  uint32_t S;          // split-M factor of the MV pass: workgroups per memory
  uint32_t mv_bs;      // threads per workgroup of the MV pass
  uint32_t mv_u;       // 16-byte loads per lane of the MV pass
  uint32_t fused;      // 1: the whole step is one launch of decode_fused_kernel
  uint32_t fuse_norm;  // 1: the MV pass merges the per-tile statistics itself, no normaliser launch
  float rscale_l2e, wscale_l2e;  // scale * log2(e)
  // strides (in elements) between consecutive batch entries of q/out and wq/wv;
  // [B][H][d] inputs use H*d, a token t of a [B][T][H][d] chunk uses T*H*d.
  uint64_t q_bstride, kv_bstride;
  // optional step size per memory (section 3.5, learning-rate adaptation): eta of memory (b, h) at
  // gate[b * gate_bstride + h]; null = 1.  Scales the write weights.
  const float* gate;
  uint64_t gate_bstride;
};

// One prefill chunk of a bf16 cache: everything its launches need.
struct PrefillParams {
  const uint16_t* mk;  // [Hkv][M][d] or [B][Hkv][M][d]
  uint16_t* mv;        // [B][Hkv][M][d], updated in place
  const uint16_t* q;   // [B][T][Hq][d] or null
  const uint16_t* wq;  // [B][T][Hkv][d] or null
  const uint16_t* wv;  // [B][T][Hkv][d] or null
  uint16_t* out;       // [B][T][Hq][d] or null
  float2* norm_w;      // [B*Hkv][T]   (max, 1/sum) of each write row
  float2* norm_r;      // [B*Hkv][T*G] (max, 1/sum) of each read row
  uint16_t* snap;      // [ceil(T/128)][B*Hkv][d][M]: MV at the start of each sub-chunk, transposed
  uint16_t* wvt;       // [B*Hkv][d][Tpad]: WV transposed, zero beyond T
  uint32_t Tpad;       // T rounded up to whole sub-chunks
  uint32_t B, Hq, Hkv, G, M, d, T;
  uint32_t has_write, has_read, mk_per_seq;
  float rscale_l2e, wscale_l2e;
  uint32_t c_begin;    // first sub-chunk of a read launch
  uint32_t stats_read; // the statistics kernel also covers the read rows (chunks that only read)
  const float* gate;   // [B][T][Hkv] step sizes (any sign) or null
};
constexpr uint32_t kPrefillSubChunk = 128;
hipError_t launch_prefill_bf16(const PrefillParams& p, hipStream_t s);


// dtype: 0 = fp32, 1 = bf16 (the ABI's bct_dtype values).
hipError_t launch_scores(const DecodeParams& p, int dtype, hipStream_t s);
hipError_t launch_normalise(const DecodeParams& p, hipStream_t s);
hipError_t launch_stream(const DecodeParams& p, int dtype, hipStream_t s);
hipError_t launch_stream_gqa(const DecodeParams& p, hipStream_t s);   // bf16, d = 128, G > 2, with a read
hipError_t launch_merge(const DecodeParams& p, int dtype, hipStream_t s);
hipError_t launch_fused(const DecodeParams& p, int dtype, hipStream_t s);
hipError_t launch_fill_zero(void* dst, size_t n_bytes, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, size_t n_bytes, hipStream_t s);
hipError_t launch_randomize(void* dst, size_t n_bytes, int dtype, uint64_t seed, float amplitude, hipStream_t s);

// Launches indexed by memory (unit = b * Hkv + h) put the unit on grid.y and, beyond the 65535 that a grid
// dimension other than x holds, on grid.z as well: unit = blockIdx.z * kUnitsPerZ + blockIdx.y.  A workgroup
// whose unit is past the end returns at once (the test is uniform over the workgroup).
constexpr uint32_t kUnitsPerZ = 32768;
inline dim3 unit_grid(uint32_t x, uint64_t units) {
  return dim3(x, (unsigned)(units < kUnitsPerZ ? units : kUnitsPerZ), (unsigned)((units + kUnitsPerZ - 1) / kUnitsPerZ));
}

// Chooses stat_tile / n_tiles (scores pass) and the MV pass shape (mv_bs, mv_u, S).
void plan_decode(DecodeParams& p, int dtype);
void plan_mv_pass(DecodeParams& p, int dtype);

}  // namespace bct

#endif
