// C ABI of libbct: argument checks, the per-cache plan and the launch
// sequence.  Every check runs before the first HIP call of an entry point.
#include "../../include/bct.h"
#include "../../include/bct_measure.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "bct_internal.h"

struct bct_cache {
  bct_cache_desc desc;
  uint32_t max_T;
  char* mk;
  char* mv;
  size_t mk_bytes, mv_bytes;
  char* ws;
  size_t ws_bytes;
  // workspace carve-up (byte offsets)
  size_t off_scores, off_stats, off_norm, off_partial, off_pf_norm_w, off_pf_norm_r, off_pf_wvt, off_pf_snap;
  size_t ws_decode_bytes;  // the part of the workspace a decode step uses (it comes first)
  uint64_t steps;
  bool keys_set;
  bct::DecodeParams plan;  // shape, strides and launch plan; pointers filled per call
  // optional per-launch timing: 4 events per recorded step
  std::vector<hipEvent_t> prof_ev;
  uint32_t prof_cap = 0, prof_n = 0;
};

// Scratch of bct_decode_step_static: the scores, the per-tile statistics, the row normalisers and
// the split-M partial outputs of one decode step live here instead of in a caller's workspace.
// Every GPU the library runs on holds its own copy of this array until the process ends.
#define BCT_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[BCT_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

bct_status fail(bct_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

bct_status hip_fail(hipError_t e, const char* what) {
  return fail(BCT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }
inline size_t esize(int dtype) { return dtype == BCT_F32 ? 4 : 2; }

bct_status check_desc(const bct_cache_desc* d) {
  if (!d) return fail(BCT_ERR_INVALID_ARG, "desc is NULL");
  if (d->capacity_M == 0 || d->batch == 0 || d->n_q_heads == 0 || d->n_kv_heads == 0 || d->head_dim == 0)
    return fail(BCT_ERR_INVALID_ARG, "capacity_M, batch, n_q_heads, n_kv_heads and head_dim must be positive");
  if (d->n_q_heads % d->n_kv_heads != 0)
    return fail(BCT_ERR_INVALID_ARG, "n_q_heads (%u) is not a multiple of n_kv_heads (%u)", d->n_q_heads,
                d->n_kv_heads);
  if (!isfinite(d->read_scale) || !isfinite(d->write_scale))
    return fail(BCT_ERR_INVALID_ARG, "read_scale and write_scale must be finite");
  if (d->dtype != BCT_F32 && d->dtype != BCT_BF16) return fail(BCT_ERR_UNSUPPORTED, "dtype %d", d->dtype);
  if (d->head_dim != 64 && d->head_dim != 128)
    return fail(BCT_ERR_UNSUPPORTED, "head_dim %u (64 or 128)", d->head_dim);
  if (d->capacity_M % 64 != 0 || d->capacity_M > 65536)
    return fail(BCT_ERR_UNSUPPORTED, "capacity_M %u (a multiple of 64, at most 65536)", d->capacity_M);
  if (d->n_q_heads / d->n_kv_heads > bct::kMaxG)
    return fail(BCT_ERR_UNSUPPORTED, "n_q_heads / n_kv_heads = %u (at most %u)", d->n_q_heads / d->n_kv_heads,
                bct::kMaxG);
  if (d->flags & ~(uint32_t)(BCT_MK_PER_SEQUENCE | BCT_STEP_STREAMING)) return fail(BCT_ERR_UNSUPPORTED, "unknown flags 0x%x", d->flags);
  if ((uint64_t)d->batch * d->n_kv_heads > (1u << 24))
    return fail(BCT_ERR_UNSUPPORTED, "batch * n_kv_heads = %llu (at most 16777216)",
                (unsigned long long)d->batch * d->n_kv_heads);
  return BCT_OK;
}

struct Sizes {
  size_t mk_bytes, mv_bytes, cache_bytes;
  size_t off_scores, off_stats, off_norm, off_partial, off_pf_norm_w, off_pf_norm_r, off_pf_wvt, off_pf_snap, ws_bytes;
  size_t ws_decode_bytes;
};

void fill_plan(const bct_cache_desc* d, bct::DecodeParams& p) {
  memset(&p, 0, sizeof(p));
  p.B = d->batch;
  p.Hq = d->n_q_heads;
  p.Hkv = d->n_kv_heads;
  p.G = p.Hq / p.Hkv;
  p.M = d->capacity_M;
  p.d = d->head_dim;
  p.mk_per_seq = (d->flags & BCT_MK_PER_SEQUENCE) ? 1u : 0u;
  const double l2e = 1.4426950408889634;
  p.rscale_l2e = (float)((double)d->read_scale * l2e);
  p.wscale_l2e = (float)((double)d->write_scale * l2e);
  p.q_bstride = (uint64_t)p.Hq * p.d;
  p.kv_bstride = (uint64_t)p.Hkv * p.d;
  p.R = 1 + p.G;
  p.has_write = p.has_read = 1;
  bct::plan_decode(p, d->dtype);
  if (d->flags & BCT_STEP_STREAMING) p.fused = 0u;
}

Sizes compute_sizes(const bct_cache_desc* d, uint32_t max_T) {
  Sizes z;
  const size_t sz = esize(d->dtype);
  const size_t per_head = (size_t)d->capacity_M * d->head_dim * sz;
  const size_t units = (size_t)d->batch * d->n_kv_heads;
  z.mk_bytes = ((d->flags & BCT_MK_PER_SEQUENCE) ? units : (size_t)d->n_kv_heads) * per_head;
  z.mv_bytes = units * per_head;
  z.cache_bytes = align_up(z.mk_bytes, 256) + z.mv_bytes;
  bct::DecodeParams p;
  fill_plan(d, p);
  const size_t rows = 1 + p.G;
  size_t off = 0;
  z.off_scores = off;
  off += align_up(units * rows * p.M * sizeof(float), 256);
  z.off_stats = off;
  off += align_up(units * rows * (p.M / bct::kMinStatTile) * sizeof(float2), 256);
  z.off_norm = off;
  off += align_up(units * rows * sizeof(float2), 256);
  z.off_partial = off;
  off += align_up((size_t)p.S * d->batch * d->n_q_heads * d->head_dim * sizeof(float), 256);
  z.ws_decode_bytes = off;
  // prefill of a bf16 cache: row normalisers and the MV snapshots at sub-chunk starts
  z.off_pf_norm_w = z.off_pf_norm_r = z.off_pf_wvt = z.off_pf_snap = off;
  if (max_T > 0 && d->dtype == BCT_BF16) {
    z.off_pf_norm_w = off;
    off += align_up(units * max_T * sizeof(float2), 256);
    z.off_pf_norm_r = off;
    off += align_up(units * max_T * p.G * sizeof(float2), 256);
    const size_t nb = (max_T + bct::kPrefillSubChunk - 1) / bct::kPrefillSubChunk;
    z.off_pf_wvt = off;
    off += align_up(units * d->head_dim * nb * bct::kPrefillSubChunk * sz, 256);
    z.off_pf_snap = off;
    off += align_up(nb * z.mv_bytes, 256);
  }
  z.ws_bytes = off;
  return z;
}

bct_status check_io(const bct_cache* c, const void* q, const void* k_new, const void* v_new, const void* out) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if ((k_new == nullptr) != (v_new == nullptr))
    return fail(BCT_ERR_INVALID_ARG, "k_new and v_new must both be given or both be NULL");
  if ((q == nullptr) != (out == nullptr))
    return fail(BCT_ERR_INVALID_ARG, "q and out must both be given or both be NULL");
  if (!q && !k_new) return fail(BCT_ERR_INVALID_ARG, "neither a read (q, out) nor a write (k_new, v_new) given");
  if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out))
    return fail(BCT_ERR_MISALIGNED, "q, k_new, v_new and out must be 16-byte aligned");
  if (!c->keys_set) return fail(BCT_ERR_STATE, "bct_cache_set_keys has not been called");
  return BCT_OK;
}

// The three launches of one decode step; q/kv batch strides allow a token of
// a [B][T][H][d] chunk to be stepped in place.
// key_new (optional): the keyed step, whose write also moves the per-sequence keys; key_gate its step sizes.
bct_status run_decode(bct_cache* c, char* ws, const void* q, const void* k_new, const void* v_new, void* out,
                      uint64_t q_bstride, uint64_t kv_bstride, const float* gate, uint64_t gate_bstride,
                      hipStream_t s, const void* key_new = nullptr, const float* key_gate = nullptr) {
  bct::DecodeParams p = c->plan;
  p.mk = c->mk;
  p.mv = c->mv;
  p.q = q;
  p.wq = k_new;
  p.wv = v_new;
  p.out = out;
  p.scores = (float*)(ws + c->off_scores);
  p.stats = (float2*)(ws + c->off_stats);
  p.norm = (float2*)(ws + c->off_norm);
  p.partial = (float*)(ws + c->off_partial);
  p.has_write = k_new ? 1u : 0u;
  p.has_read = q ? 1u : 0u;
  p.R = p.has_write + (p.has_read ? p.G : 0u);
  p.q_bstride = q_bstride;
  p.kv_bstride = kv_bstride;
  p.gate = gate;
  p.gate_bstride = gate_bstride;
  hipError_t e;
  hipEvent_t* ev = (c->prof_n < c->prof_cap) ? &c->prof_ev[(size_t)c->prof_n * 4] : nullptr;
  if (ev && (e = hipEventRecord(ev[0], s)) != hipSuccess) return hip_fail(e, "event record");
  if (key_new) p.fused = 0u;   // the one-launch step has no key update: take the streaming launches
  if (p.fused) {
    // a small cache: the whole step in one launch (timed as the MV pass)
    if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return hip_fail(e, "event record");
    if ((e = bct::launch_fused(p, c->desc.dtype, s)) != hipSuccess) return hip_fail(e, "fused step launch");
    if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return hip_fail(e, "event record");
  } else {
    if ((e = bct::launch_scores(p, c->desc.dtype, s)) != hipSuccess) return hip_fail(e, "scores launch");
    if ((e = bct::launch_normalise(p, s)) != hipSuccess) return hip_fail(e, "normaliser launch");
    if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return hip_fail(e, "event record");
    if ((e = bct::launch_stream(p, c->desc.dtype, s)) != hipSuccess) return hip_fail(e, "MV pass launch");
    if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return hip_fail(e, "event record");
    if ((e = bct::launch_merge(p, c->desc.dtype, s)) != hipSuccess) return hip_fail(e, "merge launch");
    if (key_new) {
      // MK += kappa * ww^T wk: the same pass over a memory of M rows, now the keys of each sequence, with
      // the write row's scores and statistics still in the scratch (computed from the keys as they
      // were); no read.  Row 0 of every memory stays the write row: R keeps its value.
      bct::DecodeParams pk = p;
      pk.mv = c->mk;
      pk.wv = key_new;
      pk.gate = key_gate;
      pk.has_read = 0u;
      if ((e = bct::launch_normalise(pk, s)) != hipSuccess) return hip_fail(e, "normaliser launch (keys)");
      if ((e = bct::launch_stream(pk, c->desc.dtype, s)) != hipSuccess) return hip_fail(e, "key pass launch");
    }
  }
  if (ev) {
    if ((e = hipEventRecord(ev[3], s)) != hipSuccess) return hip_fail(e, "event record");
    c->prof_n += 1;
  }
  return BCT_OK;
}

// Device address of `scratch` on each GPU.  In host code the array's name is only a handle for
// hipGetSymbolAddress, not an address a kernel can use: the address is looked up once per device,
// with that device current, and everything below uses the pointer.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[kMaxDevices] = {};

bct_status static_scratch(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(BCT_ERR_UNSUPPORTED, "device %d (at most %d devices)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!ptr || ((uintptr_t)ptr & 255u)) return fail(BCT_ERR_HIP, "hipGetSymbolAddress(scratch) gave %p", ptr);
    g_scratch_ptr[dev] = (char*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return BCT_OK;
}

}  // namespace

extern "C" {

bct_status bct_cache_query(const bct_cache_desc* desc, uint32_t max_prefill_T, size_t* cache_bytes,
                           size_t* workspace_bytes) {
  bct_status st = check_desc(desc);
  if (st != BCT_OK) return st;
  const Sizes z = compute_sizes(desc, max_prefill_T);
  if (cache_bytes) *cache_bytes = z.cache_bytes;
  if (workspace_bytes) *workspace_bytes = z.ws_bytes;
  return BCT_OK;
}

bct_status bct_cache_init(const bct_cache_desc* desc, uint32_t max_prefill_T, void* cache_mem, size_t cache_bytes,
                          void* workspace, size_t workspace_bytes, void* hip_stream, bct_cache** out) {
  if (!out) return fail(BCT_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  bct_status st = check_desc(desc);
  if (st != BCT_OK) return st;
  if (!cache_mem || !workspace) return fail(BCT_ERR_INVALID_ARG, "cache_mem and workspace must not be NULL");
  if (((uintptr_t)cache_mem & 255u) || ((uintptr_t)workspace & 255u))
    return fail(BCT_ERR_MISALIGNED, "cache_mem and workspace must be 256-byte aligned");
  const Sizes z = compute_sizes(desc, max_prefill_T);
  if (cache_bytes < z.cache_bytes)
    return fail(BCT_ERR_BUFFER_TOO_SMALL, "cache_bytes %zu < %zu", cache_bytes, z.cache_bytes);
  if (workspace_bytes < z.ws_bytes)
    return fail(BCT_ERR_BUFFER_TOO_SMALL, "workspace_bytes %zu < %zu", workspace_bytes, z.ws_bytes);
  bct_cache* c = new (std::nothrow) bct_cache();
  if (!c) return fail(BCT_ERR_INVALID_ARG, "out of host memory");
  c->desc = *desc;
  c->max_T = max_prefill_T;
  c->mk = (char*)cache_mem;
  c->mv = (char*)cache_mem + align_up(z.mk_bytes, 256);
  c->mk_bytes = z.mk_bytes;
  c->mv_bytes = z.mv_bytes;
  c->ws = (char*)workspace;
  c->ws_bytes = z.ws_bytes;
  c->off_scores = z.off_scores;
  c->off_stats = z.off_stats;
  c->off_norm = z.off_norm;
  c->off_partial = z.off_partial;
  c->off_pf_norm_w = z.off_pf_norm_w;
  c->off_pf_norm_r = z.off_pf_norm_r;
  c->off_pf_wvt = z.off_pf_wvt;
  c->off_pf_snap = z.off_pf_snap;
  c->ws_decode_bytes = z.ws_decode_bytes;
  c->steps = 0;
  c->keys_set = false;
  fill_plan(desc, c->plan);
  {
    // set-up time is where the static scratch's address is looked up on this device (a caller of
    // bct_decode_step_static may be unable to make such a call later, e.g. under graph capture)
    char* unused = nullptr;
    const bct_status ss = static_scratch(&unused);
    if (ss != BCT_OK) {
      delete c;
      return ss;
    }
  }
  const hipError_t e = bct::launch_fill_zero(c->mv, c->mv_bytes, (hipStream_t)hip_stream);
  if (e != hipSuccess) {
    delete c;
    return hip_fail(e, "zeroing MV");
  }
  *out = c;
  return BCT_OK;
}

bct_status bct_cache_set_keys(bct_cache* c, const void* mk_dev, void* hip_stream) {
  if (!c || !mk_dev) return fail(BCT_ERR_INVALID_ARG, "cache handle or mk_dev is NULL");
  if (!aligned16(mk_dev)) return fail(BCT_ERR_MISALIGNED, "mk_dev must be 16-byte aligned");
  const hipError_t e = bct::launch_copy(c->mk, mk_dev, c->mk_bytes, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "copying MK");
  c->keys_set = true;
  return BCT_OK;
}

bct_status bct_cache_set_values(bct_cache* c, const void* mv0_dev, void* hip_stream) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if (!aligned16(mv0_dev)) return fail(BCT_ERR_MISALIGNED, "mv0_dev must be 16-byte aligned");
  const hipError_t e = mv0_dev ? bct::launch_copy(c->mv, mv0_dev, c->mv_bytes, (hipStream_t)hip_stream)
                               : bct::launch_fill_zero(c->mv, c->mv_bytes, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "setting MV");
  return BCT_OK;
}

bct_status bct_cache_randomize_values(bct_cache* c, uint64_t seed, float amplitude, void* hip_stream) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if (!(amplitude == amplitude) || amplitude - amplitude != 0.0f)
    return fail(BCT_ERR_INVALID_ARG, "amplitude must be finite");
  const hipError_t e = bct::launch_randomize(c->mv, c->mv_bytes, c->desc.dtype, seed, amplitude, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "randomising MV");
  return BCT_OK;
}

// One sequence's slice of MV (and of MK when the keys are per sequence) is contiguous.
static bct_status sequence_copy(bct_cache* c, uint32_t b, void* mk_ext, void* mv_ext, bool out, hipStream_t s) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if (b >= c->desc.batch) return fail(BCT_ERR_INVALID_ARG, "sequence %u of a batch of %u", b, c->desc.batch);
  if (!mk_ext && !mv_ext) return fail(BCT_ERR_INVALID_ARG, "nothing to copy");
  if (mk_ext && !(c->desc.flags & BCT_MK_PER_SEQUENCE))
    return fail(BCT_ERR_INVALID_ARG, "the keys are shared by the batch: there is no per-sequence MK");
  if (!aligned16(mk_ext) || !aligned16(mv_ext)) return fail(BCT_ERR_MISALIGNED, "buffers must be 16-byte aligned");
  const size_t per = c->mv_bytes / c->desc.batch;
  hipError_t e;
  if (mv_ext) {
    char* in = (char*)c->mv + (size_t)b * per;
    if ((e = out ? bct::launch_copy(mv_ext, in, per, s) : bct::launch_copy(in, mv_ext, per, s)) != hipSuccess)
      return hip_fail(e, "copying a sequence's MV");
  }
  if (mk_ext) {
    char* in = (char*)c->mk + (size_t)b * per;
    if ((e = out ? bct::launch_copy(mk_ext, in, per, s) : bct::launch_copy(in, mk_ext, per, s)) != hipSuccess)
      return hip_fail(e, "copying a sequence's MK");
  }
  return BCT_OK;
}

bct_status bct_cache_export_sequence(const bct_cache* c, uint32_t b, void* mk_dst, void* mv_dst, void* hip_stream) {
  return sequence_copy(const_cast<bct_cache*>(c), b, mk_dst, mv_dst, true, (hipStream_t)hip_stream);
}

bct_status bct_cache_import_sequence(bct_cache* c, uint32_t b, const void* mk_src, const void* mv_src,
                                     void* hip_stream) {
  return sequence_copy(c, b, const_cast<void*>(mk_src), const_cast<void*>(mv_src), false, (hipStream_t)hip_stream);
}

bct_status bct_decode_step_gated(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                                 const float* gate, void* out, void* hip_stream) {
  bct_status st = check_io(c, q, k_new, v_new, out);
  if (st != BCT_OK) return st;
  if (gate && !k_new) return fail(BCT_ERR_INVALID_ARG, "a gate needs a write (k_new, v_new)");
  if (((uintptr_t)gate & 3u) != 0) return fail(BCT_ERR_MISALIGNED, "gate must be 4-byte aligned");
  st = run_decode(c, c->ws, q, k_new, v_new, out, (uint64_t)c->desc.n_q_heads * c->desc.head_dim,
                  (uint64_t)c->desc.n_kv_heads * c->desc.head_dim, gate, c->desc.n_kv_heads, (hipStream_t)hip_stream);
  if (st != BCT_OK) return st;
  c->steps += 1;
  return BCT_OK;
}

bct_status bct_decode_step(bct_cache* c, const void* q, const void* k_new, const void* v_new, void* out,
                           void* hip_stream) {
  return bct_decode_step_gated(c, q, k_new, v_new, nullptr, out, hip_stream);
}

bct_status bct_decode_step_keyed(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                                 const void* key_new, const float* gate, const float* key_gate, void* out,
                                 void* hip_stream) {
  bct_status st = check_io(c, q, k_new, v_new, out);
  if (st != BCT_OK) return st;
  if (!k_new || !key_new) return fail(BCT_ERR_INVALID_ARG, "the keyed step needs a write (k_new, v_new) and key_new");
  if (!aligned16(key_new)) return fail(BCT_ERR_MISALIGNED, "key_new must be 16-byte aligned");
  if ((((uintptr_t)gate) | ((uintptr_t)key_gate)) & 3u) return fail(BCT_ERR_MISALIGNED, "gates must be 4-byte aligned");
  if (!(c->desc.flags & BCT_MK_PER_SEQUENCE))
    return fail(BCT_ERR_STATE, "the keys are shared by the batch: only per-sequence keys (BCT_MK_PER_SEQUENCE) can be written");
  st = run_decode(c, c->ws, q, k_new, v_new, out, (uint64_t)c->desc.n_q_heads * c->desc.head_dim,
                  (uint64_t)c->desc.n_kv_heads * c->desc.head_dim, gate, c->desc.n_kv_heads, (hipStream_t)hip_stream,
                  key_new, key_gate);
  if (st != BCT_OK) return st;
  c->steps += 1;
  return BCT_OK;
}

size_t bct_static_scratch_bytes(void) { return BCT_STATIC_SCRATCH_BYTES; }

bct_status bct_decode_step_static(bct_cache* c, const void* q, const void* k_new, const void* v_new, void* out,
                                  void* hip_stream) {
  bct_status st = check_io(c, q, k_new, v_new, out);
  if (st != BCT_OK) return st;
  if (c->ws_decode_bytes > BCT_STATIC_SCRATCH_BYTES)
    return fail(BCT_ERR_BUFFER_TOO_SMALL,
                "a decode step of this cache needs %zu bytes of scratch, the static scratch holds %zu: "
                "use bct_decode_step with a workspace",
                c->ws_decode_bytes, (size_t)BCT_STATIC_SCRATCH_BYTES);
  char* ws = nullptr;
  if ((st = static_scratch(&ws)) != BCT_OK) return st;
  // Nothing in the scratch has to start at zero: the scores pass writes every score and every
  // (max, sum) pair the later launches read, and the MV pass writes every partial output the
  // merge reads.
  st = run_decode(c, ws, q, k_new, v_new, out, (uint64_t)c->desc.n_q_heads * c->desc.head_dim,
                  (uint64_t)c->desc.n_kv_heads * c->desc.head_dim, nullptr, c->desc.n_kv_heads, (hipStream_t)hip_stream);
  if (st != BCT_OK) return st;
  c->steps += 1;
  return BCT_OK;
}

bct_status bct_prefill_gated(bct_cache* c, const void* q, const void* k_new, const void* v_new, const float* gate,
                             uint32_t T, void* out, void* hip_stream) {
  bct_status st = check_io(c, q, k_new, v_new, out);
  if (st != BCT_OK) return st;
  if (T == 0) return fail(BCT_ERR_INVALID_ARG, "T must be positive");
  if (T > c->max_T) return fail(BCT_ERR_BUFFER_TOO_SMALL, "T %u exceeds max_prefill_T %u given at init", T, c->max_T);
  if (gate && !k_new) return fail(BCT_ERR_INVALID_ARG, "a gate needs a write (k_new, v_new)");
  if (((uintptr_t)gate & 3u) != 0) return fail(BCT_ERR_MISALIGNED, "gate must be 4-byte aligned");
  const size_t sz = esize(c->desc.dtype);
  const uint64_t qs = (uint64_t)c->desc.n_q_heads * c->desc.head_dim;
  const uint64_t ks = (uint64_t)c->desc.n_kv_heads * c->desc.head_dim;
  if (c->desc.dtype == BCT_F32) {
    // fp32 storage: the fp32 running copy of MV IS the stored state, so the
    // chunk is exactly T decode steps in token order.
    for (uint32_t t = 0; t < T; ++t) {
      st = run_decode(c, c->ws, q ? (const char*)q + t * qs * sz : nullptr, k_new ? (const char*)k_new + t * ks * sz : nullptr,
                      v_new ? (const char*)v_new + t * ks * sz : nullptr, out ? (char*)out + t * qs * sz : nullptr,
                      (uint64_t)T * qs, (uint64_t)T * ks, gate ? gate + (size_t)t * c->desc.n_kv_heads : nullptr,
                      (uint64_t)T * c->desc.n_kv_heads, (hipStream_t)hip_stream);
      if (st != BCT_OK) return st;
    }
    c->steps += T;
    return BCT_OK;
  }
  bct::PrefillParams pp;
  memset(&pp, 0, sizeof(pp));
  pp.mk = (const uint16_t*)c->mk;
  pp.mv = (uint16_t*)c->mv;
  pp.q = (const uint16_t*)q;
  pp.wq = (const uint16_t*)k_new;
  pp.wv = (const uint16_t*)v_new;
  pp.out = (uint16_t*)out;
  pp.gate = gate;
  pp.norm_w = (float2*)(c->ws + c->off_pf_norm_w);
  pp.norm_r = (float2*)(c->ws + c->off_pf_norm_r);
  pp.snap = (uint16_t*)(c->ws + c->off_pf_snap);
  pp.wvt = (uint16_t*)(c->ws + c->off_pf_wvt);
  pp.B = c->plan.B;
  pp.Hq = c->plan.Hq;
  pp.Hkv = c->plan.Hkv;
  pp.G = c->plan.G;
  pp.M = c->plan.M;
  pp.d = c->plan.d;
  pp.T = T;
  pp.has_write = k_new ? 1u : 0u;
  pp.has_read = q ? 1u : 0u;
  pp.mk_per_seq = c->plan.mk_per_seq;
  pp.rscale_l2e = c->plan.rscale_l2e;
  pp.wscale_l2e = c->plan.wscale_l2e;
  const hipError_t e = bct::launch_prefill_bf16(pp, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "prefill launch");
  c->steps += T;
  return BCT_OK;
}

bct_status bct_prefill(bct_cache* c, const void* q, const void* k_new, const void* v_new, uint32_t T, void* out,
                       void* hip_stream) {
  return bct_prefill_gated(c, q, k_new, v_new, nullptr, T, out, hip_stream);
}

bct_status bct_cache_export(const bct_cache* c, void* mk_dst, void* mv_dst, uint64_t* steps, void* hip_stream) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if (!aligned16(mk_dst) || !aligned16(mv_dst)) return fail(BCT_ERR_MISALIGNED, "destinations must be 16-byte aligned");
  hipError_t e;
  if (mk_dst && (e = bct::launch_copy(mk_dst, c->mk, c->mk_bytes, (hipStream_t)hip_stream)) != hipSuccess)
    return hip_fail(e, "exporting MK");
  if (mv_dst && (e = bct::launch_copy(mv_dst, c->mv, c->mv_bytes, (hipStream_t)hip_stream)) != hipSuccess)
    return hip_fail(e, "exporting MV");
  if (steps) *steps = c->steps;
  return BCT_OK;
}

bct_status bct_cache_import(bct_cache* c, const void* mk_src, const void* mv_src, uint64_t steps, void* hip_stream) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if (!aligned16(mk_src) || !aligned16(mv_src)) return fail(BCT_ERR_MISALIGNED, "sources must be 16-byte aligned");
  hipError_t e;
  if (mk_src) {
    if ((e = bct::launch_copy(c->mk, mk_src, c->mk_bytes, (hipStream_t)hip_stream)) != hipSuccess)
      return hip_fail(e, "importing MK");
    c->keys_set = true;
  }
  if (mv_src && (e = bct::launch_copy(c->mv, mv_src, c->mv_bytes, (hipStream_t)hip_stream)) != hipSuccess)
    return hip_fail(e, "importing MV");
  c->steps = steps;
  return BCT_OK;
}

bct_status bct_cache_steps(const bct_cache* c, uint64_t* steps) {
  if (!c || !steps) return fail(BCT_ERR_INVALID_ARG, "cache handle or steps is NULL");
  *steps = c->steps;
  return BCT_OK;
}

bct_status bct_plan_query(const bct_cache_desc* desc, bct_plan_info* info) {
  const bct_status st = check_desc(desc);
  if (st != BCT_OK) return st;
  if (!info) return fail(BCT_ERR_INVALID_ARG, "info is NULL");
  bct::DecodeParams p;
  fill_plan(desc, p);
  info->one_launch = p.fused;
  info->scores_mfma = (desc->dtype == BCT_BF16 && !p.mk_per_seq) ? 1u : 0u;
  info->slots_per_stat = p.stat_tile;
  info->normaliser_launch = (!p.fused && !p.fuse_norm) ? 1u : 0u;
  info->mv_workgroup = p.mv_bs;
  info->mv_loads_per_lane = p.mv_u;
  info->mv_splits = p.S;
  info->launches = p.fused ? 1u : 2u + info->normaliser_launch + (p.S > 1 ? 1u : 0u);
  return BCT_OK;
}

bct_status bct_cache_regions(const bct_cache* c, void** mk_dev, size_t* mk_bytes, void** mv_dev, size_t* mv_bytes) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if (mk_dev) *mk_dev = c->mk;
  if (mk_bytes) *mk_bytes = c->mk_bytes;
  if (mv_dev) *mv_dev = c->mv;
  if (mv_bytes) *mv_bytes = c->mv_bytes;
  return BCT_OK;
}

void bct_cache_destroy(bct_cache* c) {
  if (!c) return;
  for (hipEvent_t ev : c->prof_ev) (void)hipEventDestroy(ev);
  delete c;
}

bct_status bct_profile_enable(bct_cache* c, uint32_t n_steps) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  if (n_steps > 65536) return fail(BCT_ERR_INVALID_ARG, "n_steps %u (at most 65536)", n_steps);
  for (hipEvent_t ev : c->prof_ev) (void)hipEventDestroy(ev);
  c->prof_ev.clear();
  c->prof_cap = c->prof_n = 0;
  for (uint32_t i = 0; i < n_steps * 4; ++i) {
    hipEvent_t ev;
    const hipError_t e = hipEventCreate(&ev);
    if (e != hipSuccess) {
      for (hipEvent_t x : c->prof_ev) (void)hipEventDestroy(x);
      c->prof_ev.clear();
      return hip_fail(e, "hipEventCreate");
    }
    c->prof_ev.push_back(ev);
  }
  c->prof_cap = n_steps;
  return BCT_OK;
}

bct_status bct_profile_read(bct_cache* c, uint32_t* n_recorded, float* ms_scores, float* ms_mv_pass,
                            float* ms_merge) {
  if (!c) return fail(BCT_ERR_INVALID_ARG, "cache handle is NULL");
  double acc[3] = {0, 0, 0};
  for (uint32_t i = 0; i < c->prof_n; ++i) {
    hipEvent_t* ev = &c->prof_ev[(size_t)i * 4];
    hipError_t e = hipEventSynchronize(ev[3]);
    if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
    for (int k = 0; k < 3; ++k) {
      float ms = 0.f;
      if ((e = hipEventElapsedTime(&ms, ev[k], ev[k + 1])) != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
      acc[k] += ms;
    }
  }
  const double n = c->prof_n ? (double)c->prof_n : 1.0;
  if (n_recorded) *n_recorded = c->prof_n;
  if (ms_scores) *ms_scores = (float)(acc[0] / n);
  if (ms_mv_pass) *ms_mv_pass = (float)(acc[1] / n);
  if (ms_merge) *ms_merge = (float)(acc[2] / n);
  c->prof_n = 0;
  return BCT_OK;
}

const char* bct_strerror(bct_status s) {
  switch (s) {
    case BCT_OK: return "ok";
    case BCT_ERR_INVALID_ARG: return "invalid argument";
    case BCT_ERR_UNSUPPORTED: return "unsupported shape, dtype or flag";
    case BCT_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case BCT_ERR_MISALIGNED: return "misaligned pointer";
    case BCT_ERR_STATE: return "call out of order";
    case BCT_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

const char* bct_last_error(void) { return g_err; }

bct_status bct_stream_copy(void* dst, const void* src, size_t n_bytes, void* hip_stream) {
  if (!dst || !src) return fail(BCT_ERR_INVALID_ARG, "dst or src is NULL");
  if (n_bytes % 16 != 0) return fail(BCT_ERR_INVALID_ARG, "n_bytes must be a multiple of 16");
  if (!aligned16(dst) || !aligned16(src)) return fail(BCT_ERR_MISALIGNED, "dst and src must be 16-byte aligned");
  const hipError_t e = bct::launch_copy(dst, src, n_bytes, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "copy launch");
  return BCT_OK;
}

}  // extern "C"
