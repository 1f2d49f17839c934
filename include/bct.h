/* libbct -- Bounded-Cache Transformer decode path on AMD MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only.  Unless a parameter says "host",
 * every data pointer is DEVICE memory owned by the caller; the library never
 * allocates or frees device memory.  A bct_cache handle owns a small host
 * struct only.  All calls that take a stream enqueue work on it and return
 * without synchronising; calls on one cache must be stream-ordered by the
 * caller.  Argument checks run before the first HIP call, so they can be
 * exercised on a machine without a GPU.
 *
 * The method (arXiv 2411.15785):
 *   state   MK  M key vectors per KV head, predefined capacity M (section 3.1);
 *               an input of Algorithm 1 that no step ever assigns to.
 *           MV  M key-value vectors per (batch element, KV head) (section 3.1),
 *               zero or random at the start.
 *   write   ww = softmax(write_scale * wq . MK^T)      (section 3.2 step 2, Alg. 1)
 *           MV = MV' + ww^T . wv  for ALL M slots      (section 3.2 step 4, 3.4 eq.)
 *           stored back in place                       (section 3.2 step 5)
 *   read    out = softmax(read_scale * q . MK^T) . MV  (attention of the layer's
 *           query over the bounded cache; the read follows the write of the same
 *           token)
 * k_new is the paper's write query wq_t, v_new its write key-value vector wv_t,
 * both already projected by the caller (W_wq, W_wv stay outside the library).
 *
 * Layouts (row-major, innermost contiguous, element type = desc.dtype):
 *   q, out        [B][Hq][d]            prefill: [B][T][Hq][d]
 *   k_new, v_new  [B][Hkv][d]           prefill: [B][T][Hkv][d]
 *   MK            [Hkv][M][d]           or [B][Hkv][M][d] with BCT_MK_PER_SEQUENCE
 *   MV            [B][Hkv][M][d]
 * Query head hq reads the memory of KV head hq / (Hq/Hkv).
 * Every pointer must be 16-byte aligned.
 */
#ifndef BCT_H
#define BCT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BCT_OK = 0,
  BCT_ERR_INVALID_ARG = 1,      /* NULL where data is needed, bad NULL mix, zero size   */
  BCT_ERR_UNSUPPORTED = 2,      /* shape / dtype / flag outside what the kernels handle */
  BCT_ERR_BUFFER_TOO_SMALL = 3, /* cache_bytes or workspace_bytes below bct_cache_query */
  BCT_ERR_MISALIGNED = 4,       /* a pointer is not 16-byte aligned                     */
  BCT_ERR_STATE = 5,            /* step before bct_cache_set_keys                       */
  BCT_ERR_HIP = 6               /* a HIP call failed; text in bct_last_error()          */
} bct_status;

typedef enum { BCT_F32 = 0, BCT_BF16 = 1 } bct_dtype;

enum {
  BCT_MK_PER_SEQUENCE = 1u, /* desc.flags: one key table per batch element */
  BCT_STEP_STREAMING = 2u   /* desc.flags: always take the four-launch decode step, also for a cache small
                             * enough for the one-launch step (same results to the stated tolerances;
                             * for comparing the two) */
};

typedef struct {
  uint32_t capacity_M;  /* M > 0, multiple of 64, at most 65536                        */
  uint32_t batch;       /* B > 0                                                       */
  uint32_t n_q_heads;   /* Hq, multiple of n_kv_heads, Hq/Hkv at most 8                */
  uint32_t n_kv_heads;  /* Hkv > 0                                                     */
  uint32_t head_dim;    /* d: 64 or 128                                                */
  int32_t  dtype;       /* bct_dtype: storage and I/O type of MK, MV, q, k_new, v_new, out */
  float    read_scale;  /* multiplies q . MK^T, e.g. 1/sqrt(d)                         */
  float    write_scale; /* multiplies wq . MK^T; 1.0 = Algorithm 1 as printed          */
  uint32_t flags;       /* 0 or an OR of the flags above                               */
} bct_cache_desc;

typedef struct bct_cache bct_cache; /* opaque, host memory */

/* Sizes the caller must provide for a cache of this shape (host call, no GPU
 * needed).  cache_bytes covers MK and MV and never changes afterwards: memory
 * use is constant in the number of tokens (section 4.3).  workspace_bytes is
 * scratch for scores and split-M partial results of one step; max_prefill_T
 * states the longest prefill chunk that workspace must serve (0 = decode only).
 * Either output pointer may be NULL. */
bct_status bct_cache_query(const bct_cache_desc* desc, uint32_t max_prefill_T,
                           size_t* cache_bytes, size_t* workspace_bytes);

/* Creates the handle over caller-owned device memory, sets MV := 0
 * (section 3.1) and steps := 0.  MK is unset until bct_cache_set_keys.
 * Errors: INVALID_ARG, UNSUPPORTED, BUFFER_TOO_SMALL, MISALIGNED, HIP. */
bct_status bct_cache_init(const bct_cache_desc* desc, uint32_t max_prefill_T,
                          void* cache_mem, size_t cache_bytes,
                          void* workspace, size_t workspace_bytes,
                          void* hip_stream, bct_cache** out);

/* Copies the key table (device, MK layout above) into the cache.  The keys
 * are static: no other call writes them (Algorithm 1 takes MK as an input). */
bct_status bct_cache_set_keys(bct_cache* c, const void* mk_dev, void* hip_stream);

/* MV := mv0_dev (device, MV layout), or zero if NULL (section 3.1 lets the
 * initial contents be zero or random).  Does not touch steps. */
bct_status bct_cache_set_values(bct_cache* c, const void* mv0_dev, void* hip_stream);

/* MV := amplitude * u with u uniform on [-1, 1) (section 3.1 allows random initial contents and names
 * no distribution).  Reproducible anywhere: element i of the flat [B][Hkv][M][d] array takes the
 * (i + 1)-th output z of the splitmix64 generator started at seed, u = ((z >> 40) - 2^23) / 2^23,
 * one fp32 multiplication by amplitude, one rounding to the storage dtype.  Does not touch steps. */
bct_status bct_cache_randomize_values(bct_cache* c, uint64_t seed, float amplitude, void* hip_stream);

/* One token per sequence (section 3.2 steps 2-5 for the write, then the read).
 *   k_new == v_new == NULL : read-only step, MV untouched.
 *   q == out == NULL       : write-only step = one iteration of Algorithm 1.
 *   any other NULL mix     : BCT_ERR_INVALID_ARG.
 * steps += 1.  Errors: INVALID_ARG, MISALIGNED, STATE, HIP. */
bct_status bct_decode_step(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                           void* out, void* hip_stream);

/* For callers that cannot allocate device memory and have no workspace to hand over when they step
 * (code under HIP graph capture, tight serving loops, harnesses that forbid allocation): the same
 * step as bct_decode_step, same arguments, same results bit for bit, but the scratch of its kernels
 * (scores, per-tile statistics, normalisers, split-M partial outputs) is a fixed array inside the
 * library's device image instead of the workspace given to bct_cache_init.  The array holds
 * bct_static_scratch_bytes() bytes (8 MiB) on every GPU the library runs on, for the life of the
 * process; a cache whose decode step needs more returns BCT_ERR_BUFFER_TOO_SMALL (config 2 of the
 * benchmark, B = 8, H = 32, M = 1024, needs 2.3 MiB; config 3 needs 101 MiB and does not fit).  The
 * call makes no allocation of any kind.  The device that is current at the call must be the cache's.
 * All calls on one GPU share that GPU's array (it keeps the last call's contents; nothing in it has
 * to be cleared between calls): calls that overlap in time on one GPU, from different streams or
 * threads, race.  Calls on one stream are safe.  Errors: those of bct_decode_step. */
bct_status bct_decode_step_static(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                                  void* out, void* hip_stream);
size_t bct_static_scratch_bytes(void);

/* A chunk of T tokens per sequence (1 <= T <= max_prefill_T), equal to T decode
 * steps in token order except that MV is carried in fp32 through the chunk and
 * rounded to the storage dtype once at its end (the accumulation over tokens is
 * order-free: section 3.5).  Same NULL conventions.  steps += T. */
bct_status bct_prefill(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                       uint32_t T, void* out, void* hip_stream);

/* The same two calls with a step size per token (section 3.5 lists a "learning rate adaptation" that
 * sets the step size of each token, without an equation; taken here as one scalar eta_t per memory on
 * the write: MV <- MV + eta_t * ww^T wv).  gate: DEVICE, float32, [B][n_kv_heads] for a decode step,
 * [B][T][n_kv_heads] for a chunk; NULL = 1 everywhere = the plain call.  eta may be any finite value
 * on every path and dtype: 0 writes nothing, a negative eta subtracts (eta = -1 equals the plain write
 * of -wv, bit for bit); a NaN or infinite eta gives NaN in that memory.  A gate without a write is
 * BCT_ERR_INVALID_ARG.  The read is unchanged. */
bct_status bct_decode_step_gated(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                                 const float* gate, void* out, void* hip_stream);
bct_status bct_prefill_gated(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                             const float* gate, uint32_t T, void* out, void* hip_stream);

/* The keyed step: a decode step whose write also moves the keys.  The paper never assigns MK (Algorithm 1
 * takes it as an input) and names an adaptive update rule without an equation (section 3.5); this call is
 * this library's reading of "keys updated by the same soft write": per memory, after the token's write
 * to MV and its read, both addressed through the keys as they were,
 *     MK = MK + kappa * ww^T . key_new      (the section 3.4 update applied to the key table, with the
 *                                            token's own write weights ww; one fp32 FMA and one rounding
 *                                            to the storage dtype per element)
 * so the moved keys address the NEXT token.  key_new: [B][n_kv_heads][head_dim], storage dtype;
 * key_gate: float32 [B][n_kv_heads] step sizes kappa, NULL = 1; gate as in bct_decode_step_gated.
 * Needs per-sequence keys (BCT_MK_PER_SEQUENCE, else BCT_ERR_STATE) and a write (k_new, v_new); the
 * read (q, out) may be absent.  key_gate = 0 is bct_decode_step_gated bit for bit and leaves MK alone.
 * This is the only call besides bct_cache_set_keys / import that writes MK.  There is no chunk form:
 * unrolling a chunk (section 3.5) needs keys that do not move.  Moves 2 MK more bytes than the plain
 * step (the keys of every sequence are read and written once more). */
bct_status bct_decode_step_keyed(bct_cache* c, const void* q, const void* k_new, const void* v_new,
                                 const void* key_new, const float* gate, const float* key_gate, void* out,
                                 void* hip_stream);

/* Session swap: copies sequence b's slice of the state, MV[b] = n_kv_heads * M * head_dim contiguous
 * elements (device pointers), out of / into the cache; the memory of a sequence has a fixed size
 * whatever its length (section 4.3), so parking a session is one constant-size copy.  mk_* must be
 * NULL unless the keys are per sequence (then MK[b], same size).  The step counter is the cache's
 * and is not touched. */
bct_status bct_cache_export_sequence(const bct_cache* c, uint32_t b, void* mk_dst, void* mv_dst,
                                     void* hip_stream);
bct_status bct_cache_import_sequence(bct_cache* c, uint32_t b, const void* mk_src, const void* mv_src,
                                     void* hip_stream);

/* Checkpoint.  The whole recurrent state of a layer is (MK, MV_t): section 3.2 step 3 retrieves the
 * previous MV from the cache and step 5 stores the updated one back, so continuing a stream elsewhere
 * or later needs exactly these bytes.  Copies MK and/or MV out of / into the cache (device pointers,
 * either may be NULL) together with the step counter (host).  bct_cache_import with both pointers
 * NULL only sets the counter. */
bct_status bct_cache_export(const bct_cache* c, void* mk_dst, void* mv_dst, uint64_t* steps,
                            void* hip_stream);
bct_status bct_cache_import(bct_cache* c, const void* mk_src, const void* mv_src, uint64_t steps,
                            void* hip_stream);

/* Tokens written or read through this handle so far.  The counter lives in the host handle and counts
 * CALLS (a decode step 1, a chunk T): replaying a captured HIP graph steps the cache on the GPU without
 * a call, so after graph replays the caller adds the replayed steps itself (bct_cache_import(c, NULL,
 * NULL, steps) sets the counter).  Nothing on the GPU depends on it. */
bct_status bct_cache_steps(const bct_cache* c, uint64_t* steps);

/* The launch plan the library would use for a decode step (section 3.2 steps 2-5 and the read) of this
 * descriptor: how many launches, and the shape of the pass over MV.  Host logic only (no GPU needed);
 * for inspection, tests and for naming the kernel a measurement belongs to. */
typedef struct bct_plan_info {
  uint32_t launches;          /* kernels per decode step with both a write and a read: 1, 3 or 4       */
  uint32_t one_launch;        /* 1: the small-cache single-workgroup step                               */
  uint32_t scores_mfma;       /* 1: scores by MFMA (bf16, keys shared by the batch), else dot products  */
  uint32_t slots_per_stat;    /* slots per (max, sum) partial of the scores pass                        */
  uint32_t normaliser_launch; /* 1: the partials are merged by a launch of their own                    */
  uint32_t mv_workgroup;      /* threads per workgroup of the MV pass                                   */
  uint32_t mv_loads_per_lane; /* 16-byte loads each lane of the MV pass has in flight                   */
  uint32_t mv_splits;         /* workgroups per memory in the MV pass (> 1: a merge launch follows)     */
} bct_plan_info;
bct_status bct_plan_query(const bct_cache_desc* desc, bct_plan_info* info);

/* Device addresses of the two regions inside cache_mem, MK first, then MV (section 3.1's two
 * sequences), for zero-copy views of the state: the bounded-cache layout in HBM as the caller sees it. */
bct_status bct_cache_regions(const bct_cache* c, void** mk_dev, size_t* mk_bytes,
                             void** mv_dev, size_t* mv_bytes);

/* Frees the host handle only; device memory stays with the caller. */
void bct_cache_destroy(bct_cache* c);

const char* bct_strerror(bct_status s);
const char* bct_last_error(void); /* thread-local detail of the last failure */

#ifdef __cplusplus
}
#endif
#endif /* BCT_H */
