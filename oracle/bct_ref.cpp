// libbct_ref -- CPU oracle for the Bounded-Cache Transformer decode path.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
// step-by-step statement of what the path computes, written from the paper
// (arXiv 2411.15785), used only by the tests, the smoke check and the
// cpu_baseline leg of the benchmark.  It shares no code, header, table or
// helper with the HIP library and neither includes the other.
//
// What is computed (paper section 3.1, 3.2, Algorithm 1, section 3.4):
//   state   MK : M key vectors per KV head      (static input of Algorithm 1)
//           MV : M key-value vectors per (batch, KV head)   (section 3.1)
//   write   score = wq . MK^T                   (section 3.2 step 2; Alg. 1)
//           ww    = softmax(score)              (section 3.2 step 2; Alg. 1)
//           MV    = MV' + ww^T . wv             (section 3.2 step 4; 3.4 eq.)
//           MV stored back for the next step    (section 3.2 step 5)
//   read    out   = softmax(read_scale * q . MK^T) . MV
//           The paper applies the mechanism to the attention layers of a
//           decoder-only Transformer (sections 1 and 3.1) and never writes
//           the read out; standard softmax attention of the
//           layer's query over keys MK and values MV is the reading taken.
//
// Readings where the paper is silent or at odds with itself:
//   * Every token writes, the first one included (section 3.2 steps 3-4 and
//     the section 3.4 equation have no first-token exception; Algorithm 1's
//     t = 1 branch is reachable by passing no write on that step).
//   * Token t's read sees its own write (section 3.2 step 5 stores the
//     updated MV back for the steps that follow; a causal token attends to
//     itself).
//   * MK is never modified by any step of the paper's method.  The one exception is the keyed step
//     below (bct_ref_decode_step_keyed), a widening that the paper only gestures at (section 3.5,
//     the adaptive update rule: no equation): the section 3.4 update applied to the key table too,
//     MK_t = MK_(t-1) + kappa_t * ww_t^T wk_t, with the token's own addressing weights ww_t, which
//     like its read weights come from MK_(t-1); the new keys address the NEXT token.
//   * One independent memory per (batch element, KV head); G = Hq / Hkv
//     query heads read the memory of KV head hq / G; MK is shared over the
//     batch unless per-sequence keys are requested.
//   * write_scale multiplies the write score (1.0 = Algorithm 1 as printed).
//   * Precision: scores, softmax and the read sum in double; the write weight
//     is cast to float; the state update is ONE float fused multiply-add per
//     element, then round-to-nearest-even to the storage dtype (identity for
//     float).  Prefill keeps a float copy of MV for the whole chunk and rounds
//     once at the end of the chunk (the accumulation is order-free: section
//     3.5, "Optimized for Parallelism").
//
// Parity pins (tests/test_oracle_pins.py): brute-force attention, capacity
// invariant, mass conservation, closed form MV_N = MV_0 + WW^T WV, zero-key
// uniform weights, hard-addressing limit (bit exact), M = 1, slot permutation,
// linearity in wv, unit independence / GQA duplication, first-step no-write,
// prefill vs sequential, hand-worked example, bf16 rounding vs a library cast.
// The paper prints no numeric worked example of its own, so output VALUES are
// parity-unpinned against the authors' implementation; every equation the
// paper states is pinned by the list above.

#include <omp.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

namespace {

enum { REF_F32 = 0, REF_BF16 = 1 };
enum { REF_FLAG_MK_PER_SEQUENCE = 1u };

struct RefDesc {
  uint32_t M, B, Hq, Hkv, d;
  int32_t dtype;
  float read_scale, write_scale;
  uint32_t flags;
};

struct RefCache {
  RefDesc ds;
  std::vector<unsigned char> mk;  // [Hkv][M][d] or [B][Hkv][M][d], storage dtype
  std::vector<unsigned char> mv;  // [B][Hkv][M][d], storage dtype
  uint64_t steps;
  bool keys_set;
};

inline size_t esize(int dtype) { return dtype == REF_F32 ? 4 : 2; }

// ---- storage dtype <-> arithmetic ------------------------------------------

inline float bf16_bits_to_float(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// Round a double to the nearest value with `p` significand bits (hidden bit
// included) and minimum exponent emin, ties to even: scale so that the grid
// spacing is 1, round to the nearest integer (ties to even in the default
// rounding mode), scale back.  All scalings are by powers of two, hence exact.
inline double round_to_grid(double x, int p, int emin) {
  if (x == 0.0 || !std::isfinite(x)) return x;
  int e;
  std::frexp(std::fabs(x), &e);  // |x| = f * 2^e, f in [0.5, 1)
  int E = e - 1;
  if (E < emin) E = emin;
  double q = std::ldexp(1.0, E - (p - 1));
  return std::nearbyint(x / q) * q;
}

inline uint16_t double_to_bf16_bits(double x) {
  double r = round_to_grid(x, 8, -126);
  float f = (float)r;  // exact unless r overflowed the float range -> inf
  if (std::fabs(r) >= std::ldexp(1.0, 128)) f = r > 0 ? INFINITY : -INFINITY;
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

// Float -> bf16, ties to even, by the usual integer carry trick.  Pinned in
// the tests against round_to_grid above and against a library cast.
inline uint16_t float_to_bf16_bits(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN stays NaN
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

inline double load_elem(const void* p, size_t i, int dtype) {
  if (dtype == REF_F32) return (double)((const float*)p)[i];
  return (double)bf16_bits_to_float(((const uint16_t*)p)[i]);
}

inline float load_elem_f(const void* p, size_t i, int dtype) {
  if (dtype == REF_F32) return ((const float*)p)[i];
  return bf16_bits_to_float(((const uint16_t*)p)[i]);
}

inline void store_from_float(void* p, size_t i, int dtype, float v) {
  if (dtype == REF_F32) ((float*)p)[i] = v;
  else ((uint16_t*)p)[i] = float_to_bf16_bits(v);
}

inline void store_from_double(void* p, size_t i, int dtype, double v) {
  if (dtype == REF_F32) ((float*)p)[i] = (float)v;
  else ((uint16_t*)p)[i] = double_to_bf16_bits(v);
}

// ---- the method ---------------------------------------------------------------

// softmax(scale * vec . MK^T) over the M slots, in double.
// vec: d elements at element offset voff of `vecs`; keys: M*d elements at koff.
void softmax_weights(const RefCache& c, const void* vecs, size_t voff, size_t koff,
                     double scale, double* w) {
  const uint32_t M = c.ds.M, d = c.ds.d;
  const int dt = c.ds.dtype;
  double mx = -INFINITY;
  for (uint32_t m = 0; m < M; ++m) {
    double acc = 0.0;
    for (uint32_t j = 0; j < d; ++j)
      acc += load_elem(vecs, voff + j, dt) * load_elem(c.mk.data(), koff + (size_t)m * d + j, dt);
    w[m] = scale * acc;
    if (w[m] > mx) mx = w[m];
  }
  double z = 0.0;
  for (uint32_t m = 0; m < M; ++m) {
    w[m] = std::exp(w[m] - mx);
    z += w[m];
  }
  for (uint32_t m = 0; m < M; ++m) w[m] /= z;
}

inline size_t key_offset(const RefCache& c, uint32_t b, uint32_t h) {
  const size_t per_head = (size_t)c.ds.M * c.ds.d;
  if (c.ds.flags & REF_FLAG_MK_PER_SEQUENCE) return ((size_t)b * c.ds.Hkv + h) * per_head;
  return (size_t)h * per_head;
}

// One decode step of one (b, h) memory.  Any of the write (wq, wv) and the
// read (q, out) may be absent.  Vectors are addressed through explicit element
// offsets so that the same routine serves [B][H][d] and [B][T][H][d] inputs.
// wk (optional, with wq): the key write vector of the keyed step at element offset wv_off; kappa its step
// size; wwk: M doubles of scratch for the write weights, which the key update needs after the read.
void unit_decode_step(RefCache& c, uint32_t b, uint32_t h, const void* q, size_t q_off, size_t q_head_stride,
                      const void* wq, size_t wq_off, const void* wv, size_t wv_off, void* out, size_t out_off,
                      size_t out_head_stride, double* w, double eta = 1.0, const void* wk = nullptr,
                      double kappa = 1.0, double* wwk = nullptr) {
  const uint32_t M = c.ds.M, d = c.ds.d, G = c.ds.Hq / c.ds.Hkv;
  const int dt = c.ds.dtype;
  const size_t koff = key_offset(c, b, h);
  const size_t voff = ((size_t)b * c.ds.Hkv + h) * (size_t)M * d;
  void* mv = c.mv.data();

  if (wq) {
    softmax_weights(c, wq, wq_off, koff, (double)c.ds.write_scale, w);
    if (wk)
      for (uint32_t m = 0; m < M; ++m) wwk[m] = w[m];
    for (uint32_t m = 0; m < M; ++m) {
      const float wwm = (float)(eta * w[m]);   // the token's step size scales its write weights
      for (uint32_t j = 0; j < d; ++j) {
        const size_t i = voff + (size_t)m * d + j;
        const float upd = std::fmaf(wwm, load_elem_f(wv, wv_off + j, dt), load_elem_f(mv, i, dt));
        store_from_float(mv, i, dt, upd);
      }
    }
  }
  if (q) {
    std::vector<double> acc(d);
    for (uint32_t g = 0; g < G; ++g) {
      softmax_weights(c, q, q_off + (size_t)g * q_head_stride, koff, (double)c.ds.read_scale, w);
      for (uint32_t j = 0; j < d; ++j) acc[j] = 0.0;
      for (uint32_t m = 0; m < M; ++m)
        for (uint32_t j = 0; j < d; ++j) acc[j] += w[m] * load_elem(mv, voff + (size_t)m * d + j, dt);
      for (uint32_t j = 0; j < d; ++j) store_from_double(out, out_off + (size_t)g * out_head_stride + j, dt, acc[j]);
    }
  }
  if (wq && wk) {
    // the keys move last: the token's write and read were addressed through MK_(t-1)
    void* mk = c.mk.data();
    for (uint32_t m = 0; m < M; ++m) {
      const float kwm = (float)(kappa * wwk[m]);
      for (uint32_t j = 0; j < d; ++j) {
        const size_t i = koff + (size_t)m * d + j;
        const float upd = std::fmaf(kwm, load_elem_f(wk, wv_off + j, dt), load_elem_f(mk, i, dt));
        store_from_float(mk, i, dt, upd);
      }
    }
  }
}

// A chunk of T tokens for one (b, h) memory: the same recurrence, with MV held
// in float for the whole chunk and rounded to the storage dtype once at the end.
void unit_prefill(RefCache& c, uint32_t b, uint32_t h, const void* q, const void* wq, const void* wv,
                  const float* gate, uint32_t T, void* out, double* w, float* shadow) {
  const uint32_t M = c.ds.M, d = c.ds.d, Hq = c.ds.Hq, Hkv = c.ds.Hkv, G = Hq / Hkv;
  const int dt = c.ds.dtype;
  const size_t koff = key_offset(c, b, h);
  const size_t voff = ((size_t)b * Hkv + h) * (size_t)M * d;
  void* mv = c.mv.data();
  for (size_t i = 0; i < (size_t)M * d; ++i) shadow[i] = load_elem_f(mv, voff + i, dt);
  std::vector<double> acc(d);
  for (uint32_t t = 0; t < T; ++t) {
    if (wq) {
      const size_t woff = (((size_t)b * T + t) * Hkv + h) * d;
      softmax_weights(c, wq, woff, koff, (double)c.ds.write_scale, w);
      const double eta = gate ? (double)gate[((size_t)b * T + t) * Hkv + h] : 1.0;
      for (uint32_t m = 0; m < M; ++m) {
        const float wwm = (float)(eta * w[m]);
        for (uint32_t j = 0; j < d; ++j)
          shadow[(size_t)m * d + j] = std::fmaf(wwm, load_elem_f(wv, woff + j, dt), shadow[(size_t)m * d + j]);
      }
    }
    if (q) {
      for (uint32_t g = 0; g < G; ++g) {
        const size_t qoff = (((size_t)b * T + t) * Hq + (size_t)h * G + g) * d;
        softmax_weights(c, q, qoff, koff, (double)c.ds.read_scale, w);
        for (uint32_t j = 0; j < d; ++j) acc[j] = 0.0;
        for (uint32_t m = 0; m < M; ++m)
          for (uint32_t j = 0; j < d; ++j) acc[j] += w[m] * (double)shadow[(size_t)m * d + j];
        for (uint32_t j = 0; j < d; ++j) store_from_double(out, qoff + j, dt, acc[j]);
      }
    }
  }
  if (wq)
    for (size_t i = 0; i < (size_t)M * d; ++i) store_from_float(mv, voff + i, dt, shadow[i]);
}

bool desc_ok(const RefDesc& d) {
  if (d.M == 0 || d.B == 0 || d.Hq == 0 || d.Hkv == 0 || d.d == 0) return false;
  if (d.Hq % d.Hkv != 0) return false;
  if (d.dtype != REF_F32 && d.dtype != REF_BF16) return false;
  return true;
}

}  // namespace

extern "C" {

typedef struct RefCache bct_ref_cache;

int bct_ref_cache_create(const RefDesc* ds, bct_ref_cache** out) {
  if (!ds || !out || !desc_ok(*ds)) return 1;
  RefCache* c = new (std::nothrow) RefCache();
  if (!c) return 1;
  c->ds = *ds;
  const size_t per_head = (size_t)ds->M * ds->d * esize(ds->dtype);
  const size_t nk = (ds->flags & REF_FLAG_MK_PER_SEQUENCE) ? (size_t)ds->B * ds->Hkv : (size_t)ds->Hkv;
  c->mk.assign(nk * per_head, 0);
  c->mv.assign((size_t)ds->B * ds->Hkv * per_head, 0);  // MV_0 = 0 (section 3.1)
  c->steps = 0;
  c->keys_set = false;
  *out = c;
  return 0;
}

void bct_ref_cache_destroy(bct_ref_cache* c) { delete c; }

// Bytes of state held for this cache: constant for its whole life.
size_t bct_ref_cache_bytes(const bct_ref_cache* c) { return c ? c->mk.size() + c->mv.size() : 0; }
size_t bct_ref_keys_bytes(const bct_ref_cache* c) { return c ? c->mk.size() : 0; }
size_t bct_ref_values_bytes(const bct_ref_cache* c) { return c ? c->mv.size() : 0; }

int bct_ref_cache_set_keys(bct_ref_cache* c, const void* mk) {
  if (!c || !mk) return 1;
  std::memcpy(c->mk.data(), mk, c->mk.size());
  c->keys_set = true;
  return 0;
}

// mv0 == NULL -> zero (section 3.1: MV_0 may be zero or random).
int bct_ref_cache_set_values(bct_ref_cache* c, const void* mv0) {
  if (!c) return 1;
  if (mv0) std::memcpy(c->mv.data(), mv0, c->mv.size());
  else std::memset(c->mv.data(), 0, c->mv.size());
  return 0;
}

// MV := random values (section 3.1 allows random initial contents; the distribution is not
// given).  Element i (flat index of [B][Hkv][M][d]) is amplitude * u_i, u_i uniform on the 2^24-point
// grid of [-1, 1): u_i = ((z_i >> 40) - 2^23) / 2^23 with z_i the (i + 1)-th output of the splitmix64
// generator (Steele, Lea, Flood 2014) started at `seed`; the product is one fp32 multiplication,
// then one rounding to the storage dtype.  Every step is exact or a single IEEE rounding, so another
// implementation can reproduce the bits.
uint64_t splitmix64_at(uint64_t seed, uint64_t n) {  // n-th output, n >= 1
  uint64_t z = seed + n * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

int bct_ref_cache_randomize_values(bct_ref_cache* c, uint64_t seed, float amplitude) {
  if (!c || !std::isfinite(amplitude)) return 1;
  const size_t n = (size_t)c->ds.B * c->ds.Hkv * c->ds.M * c->ds.d;
  for (size_t i = 0; i < n; ++i) {
    const int32_t k = (int32_t)(splitmix64_at(seed, (uint64_t)i + 1) >> 40) - (1 << 23);
    const float u = (float)k * (1.0f / 8388608.0f);
    store_from_float(c->mv.data(), i, c->ds.dtype, u * amplitude);
  }
  return 0;
}

uint64_t bct_ref_splitmix64_at(uint64_t seed, uint64_t n) { return splitmix64_at(seed, n); }

// One sequence's state, for swapping a session in and out: MV[b] is Hkv * M * d contiguous elements
// (and MK[b] likewise when the keys are per sequence; mk may be NULL).
int bct_ref_cache_export_sequence(const bct_ref_cache* c, uint32_t b, void* mk_dst, void* mv_dst) {
  if (!c || b >= c->ds.B) return 1;
  const size_t per = (size_t)c->ds.Hkv * c->ds.M * c->ds.d * esize(c->ds.dtype);
  if (mv_dst) std::memcpy(mv_dst, c->mv.data() + (size_t)b * per, per);
  if (mk_dst) {
    if (!(c->ds.flags & REF_FLAG_MK_PER_SEQUENCE)) return 1;
    std::memcpy(mk_dst, c->mk.data() + (size_t)b * per, per);
  }
  return 0;
}

int bct_ref_cache_import_sequence(bct_ref_cache* c, uint32_t b, const void* mk_src, const void* mv_src) {
  if (!c || b >= c->ds.B) return 1;
  const size_t per = (size_t)c->ds.Hkv * c->ds.M * c->ds.d * esize(c->ds.dtype);
  if (mv_src) std::memcpy(c->mv.data() + (size_t)b * per, mv_src, per);
  if (mk_src) {
    if (!(c->ds.flags & REF_FLAG_MK_PER_SEQUENCE)) return 1;
    std::memcpy(c->mk.data() + (size_t)b * per, mk_src, per);
  }
  return 0;
}

int bct_ref_cache_export(const bct_ref_cache* c, void* mk_dst, void* mv_dst, uint64_t* steps) {
  if (!c) return 1;
  if (mk_dst) std::memcpy(mk_dst, c->mk.data(), c->mk.size());
  if (mv_dst) std::memcpy(mv_dst, c->mv.data(), c->mv.size());
  if (steps) *steps = c->steps;
  return 0;
}

int bct_ref_cache_import(bct_ref_cache* c, const void* mk_src, const void* mv_src, uint64_t steps) {
  if (!c) return 1;
  if (mk_src) {
    std::memcpy(c->mk.data(), mk_src, c->mk.size());
    c->keys_set = true;
  }
  if (mv_src) std::memcpy(c->mv.data(), mv_src, c->mv.size());
  c->steps = steps;
  return 0;
}

int bct_ref_cache_steps(const bct_ref_cache* c, uint64_t* steps) {
  if (!c || !steps) return 1;
  *steps = c->steps;
  return 0;
}

// q, out: [B][Hq][d]; wq (k_new), wv (v_new): [B][Hkv][d]; storage dtype.
// wq == wv == NULL: read-only step.  q == out == NULL: write-only step
// (Algorithm 1 alone).  Any other NULL mix is an error.  5 = keys not set.
// gate: NULL, or one step size per memory, float [B][Hkv] (the "learning rate adaptation" item of
// section 3.5 read as a per-token scalar on the write: MV <- MV + eta * ww^T wv).  Needs a write.
int bct_ref_decode_step_gated(bct_ref_cache* c, const void* q, const void* wq, const void* wv, const float* gate,
                              void* out) {
  if (!c) return 1;
  if (gate && !wq) return 1;
  if ((wq == nullptr) != (wv == nullptr)) return 1;
  if ((q == nullptr) != (out == nullptr)) return 1;
  if (!q && !wq) return 1;
  if (!c->keys_set) return 5;
  const uint32_t B = c->ds.B, Hkv = c->ds.Hkv, Hq = c->ds.Hq, d = c->ds.d, G = Hq / Hkv;
  const long units = (long)B * Hkv;
#pragma omp parallel
  {
    std::vector<double> w(c->ds.M);
#pragma omp for schedule(static)
    for (long u = 0; u < units; ++u) {
      const uint32_t b = (uint32_t)(u / Hkv), h = (uint32_t)(u % Hkv);
      const size_t kv_off = ((size_t)b * Hkv + h) * d;
      const size_t q_off = ((size_t)b * Hq + (size_t)h * G) * d;
      unit_decode_step(*c, b, h, q, q_off, d, wq, kv_off, wv, kv_off, out, q_off, d, w.data(),
                       gate ? (double)gate[(size_t)b * Hkv + h] : 1.0);
    }
  }
  c->steps += 1;
  return 0;
}

int bct_ref_decode_step(bct_ref_cache* c, const void* q, const void* wq, const void* wv, void* out) {
  return bct_ref_decode_step_gated(c, q, wq, wv, nullptr, out);
}

// The keyed step: a decode step whose write also moves the keys (per-sequence keys only).
// wk: [B][Hkv][d], the key write vectors; kgate: NULL (1 everywhere) or float [B][Hkv], their step
// sizes kappa.  Per memory, in this order: ww = softmax(write_scale * wq . MK^T); MV += eta ww^T wv;
// out = softmax(read_scale * q . MK^T) . MV; MK += kappa ww^T wk (one float fused multiply-add per
// element, rounded to the storage dtype, like MV).  The write (wq, wv) must be present; the read is
// optional.  2 = keys shared by the batch.
int bct_ref_decode_step_keyed(bct_ref_cache* c, const void* q, const void* wq, const void* wv, const void* wk,
                              const float* gate, const float* kgate, void* out) {
  if (!c || !wq || !wv || !wk) return 1;
  if ((q == nullptr) != (out == nullptr)) return 1;
  if (!(c->ds.flags & REF_FLAG_MK_PER_SEQUENCE)) return 2;
  if (!c->keys_set) return 5;
  const uint32_t B = c->ds.B, Hkv = c->ds.Hkv, Hq = c->ds.Hq, d = c->ds.d, G = Hq / Hkv;
  const long units = (long)B * Hkv;
#pragma omp parallel
  {
    std::vector<double> w(c->ds.M), wwk(c->ds.M);
#pragma omp for schedule(static)
    for (long u = 0; u < units; ++u) {
      const uint32_t b = (uint32_t)(u / Hkv), h = (uint32_t)(u % Hkv);
      const size_t kv_off = ((size_t)b * Hkv + h) * d;
      const size_t q_off = ((size_t)b * Hq + (size_t)h * G) * d;
      unit_decode_step(*c, b, h, q, q_off, d, wq, kv_off, wv, kv_off, out, q_off, d, w.data(),
                       gate ? (double)gate[(size_t)b * Hkv + h] : 1.0, wk,
                       kgate ? (double)kgate[(size_t)b * Hkv + h] : 1.0, wwk.data());
    }
  }
  c->steps += 1;
  return 0;
}

// q, out: [B][T][Hq][d]; wq, wv: [B][T][Hkv][d].  Same NULL conventions.
// gate: NULL, or float [B][T][Hkv].
int bct_ref_prefill_gated(bct_ref_cache* c, const void* q, const void* wq, const void* wv, const float* gate,
                          uint32_t T, void* out) {
  if (!c || T == 0) return 1;
  if (gate && !wq) return 1;
  if ((wq == nullptr) != (wv == nullptr)) return 1;
  if ((q == nullptr) != (out == nullptr)) return 1;
  if (!q && !wq) return 1;
  if (!c->keys_set) return 5;
  const uint32_t B = c->ds.B, Hkv = c->ds.Hkv;
  const long units = (long)B * Hkv;
#pragma omp parallel
  {
    std::vector<double> w(c->ds.M);
    std::vector<float> shadow((size_t)c->ds.M * c->ds.d);
#pragma omp for schedule(static)
    for (long u = 0; u < units; ++u) {
      const uint32_t b = (uint32_t)(u / Hkv), h = (uint32_t)(u % Hkv);
      unit_prefill(*c, b, h, q, wq, wv, gate, T, out, w.data(), shadow.data());
    }
  }
  c->steps += T;
  return 0;
}

int bct_ref_prefill(bct_ref_cache* c, const void* q, const void* wq, const void* wv, uint32_t T, void* out) {
  return bct_ref_prefill_gated(c, q, wq, wv, nullptr, T, out);
}

// Test probes: the softmax weights of one vector (d storage-dtype elements)
// against the keys of memory (b, h), in double; and the two rounding routines.
int bct_ref_probe_weights(const bct_ref_cache* c, uint32_t b, uint32_t h, const void* vec, double scale, double* w) {
  if (!c || !vec || !w || b >= c->ds.B || h >= c->ds.Hkv) return 1;
  softmax_weights(*c, vec, 0, key_offset(*c, b, h), scale, w);
  return 0;
}

// Threads the outer loop over (batch, KV head) memories will use.
int bct_ref_num_threads(void) { return omp_get_max_threads(); }

uint16_t bct_ref_round_bf16_from_float(float f) { return float_to_bf16_bits(f); }
uint16_t bct_ref_round_bf16_from_double(double x) { return double_to_bf16_bits(x); }

}  // extern "C"
