// Sanitizer run of the oracle: exact-size heap buffers, every entry point, both dtypes, GQA, per-sequence keys.
#include "../oracle/bct_ref.cpp"
#include <cstdio>
#include <vector>
#include <random>
int main() {
  std::mt19937 rng(7);
  for (int dtype = 0; dtype < 2; ++dtype)
    for (int flags = 0; flags < 2; ++flags) {
      RefDesc d{};
      d.M = 64; d.B = 3; d.Hq = 4; d.Hkv = 2; d.d = 64; d.dtype = dtype;
      d.read_scale = 0.125f; d.write_scale = 0.125f; d.flags = flags;
      bct_ref_cache* c = nullptr;
      if (bct_ref_cache_create(&d, &c) != 0) { printf("create failed\n"); return 1; }
      const size_t es = dtype == 0 ? 4 : 2;
      std::vector<unsigned char> mk(bct_ref_keys_bytes(c)), mv(bct_ref_values_bytes(c));
      auto fill = [&](std::vector<unsigned char>& v) {
        for (size_t i = 0; i < v.size() / es; ++i) {
          float f = (float)((int)(rng() % 2001) - 1000) / 1000.0f;
          if (es == 4) memcpy(&v[4 * i], &f, 4);
          else { uint32_t u; memcpy(&u, &f, 4); uint16_t h = (uint16_t)(u >> 16); memcpy(&v[2 * i], &h, 2); }
        }
      };
      fill(mk); fill(mv);
      bct_ref_cache_set_keys(c, mk.data());
      bct_ref_cache_set_values(c, mv.data());
      const uint32_t T = 5;
      std::vector<unsigned char> q((size_t)3 * T * 4 * 64 * es), wq((size_t)3 * T * 2 * 64 * es), wv(wq.size()), out(q.size());
      std::vector<float> gate((size_t)3 * T * 2, 0.5f);
      fill(q); fill(wq); fill(wv);
      // single steps use the first B*H*d elements of the buffers (exact-size copies to catch overreads)
      std::vector<unsigned char> q1(q.begin(), q.begin() + 3 * 4 * 64 * es), wq1(wq.begin(), wq.begin() + 3 * 2 * 64 * es),
          wv1(wv.begin(), wv.begin() + 3 * 2 * 64 * es), out1(q1.size());
      std::vector<float> gate1(3 * 2, 0.25f);
      int rc = 0;
      rc |= bct_ref_decode_step(c, q1.data(), wq1.data(), wv1.data(), out1.data());
      rc |= bct_ref_decode_step(c, q1.data(), nullptr, nullptr, out1.data());
      rc |= bct_ref_decode_step(c, nullptr, wq1.data(), wv1.data(), nullptr);
      rc |= bct_ref_decode_step_gated(c, q1.data(), wq1.data(), wv1.data(), gate1.data(), out1.data());
      if (flags) rc |= bct_ref_decode_step_keyed(c, q1.data(), wq1.data(), wv1.data(), wv1.data(), gate1.data(), gate1.data(), out1.data());
      else rc |= bct_ref_decode_step_keyed(c, q1.data(), wq1.data(), wv1.data(), wv1.data(), nullptr, nullptr, out1.data()) != 2;
      rc |= bct_ref_prefill(c, q.data(), wq.data(), wv.data(), T, out.data());
      rc |= bct_ref_prefill_gated(c, q.data(), wq.data(), wv.data(), gate.data(), T, out.data());
      rc |= bct_ref_prefill(c, nullptr, wq.data(), wv.data(), T, nullptr);
      rc |= bct_ref_prefill(c, q.data(), nullptr, nullptr, T, out.data());
      rc |= bct_ref_cache_randomize_values(c, 12345, 0.5f);
      std::vector<unsigned char> mk2(mk.size()), mv2(mv.size());
      uint64_t steps = 0;
      rc |= bct_ref_cache_export(c, mk2.data(), mv2.data(), &steps);
      rc |= bct_ref_cache_import(c, mk2.data(), mv2.data(), steps);
      std::vector<unsigned char> smv(mv.size() / 3), smk(flags ? mk.size() / 3 : 1);
      rc |= bct_ref_cache_export_sequence(c, 2, flags ? smk.data() : nullptr, smv.data());
      rc |= bct_ref_cache_import_sequence(c, 0, flags ? smk.data() : nullptr, smv.data());
      std::vector<double> w(64);
      rc |= bct_ref_probe_weights(c, 2, 1, q1.data(), 0.125, w.data());
      rc |= bct_ref_cache_steps(c, &steps);
      printf("dtype %d flags %d: rc %d, steps %llu\n", dtype, flags, rc, (unsigned long long)steps);
      bct_ref_cache_destroy(c);
      if (rc) return 1;
    }
  printf("oracle sanitizer drive: ok\n");
  return 0;
}
