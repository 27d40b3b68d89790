// Drives every routine of the CPU oracle once on ragged, empty and extreme inputs.  Built by
// tests/test_oracle_sanitizers.py with -fsanitize=address,undefined (any finding aborts), it checks that the
// checker itself reads and writes inside its buffers and has no undefined arithmetic.  It verifies no values: the
// pins in tests/test_oracle_*.py do that.
#include "../oracle/qoda_oracle.cpp"

#include <cstdio>
#include <random>

int main() {
  const std::vector<int64_t> sizes = {1, 3, 0, 127, 128, 129, 2047, 2049, 16385, 40001};
  const int L = (int)sizes.size();
  std::mt19937 rng(7);
  std::normal_distribution<float> gauss(0.0f, 1.0f);
  const int K = 2;
  std::vector<std::vector<std::vector<float>>> g(K, std::vector<std::vector<float>>(L));
  for (int k = 0; k < K; ++k)
    for (int l = 0; l < L; ++l) {
      g[k][l].resize((size_t)sizes[l] + 1);   // one spare entry so that empty layers still have an address
      const float scale = std::pow(10.0f, (float)((l * 7 + k * 3) % 40) - 30.0f);   // 1e-30 ... 1e9
      for (int64_t e = 0; e < sizes[l]; ++e) g[k][l][e] = gauss(rng) * scale;
    }
  for (int S : {2, 3, 8, 17, 256}) {
    std::vector<int32_t> pts(L, S), types(L);
    for (int l = 0; l < L; ++l) types[l] = l % 2;
    const int32_t tp[2] = {S, S};
    std::vector<float> lev(S);
    for (int j = 0; j < S; ++j) lev[j] = (float)j / (float)(S - 1);
    std::vector<const float *> levp(L, lev.data());
    for (int scope = 0; scope < 3; ++scope)
      for (int kind = 0; kind < 3; ++kind) {
        const int64_t mb = oracle_message_bytes(L, sizes.data(), pts.data(), scope);
        std::vector<std::vector<uint8_t>> msg(K, std::vector<uint8_t>((size_t)mb)), msg2 = msg;
        std::vector<const uint8_t *> msgp;
        std::vector<int32_t> lexp(L, 3);
        std::vector<uint64_t> hist((size_t)K * L * kGridPoints, 0);
        std::vector<double> bmax((size_t)K * L, 0.0);
        for (int k = 0; k < K; ++k) {
          std::vector<const float *> gp(L);
          for (int l = 0; l < L; ++l) gp[l] = g[k][l].data();
          std::vector<double> ss(L);
          double delta = 0.0;
          oracle_quantize(L, sizes.data(), pts.data(), levp.data(), gp.data(), 11, 1, k, scope, msg[k].data(), nullptr,
                          ss.data(), &delta, scope == kScopeBucket ? lexp.data() : nullptr,
                          hist.data() + (size_t)k * L * kGridPoints, bmax.data() + (size_t)k * L, kind);
          oracle_quantize(L, sizes.data(), pts.data(), levp.data(), gp.data(), 11, 2, k, scope, msg2[k].data(),
                          msg[k].data(), nullptr, &delta, nullptr, nullptr, nullptr, kind);
          (void)oracle_delta_from_messages(L, sizes.data(), pts.data(), scope, msg2[k].data(), msg[k].data());
          (void)oracle_delta_plain(L, sizes.data(), pts.data(), scope, msg2[k].data(), nullptr);
          msgp.push_back(msg2[k].data());
        }
        std::vector<std::vector<float>> mean(L);
        std::vector<float *> meanp(L);
        for (int l = 0; l < L; ++l) { mean[l].resize((size_t)sizes[l] + 1); meanp[l] = mean[l].data(); }
        oracle_dequant_aggregate(L, sizes.data(), pts.data(), scope, K, msgp.data(), meanp.data());
        std::vector<uint64_t> counts(2 * 256, 0);
        oracle_index_counts(L, sizes.data(), pts.data(), types.data(), scope, msg2[0].data(), counts.data());
        double rep[6];
        oracle_code_length(2, tp, counts.data(), 5.0, rep);
        // the fit, from vectors and from gathered statistics
        std::vector<const float *> flat;
        for (int k = 0; k < K; ++k)
          for (int l = 0; l < L; ++l) flat.push_back(g[k][l].data());
        std::vector<float> la(lev), lb(lev);
        float *lio[2] = {la.data(), lb.data()};
        std::vector<uint32_t> rawhist((size_t)K * L * kHistBins);
        std::vector<uint64_t> pooled(2 * kGridPoints);
        oracle_fit_levels(L, sizes.data(), types.data(), 2, tp, K, scope, flat.data(), lio, rawhist.data(), pooled.data(), kind);
        int32_t ex[2] = {3, kTypeSkip};
        oracle_fit_from_stats(L, types.data(), 2, tp, K, hist.data(), bmax.data(), ex, lio, pooled.data(), kind);
        (void)oracle_fit_objective(pooled.data(), la.data(), S);
        const float *lvl[2] = {la.data(), lb.data()};
        (void)oracle_mqv_objective_plain(L, sizes.data(), types.data(), tp, K, scope, flat.data(), lvl, kind);
        // updates
        std::vector<std::vector<float>> x1(L), y(L), xn(L), xh(L);
        std::vector<const float *> x1p(L), mp(L);
        std::vector<float *> yp(L), xnp(L), xhp(L);
        for (int l = 0; l < L; ++l) {
          x1[l].assign((size_t)sizes[l] + 1, 0.5f); y[l].assign((size_t)sizes[l] + 1, 0.0f);
          xn[l] = y[l]; xh[l] = y[l];
          x1p[l] = x1[l].data(); mp[l] = mean[l].data(); yp[l] = y[l].data(); xnp[l] = xn[l].data(); xhp[l] = xh[l].data();
          oracle_oda_update(sizes[l], mean[l].data(), x1[l].data(), y[l].data(), xn[l].data(), xh[l].data(), 0.5f, 0.7f);
          oracle_extrapolate(sizes[l], mean[l].data(), x1[l].data(), 0.1f, xh[l].data());
        }
        (void)oracle_oda_update_alt(L, sizes.data(), mp.data(), x1p.data(), yp.data(), xnp.data(), xhp.data(), 1.0f, 0.5f, 0.7f);
      }
  }
  // scalars and single-layer helpers
  float eta, gamma;
  double acc = 0.0, lam = 0.0, mu = 0.0;
  const double d3[3] = {1.0, 2.5, 1e30};
  oracle_step_size(3, d3, &acc, &eta);
  oracle_alt_step_size(3.0, 2.0, 0.25, &eta, &gamma);
  oracle_alt_advance(3, d3, 0.5, &lam, &mu);
  for (double s : {0.0, 1e-300, 1e-80, 1.0, 1e77, 1e300}) (void)oracle_sqrt_floor(s);
  for (float x : {0.0f, 1e-45f, 1e-38f, 1.0f, 3e38f}) (void)oracle_rcp_floor(x);
  std::vector<float> v(5000);
  for (auto &x : v) x = gauss(rng);
  std::vector<uint8_t> sg(v.size()), ix(v.size());
  const float lev4[4] = {0.0f, 0.1f, 0.4f, 1.0f};
  oracle_quantize_range(v.data(), 100, 4999, 0.01f, lev4, 4, 1, 2, 3, 4, sg.data(), ix.data());
  std::vector<uint8_t> region((size_t)((4899 + 2047) / 2048) * (256 * 3 + 64));
  std::vector<float> bn((4899 + 127) / 128, 1.0f);
  oracle_pack_layer(sg.data(), ix.data(), 4899, 4, kScopeBucket, bn.data(), region.data());
  oracle_unpack_layer(region.data(), 4899, 4, kScopeBucket, sg.data(), ix.data(), bn.data());
  std::vector<float> dec(4899);
  oracle_decode(sg.data(), ix.data(), 4899, 2.0f, lev4, 4, dec.data());
  (void)oracle_variance_plain(v.data(), (int64_t)v.size(), lev4, 4, kNormL2);
  (void)oracle_sumsq(v.data(), (int64_t)v.size());
  (void)oracle_bucket_sumsq(v.data(), 128);
  std::vector<uint32_t> h(kHistBins, 0);
  oracle_histogram(v.data(), (int64_t)v.size(), h.data());
  uint64_t cnt[6] = {5, 0, 9, 1, 1, 40};
  (void)oracle_huffman_bits(cnt, 6);
  std::puts("oracle sanitize driver: done");
  return 0;
}
