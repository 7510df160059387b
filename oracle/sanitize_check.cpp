// Runs the CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a small drifting trajectory with
// prefill, retrievals at several budgets, appends, delayed and forced splits, a state import and the capacity
// limits.  Built and run by tests/test_oracle_pins.py; test infrastructure like the oracle itself.
//   g++ -O1 -g -std=c++17 -fsanitize=address,undefined -fno-sanitize-recover=all oracle/sanitize_check.cpp -o check
#include <cstdio>
#include <cstdlib>

#include "dynakv_oracle.cpp"

namespace {
uint64_t rng_state = 0x2511074270ull;
double uniform() {   // xorshift64*, inputs only
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 9007199254740992.0;
}
double gauss() {
  double s = 0.0;
  for (int i = 0; i < 12; ++i) s += uniform();
  return s - 6.0;
}
}  // namespace

int main() {
  const int U = 2, G = 3, d = 16, N0 = 300, M0 = 12, T = 200, P = 5;
  oracle_config c{U, G, d, M0, 40, N0 + T - 8, 4, 3, 0, 1.2f, 2.0f, 0.f, 2, 0, 0, 0};
  void* o = oracle_create(&c);
  std::vector<float> mu((size_t)P * d), K((size_t)U * N0 * d), V(K.size());
  for (float& x : mu) x = (float)(3.0 * gauss());
  for (int u = 0; u < U; ++u)
    for (int i = 0; i < N0; ++i) {
      const int p = (int)(uniform() * P) % P;
      for (int k = 0; k < d; ++k) {
        K[((size_t)u * N0 + i) * d + k] = mu[(size_t)p * d + k] + (float)(0.3 * gauss());
        V[((size_t)u * N0 + i) * d + k] = (float)gauss();
      }
    }
  std::vector<int32_t> init((size_t)U * M0);
  for (int u = 0; u < U; ++u)
    for (int j = 0; j < M0; ++j) init[(size_t)u * M0 + j] = j * (N0 / M0);
  std::vector<double> J((size_t)U * 4);
  if (oracle_build_index(o, K.data(), V.data(), N0, init.data(), J.data())) return 2;
  std::vector<float> q((size_t)U * G * d), kn((size_t)U * d), vn((size_t)U * d);
  std::vector<double> out((size_t)U * G * d), lse((size_t)U * G);
  for (int t = 0; t < T; ++t) {
    for (float& x : mu) x += (float)(0.08 * gauss());
    const int p = (int)(uniform() * P) % P;
    for (int u = 0; u < U; ++u)
      for (int k = 0; k < d; ++k) {
        kn[(size_t)u * d + k] = mu[(size_t)p * d + k] + (float)(0.3 * gauss());
        vn[(size_t)u * d + k] = (float)gauss();
        for (int g = 0; g < G; ++g) q[((size_t)u * G + g) * d + k] = kn[(size_t)u * d + k] + (float)(0.5 * gauss());
      }
    oracle_retrieve_attend(o, q.data(), t % 7 == 0 ? 0 : (t % 5 == 0 ? 1000000 : 64), out.data(), lse.data());
    oracle_append(o, kn.data(), vn.data());       // the last appends exceed max_tokens on purpose
    oracle_split(o);
    if (t == T / 2) {   // export unit 0 and import it into unit 1
      const int M = oracle_num_clusters(o, 0), N = oracle_num_tokens(o, 0);
      std::vector<float> r((size_t)M * d), kk((size_t)N * d), vv((size_t)N * d);
      std::vector<int32_t> n(M), b(M), f(M), off(M + 1), mem(N), sel(M);
      std::vector<double> m2(M);
      oracle_get_clusters(o, 0, r.data(), n.data(), b.data(), f.data(), m2.data());
      oracle_get_members(o, 0, off.data(), mem.data());
      oracle_get_kv(o, 0, kk.data(), vv.data());
      const int ns = oracle_get_selected(o, 0, sel.data(), M);
      if (oracle_import_unit(o, 1, N, kk.data(), vv.data(), M, r.data(), n.data(), b.data(), f.data(), m2.data(),
                             off.data(), mem.data(), oracle_tau(o, 0), ns, sel.data()))
        return 3;
    }
  }
  int64_t ev[3];
  oracle_get_diagnostics(o, 0, nullptr, nullptr, ev);
  std::printf("sanitize_check ok: clusters %d tokens %d splits %lld error %d\n", oracle_num_clusters(o, 0),
              oracle_num_tokens(o, 0), (long long)ev[0], oracle_error(o, 0));
  const bool good = ev[0] > 0 && (oracle_error(o, 0) & 1);
  oracle_destroy(o);
  return good ? 0 : 4;
}
