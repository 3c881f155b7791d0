// Host-only run of the selector for AddressSanitizer / UBSan: random and adversarial inputs (zero, negative, huge,
// NaN and infinite importances, zero times, every time resolution).  Built and run by tests/test_select_sanitizers.py.
#include "et_select.cpp"
#include <cstdio>
#include <random>
#include <vector>
int main() {
  std::mt19937_64 rng(1);
  long runs = 0, ok = 0;
  for (int it = 0; it < 3000; it++) {
    int n = 1 + rng() % 200;
    std::vector<double> imp(n);
    std::vector<uint64_t> dw(n), dy(n);
    int flavour = it % 6;
    for (int i = 0; i < n; i++) {
      double u = (double)(rng() % 2000001) / 1e6 - 1.0;
      imp[i] = flavour == 1 ? 0.0 : flavour == 2 ? -std::fabs(u) : flavour == 3 ? u * 1e300 : u;
      dw[i] = flavour == 4 ? (rng() % 3 ? 0 : rng() % 1000000) : rng() % (flavour == 5 ? (1ull << 40) : 5000000);
      dy[i] = rng() % 4 ? rng() % 5000000 : 0;
    }
    if (it % 97 == 0) imp[rng() % n] = NAN;
    if (it % 89 == 0) imp[rng() % n] = INFINITY;
    uint64_t fwd = rng() % 50000000;
    uint32_t rho = it % 11 == 0 ? 0 : (uint32_t)(rng() % 1200001);
    uint32_t tqs[] = {1, 2, 10, 100, 1000, 10000, 100000};
    uint32_t tq = tqs[rng() % 7];
    std::vector<uint8_t> mask(n, 7);
    uint64_t pred = 0;
    et_select_counts cnt;
    int rc = (it & 1) ? et_select(n, imp.data(), dw.data(), dy.data(), fwd, rho, tq, mask.data(), &pred)
                      : et_select_stats(n, imp.data(), dw.data(), dy.data(), fwd, rho, tq, mask.data(), &pred, &cnt);
    runs++;
    if (rc == 0) {
      ok++;
      // the returned mask must respect the budget under the time model
      long double t = fwd; int jstar = -1;
      for (int i = 0; i < n; i++) if (mask[i]) { if (jstar < 0) jstar = i; t += dw[i]; }
      if (jstar >= 0) for (int i = jstar + 1; i < n; i++) t += dy[i];
      if ((uint64_t)t != pred) { printf("predicted mismatch it=%d\n", it); return 1; }
    }
  }
  // degenerate arguments
  uint8_t m; uint64_t p; double one = 1.0; uint64_t z = 0;
  printf("n=0 -> %d, null -> %d, tq=0 -> %d\n", et_select(0, &one, &z, &z, 1, 500000, 100, &m, &p), et_select(1, nullptr, &z, &z, 1, 500000, 100, &m, &p),
         et_select(1, &one, &z, &z, 1, 500000, 0, &m, &p));
  printf("runs %ld, status 0 in %ld\n", runs, ok);
  return 0;
}
