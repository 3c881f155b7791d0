// Tensor Selector: exact integer solution of Eq. 3 (Sections 3.3 and 6).  Host only.
//
// The paper's dynamic programme indexes subproblems by backward depth and scans the closest
// selected tensor (Eq. 7), O(N^2 T_q).  The cost of a mask depends on its selection only through
// (a) the input-most selected tensor i*, which fixes the gradient-passing time sum_{i>i*} t_dy[i],
// and (b) the sum of t_dw over the selected tensors.  So for every candidate i* the best mask is
// i* plus an ordinary 0/1 knapsack over the tensors output-side of i* with the remaining budget,
// and one knapsack table built from the output side serves every i*: O(N T_q).  Same optimum,
// same tie order (larger summed importance, then the smallest mask read as a binary number with
// tensor 0 as the most significant bit).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "et.h"

namespace {

typedef unsigned __int128 u128;

// floor(a * b / c) without overflow
inline uint64_t muldiv(uint64_t a, uint64_t b, uint64_t c) { return (uint64_t)(((u128)a * (u128)b) / (u128)c); }

uint64_t time_model(int32_t n, const uint8_t* mask, const uint64_t* t_dw, const uint64_t* t_dy, uint64_t t_fwd) {
  int32_t first = -1;
  for (int32_t i = 0; i < n; i++)
    if (mask[i]) { first = i; break; }
  uint64_t t = t_fwd;
  if (first < 0) return t;
  for (int32_t i = first; i < n; i++) {
    if (mask[i]) t += t_dw[i];
    if (i > first) t += t_dy[i];
  }
  return t;
}

}  // namespace

static int select_core(int32_t n, const double* importance, const uint64_t* t_dw_ns, const uint64_t* t_dy_ns,
                uint64_t t_fwd_ns, uint32_t rho_ppm, uint32_t tq, uint8_t* mask_out, uint64_t* predicted_ns,
                et_select_counts* counts) {
  if (n <= 0 || !importance || !t_dw_ns || !t_dy_ns || !mask_out) return ET_EINVAL;
  if (counts) *counts = et_select_counts{0, 0, 0, 0, 0};
  for (int32_t i = 0; i < n; i++) mask_out[i] = 0;
  if (predicted_ns) *predicted_ns = t_fwd_ns;
  // no single time may push the 64-bit sums over the edge
  uint64_t t_b = 0;
  for (int32_t i = 0; i < n; i++) {
    uint64_t add = t_dw_ns[i] + (i >= 1 ? t_dy_ns[i] : 0);
    if (t_dw_ns[i] > (UINT64_MAX >> 2) || t_dy_ns[i] > (UINT64_MAX >> 2) || t_b + add < t_b || t_b + add > (UINT64_MAX >> 1))
      return ET_EINVAL;
    t_b += add;
  }
  if (t_fwd_ns > (UINT64_MAX >> 1) - t_b) return ET_EINVAL;
  const uint64_t t_full = t_fwd_ns + t_b;

  // ---- importance -> integers with 40 significant bits below the largest magnitude
  double imax = 0.0;
  for (int32_t i = 0; i < n; i++) {
    if (!std::isfinite(importance[i])) return ET_ENAN;
    imax = std::fmax(imax, std::fabs(importance[i]));
  }
  try {
    std::vector<int64_t> iq(n, 0);
    if (imax > 0.0) {
      int e = 0;
      std::frexp(imax, &e);
      for (int32_t i = 0; i < n; i++) iq[i] = std::llrint(std::ldexp(importance[i], 40 - e));
    }

    // ---- budget and time resolution (Eq. 8)
    const u128 allowed = ((u128)rho_ppm * (u128)t_full) / 1000000u;
    if (allowed < (u128)t_fwd_ns) return ET_INFEASIBLE;
    u128 budget128 = allowed - (u128)t_fwd_ns;
    if (budget128 > (u128)t_b) budget128 = t_b;  // nothing costs more than the full backward pass
    uint64_t budget = (uint64_t)budget128;
    const bool scale = (tq != 0 && (uint64_t)tq < t_b);
    std::vector<uint64_t> a(n), b(n);
    for (int32_t i = 0; i < n; i++) {
      a[i] = scale ? muldiv(t_dw_ns[i], tq, t_b) : t_dw_ns[i];
      b[i] = scale ? muldiv(t_dy_ns[i], tq, t_b) : t_dy_ns[i];
    }
    if (scale) budget = muldiv(budget, tq, t_b);
    if (counts) {
      // Section 6.3 on the paper's table (depth d = 1..N from the output, time 0..T): a cell is invalid
      // above the budget and redundant below the time of merely reaching depth d
      uint64_t tb_q = 0, reach = 0;
      for (int32_t i = 0; i < n; i++) tb_q += a[i] + (i >= 1 ? b[i] : 0);
      counts->budget_q = budget;
      counts->backward_q = tb_q;
      counts->cells_table = (uint64_t)n * (std::max(tb_q, budget) + 1);
      counts->cells_knapsack = (uint64_t)n * (budget + 1);
      for (int32_t i = n - 1; i >= 0; i--) {          // depth d = n - i
        if (reach + a[i] <= budget) counts->cells_pruned += budget - reach + 1;
        reach += b[i];
      }
    }
    // The table is kept as two rolling value rows plus one take/skip bit per cell for the walk back: 1/64 of
    // the memory of a full value table, so nanosecond resolution (tq = 0) on a profile of a few
    // milliseconds stays usable (Section 6.3 wants the selector far below 1 % of the training time).
    if ((u128)(budget + 1) * (u128)(n + 1) > ((u128)1 << 32)) return ET_ENOMEM;  // 512 MiB of bits: choose a coarser tq
    const size_t W = (size_t)budget + 1;
    const size_t WB = (W + 63) / 64;                       // 64-bit words per row of bits

    // ---- the capacity each candidate input-most tensor i* = i leaves for the tensors output-side of it
    //      (reach = sum of b over those tensors); deeper tensors only cost more to reach
    std::vector<uint64_t> cap(n, 0);
    std::vector<uint8_t> fits(n, 0);
    {
      uint64_t reach = 0;
      for (int32_t i = n - 1; i >= 0; i--) {
        if (reach > budget) break;
        if (reach + a[i] <= budget) { fits[i] = 1; cap[i] = budget - reach - a[i]; }
        reach += b[i];
      }
    }

    // ---- knapsack from the output side: row d uses the d output-most tensors (depth <= d); row d - 1 is what
    //      candidate i* = n - d reads, just before tensor n - d itself enters as row d.  Scanning from the output keeps, among equal values, the mask with the
    //      most leading zeros.
    std::vector<int64_t> row0(W, 0), row1(W, 0);
    std::vector<uint64_t> took((size_t)(n + 1) * WB, 0);   // bit (d, t): row d differs from row d - 1 at t
    int64_t best = 0;  // the empty mask
    int32_t best_first = -1;
    uint64_t best_cap = 0;
    int64_t* prev = row0.data();
    int64_t* cur = row1.data();
    for (int32_t d = 1; d <= n; d++) {
      const int32_t i = n - d;                             // candidate i* = i: its output side is row d - 1 = prev
      if (fits[i]) {
        const int64_t v = iq[i] + prev[cap[i]];
        if (v > best) { best = v; best_first = i; best_cap = cap[i]; }
      }
      const uint64_t w = a[i];
      uint64_t* bits = &took[(size_t)d * WB];
      for (size_t t = 0; t < W; t++) {
        int64_t v = prev[t];
        if (t >= w) {
          const int64_t take = prev[t - w] + iq[i];
          if (take > v) {
            v = take;
            bits[t >> 6] |= (uint64_t)1 << (t & 63);
          }
        }
        cur[t] = v;
      }
      std::swap(prev, cur);
    }
    if (best_first >= 0) {
      mask_out[best_first] = 1;
      uint64_t t = best_cap;
      // walk from the tensor right after i* towards the output; leave a tensor out whenever the
      // value is reachable without it
      for (int32_t i = best_first + 1; i < n; i++) {
        const int32_t d = n - i;
        if ((took[(size_t)d * WB + (t >> 6)] >> (t & 63)) & 1) {
          mask_out[i] = 1;
          t -= a[i];
        }
      }
    }
  } catch (const std::bad_alloc&) {
    for (int32_t i = 0; i < n; i++) mask_out[i] = 0;
    return ET_ENOMEM;
  }
  if (predicted_ns) *predicted_ns = time_model(n, mask_out, t_dw_ns, t_dy_ns, t_fwd_ns);
  return ET_OK;
}

extern "C" int et_select(int32_t n, const double* importance, const uint64_t* t_dw_ns, const uint64_t* t_dy_ns,
                         uint64_t t_fwd_ns, uint32_t rho_ppm, uint32_t tq, uint8_t* mask_out,
                         uint64_t* predicted_ns) {
  return select_core(n, importance, t_dw_ns, t_dy_ns, t_fwd_ns, rho_ppm, tq, mask_out, predicted_ns, nullptr);
}

extern "C" int et_select_stats(int32_t n, const double* importance, const uint64_t* t_dw_ns, const uint64_t* t_dy_ns,
                               uint64_t t_fwd_ns, uint32_t rho_ppm, uint32_t tq, uint8_t* mask_out,
                               uint64_t* predicted_ns, et_select_counts* counts) {
  if (!counts) return ET_EINVAL;
  return select_core(n, importance, t_dw_ns, t_dy_ns, t_fwd_ns, rho_ppm, tq, mask_out, predicted_ns, counts);
}
