// Minimax layer partition (Sec. 4.2: Eq. 2, Eq. 3, Alg. 1).  Host only.
//
// f[p][l] = best achievable worst-stage mini-step time when the first l layers are spread over the
// first p stages as contiguous non-empty blocks that fit their stages' memory caps;
// f[p][l] = min over k in [p-1, l-1] of max(f[p-1][k], t_p(layers k..l-1)) with Mem(k..l-1) <= cap_p,
// and f[1][l] = t_1(layers 0..l-1) if it fits (the memory constraint is stated for every stage, so
// it is applied to the first stage too).  O(P * L^2) time, O(P * L) memory; boundaries by
// backtracking the arg-min.
#include <cmath>
#include <limits>
#include <new>
#include <vector>

#include "elaswave.h"

extern "C" int ew_partition_layers(uint32_t n_layers, uint32_t n_stages, const double *t, const double *mem,
                                   const double *cap, uint32_t *out_bounds, double *out_cost) {
  const uint32_t L = n_layers, P = n_stages;
  if (L == 0 || P == 0 || P > L || !t || !mem || !cap || !out_cost || (P > 1 && !out_bounds)) return EW_EINVAL;
  if ((uint64_t)P * L * L > (1ull << 31)) return EW_EINVAL;
  const double inf = std::numeric_limits<double>::infinity();
  auto T = [&](uint32_t p, uint32_t a, uint32_t b) { return t[((size_t)p * L + a) * L + b]; };
  auto M = [&](uint32_t a, uint32_t b) { return mem[(size_t)a * L + b]; };
  try {
    // f and the arg-min, indexed [p][l] with p = 1..P stages and l = 0..L layers
    std::vector<double> f((size_t)(P + 1) * (L + 1), inf);
    std::vector<uint32_t> arg((size_t)(P + 1) * (L + 1), 0);
    auto F = [&](uint32_t p, uint32_t l) -> double & { return f[(size_t)p * (L + 1) + l]; };
    for (uint32_t l = 1; l <= L; ++l)
      if (M(0, l - 1) <= cap[0]) F(1, l) = T(0, 0, l - 1);
    for (uint32_t p = 2; p <= P; ++p)
      for (uint32_t l = p; l <= L; ++l) {
        double best = inf;
        uint32_t best_k = 0;
        for (uint32_t k = p - 1; k <= l - 1; ++k) {  // stages 1..p-1 take layers 0..k-1, stage p takes k..l-1
          if (!(M(k, l - 1) <= cap[p - 1])) continue;
          const double left = F(p - 1, k);
          if (left == inf) continue;
          const double here = T(p - 1, k, l - 1);
          const double worst = left > here ? left : here;
          if (worst < best) {
            best = worst;
            best_k = k;
          }
        }
        F(p, l) = best;
        arg[(size_t)p * (L + 1) + l] = best_k;
      }
    if (F(P, L) == inf) return EW_EINFEASIBLE;
    *out_cost = F(P, L);
    uint32_t l = L;
    for (uint32_t p = P; p >= 2; --p) {
      const uint32_t k = arg[(size_t)p * (L + 1) + l];
      out_bounds[p - 2] = k;
      l = k;
    }
  } catch (const std::bad_alloc &) {
    return EW_ENOMEM;
  }
  return EW_OK;
}
