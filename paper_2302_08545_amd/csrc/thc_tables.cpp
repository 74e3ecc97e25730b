// Host-only part of libthc: the truncation threshold t_p and the lookup-table tools (Sec. 5.2, App. B).
#include "thc.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

namespace {

// standard normal density and distribution function
double npdf(double a) { return std::exp(-0.5 * a * a) / std::sqrt(2.0 * M_PI); }
double ncdf(double a) { return 0.5 * std::erfc(-a / std::sqrt(2.0)); }

}  // namespace

extern "C" {

double thc_threshold(double p) {
  if (!(p > 0.0 && p < 1.0)) return NAN;
  // solve ncdf(t) = 1 - p/2 for t >= 0, i.e. erfc(t / sqrt 2) = p: bisection, then Newton polish
  double lo = 0.0, hi = 40.0;
  for (int it = 0; it < 200; ++it) {
    const double mid = 0.5 * (lo + hi);
    if (std::erfc(mid / std::sqrt(2.0)) > p) lo = mid; else hi = mid;
  }
  double t = 0.5 * (lo + hi);
  for (int it = 0; it < 3; ++it) {
    const double f = std::erfc(t / std::sqrt(2.0)) - p;   // decreasing in t, derivative -2 pdf(t)
    t += f / (2.0 * npdf(t));
  }
  return t;
}

int thc_solve_table(uint32_t b, uint32_t g, double p, uint8_t* table_out, double* cost_out) {
  if (!table_out || b < 1 || b > 8 || g > 255 || g < (1u << b) - 1 || !(p > 0.0 && p < 1.0)) return THC_EINVAL;
  const int L = (1 << b) - 1;   // edges of the path 0 -> g
  const int G = (int)g;
  const double tp = thc_threshold(p);
  // Expected squared error of stochastic rounding between neighbours q0 < q1 of a standard normal:
  // integral of (a - q0)(q1 - a) pdf(a) da, through the moments int pdf, int a pdf, int a^2 pdf.
  std::vector<double> q(G + 1), Phi(G + 1), phi(G + 1);
  for (int v = 0; v <= G; ++v) {
    q[v] = -tp + v * (2.0 * tp / G);
    Phi[v] = ncdf(q[v]);
    phi[v] = npdf(q[v]);
  }
  auto edge = [&](int i, int j) {
    const double m0 = Phi[j] - Phi[i];
    const double m1 = -(phi[j] - phi[i]);
    const double m2 = m0 - (q[j] * phi[j] - q[i] * phi[i]);
    return -m2 + (q[i] + q[j]) * m1 - q[i] * q[j] * m0;
  };
  const double INF = HUGE_VAL;
  std::vector<std::vector<double>> best(L + 1, std::vector<double>(G + 1, INF));   // best[e][v]: v -> g in e edges
  best[0][G] = 0.0;
  for (int e = 1; e <= L; ++e)
    for (int v = 0; v <= G; ++v)
      for (int u = v + 1; u <= G; ++u)
        if (best[e - 1][u] < INF) {
          const double c = edge(v, u) + best[e - 1][u];
          if (c < best[e][v]) best[e][v] = c;
        }
  const double opt = best[L][0];
  if (!(opt < INF)) return THC_EINVAL;
  const double tol = std::fabs(opt) * 1e-12;
  int v = 0;
  double spent = 0.0;
  table_out[0] = 0;
  for (int e = L; e >= 1; --e) {
    int pick = -1;
    for (int u = v + 1; u <= G && pick < 0; ++u)
      if (best[e - 1][u] < INF && spent + edge(v, u) + best[e - 1][u] <= opt + tol) pick = u;
    if (pick < 0) return THC_EINVAL;
    spent += edge(v, pick);
    v = pick;
    table_out[L - e + 1] = (uint8_t)v;
  }
  if (cost_out) *cost_out = opt;
  return THC_OK;
}

int thc_solve_table_bruteforce(uint32_t b, uint32_t g, double p, uint8_t* table_out, double* cost_out,
                               uint64_t* count_out) {
  if (!table_out || b < 1 || b > 8 || g > 255 || g < (1u << b) - 1 || !(p > 0.0 && p < 1.0)) return THC_EINVAL;
  const int k = (1 << b) - 1;              // bins = gaps between consecutive table values, each >= 1
  const int balls = (int)g - k;            // spare units beyond the k unit gaps
  // C(balls + k - 1, k - 1) = C(g - 1, k - 1) candidates; refuse searches that would not end in reasonable time
  long double cnt = 1.0L;
  for (int i = 1; i <= k - 1; ++i) cnt = cnt * (balls + i) / i;
  if (cnt > 4.0e9L) return THC_EUNSUPPORTED;
  const double tp = thc_threshold(p);
  const int G = (int)g;
  std::vector<double> q(G + 1), Phi(G + 1), phi(G + 1);
  for (int v = 0; v <= G; ++v) {
    q[v] = -tp + v * (2.0 * tp / G);
    Phi[v] = ncdf(q[v]);
    phi[v] = npdf(q[v]);
  }
  std::vector<double> edge((size_t)(G + 1) * (G + 1), 0.0);
  for (int i = 0; i <= G; ++i)
    for (int j = i + 1; j <= G; ++j) {
      const double m0 = Phi[j] - Phi[i], m1 = -(phi[j] - phi[i]), m2 = m0 - (q[j] * phi[j] - q[i] * phi[i]);
      edge[(size_t)i * (G + 1) + j] = -m2 + (q[i] + q[j]) * m1 - q[i] * q[j] * m0;
    }
  // A strictly increasing table from 0 to g is a choice of its k - 1 interior values out of 1 .. g-1.  The choices are
  // walked in lexicographic order (the next combination: bump the rightmost value that still has room, reset what
  // follows it to the smallest values allowed), carrying the cost of the unchanged prefix along.  Only completeness
  // matters to an exhaustive search; the count C(g-1, k-1) is returned for the caller to check.
  const int m = k - 1;                                   // interior values cur[1 .. m]; cur[0] = 0, cur[k] = g
  std::vector<int> best(k + 1, 0), cur(k + 1, 0);
  std::vector<double> prefix(k + 1, 0.0);                // prefix[i] = cost of the pairs (cur[0],cur[1]) .. (cur[i-1],cur[i])
  cur[k] = G;
  for (int i = 1; i <= m; ++i) cur[i] = i;
  double best_cost = HUGE_VAL;
  uint64_t visited = 0;
  int from = 1;                                          // first position whose prefix cost has to be refreshed
  for (;;) {
    for (int i = from; i <= k; ++i) prefix[i] = prefix[i - 1] + edge[(size_t)cur[i - 1] * (G + 1) + cur[i]];
    const double c = prefix[k];
    ++visited;
    bool take = visited == 1;
    if (!take) {
      const double tol = std::fabs(best_cost) * 1e-12;
      take = c < best_cost - tol;
      if (!take && std::fabs(c - best_cost) <= tol)
        take = std::lexicographical_compare(cur.begin(), cur.end(), best.begin(), best.end());
    }
    if (take) { best = cur; best_cost = c; }
    int i = m;
    while (i >= 1 && cur[i] == G - 1 - (m - i)) --i;     // position i can grow while the values after it still fit
    if (i < 1) break;
    ++cur[i];
    for (int j = i + 1; j <= m; ++j) cur[j] = cur[j - 1] + 1;
    from = i;
  }
  for (int i = 0; i <= k; ++i) table_out[i] = (uint8_t)best[i];
  if (cost_out) *cost_out = best_cost;
  if (count_out) *count_out = visited;
  return THC_OK;
}

}  // extern "C"
