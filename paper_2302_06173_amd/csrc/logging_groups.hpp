// Machine grouping for selective logging (paper, section "Selective Logging"): host code only.
//
// N machines host consecutive pipeline stages.  Logging records the messages between groups of
// machines, not inside a group, and a failure rolls back the failed machine's whole group.  Start
// with one group per machine; while the logging data of one checkpoint interval, T * (bytes per
// iteration on the links between groups), exceeds the limit, merge the adjacent pair with the
// smallest dR/dM:
//   R(G_i, G_{i+1}) = R(G_i) + R(G_{i+1}) + M(G_i, G_{i+1}) / B
//   dR = R(G_i, G_{i+1}) (|G_i| + |G_{i+1}|)/N - R(G_i) |G_i|/N - R(G_{i+1}) |G_{i+1}|/N
//   dM = M(G_i, G_{i+1}) T
// With parallel recovery every R(G) that enters dR is divided by floor(N/|G|).  At most N - 1
// merges, each found by a scan over the remaining pairs: O(N^2), as the paper states.  The
// expressions are evaluated in binary64 in exactly this order (the library is built without
// floating-point contraction), so ties and near-ties resolve the same way everywhere; a tie goes
// to the pair with the lowest index, and a link that carries nothing (dM = 0) is merged only
// when no other link is left.
#pragma once
#include <stdint.h>

#include <cmath>
#include <limits>
#include <vector>

namespace swift {

struct LoggingGroups {
  std::vector<int32_t> group_of;   // group index of every machine, groups numbered in pipeline order
  double storage = 0.0;            // T * bytes per iteration on the links between the final groups
  double recovery = 0.0;           // sum over groups of R(G) |G| / N (R(G) divided as above if parallel)
};

inline LoggingGroups plan_logging_groups(int64_t n, const double *R, const double *M, double T, double B,
                                         double m_max, bool parallel) {
  struct Group {
    double r;          // R(G), undivided
    int64_t size;      // |G|
    double m_next;     // M(G, next group); unused for the last group
  };
  std::vector<Group> g((size_t)n);
  for (int64_t i = 0; i < n; ++i) g[(size_t)i] = Group{R[i], 1, i + 1 < n ? M[i] : 0.0};
  const double N = (double)n;
  auto eff = [&](double r, int64_t size) { return parallel ? r / (double)(n / size) : r; };
  auto storage = [&]() {
    double s = 0.0;
    for (size_t i = 0; i + 1 < g.size(); ++i) s += g[i].m_next;
    return T * s;
  };
  while (g.size() > 1 && storage() > m_max) {
    size_t best = 0;
    double best_ratio = 0.0;
    bool have = false;
    for (size_t i = 0; i + 1 < g.size(); ++i) {
      const int64_t a = g[i].size, b = g[i + 1].size;
      const double merged = g[i].r + g[i + 1].r + g[i].m_next / B;
      const double dR = eff(merged, a + b) * (double)(a + b) / N - eff(g[i].r, a) * (double)a / N -
                        eff(g[i + 1].r, b) * (double)b / N;
      const double dM = g[i].m_next * T;
      const double ratio = dM > 0 ? dR / dM : std::numeric_limits<double>::infinity();
      if (!have || ratio < best_ratio) {
        have = true;
        best = i;
        best_ratio = ratio;
      }
    }
    g[best].r = g[best].r + g[best + 1].r + g[best].m_next / B;
    g[best].size += g[best + 1].size;
    g[best].m_next = g[best + 1].m_next;
    g.erase(g.begin() + (std::ptrdiff_t)best + 1);
  }
  LoggingGroups out;
  out.group_of.resize((size_t)n);
  int64_t machine = 0;
  for (size_t k = 0; k < g.size(); ++k) {
    for (int64_t j = 0; j < g[k].size; ++j) out.group_of[(size_t)machine++] = (int32_t)k;
    out.recovery += eff(g[k].r, g[k].size) * (double)g[k].size / N;
  }
  out.storage = storage();
  return out;
}

}  // namespace swift
