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
// With parallel recovery every R(G) that enters dR is divided by floor(N/|G|).  A tie goes to the pair
// with the lowest index, and a link that carries nothing (dM = 0) is merged only when no other link
// is left.  The expressions are evaluated in binary64 in exactly this order (the library is built
// without floating-point contraction), so ties and near-ties resolve the same way everywhere.
//
// How: a merge changes the ratios of at most two pairs, the merged group with its left and with its
// right neighbour.  So the groups form a doubly linked list over the index of their first machine and
// the candidate pairs sit in a priority queue ordered by (ratio, position); entries that a later
// merge has outdated carry an old version number and are skipped when they surface.  Selection costs
// O(log N) per merge instead of the scan over all pairs that the paper's O(N^2) bound describes.  The
// storage that the loop tests and the call reports is the plain in-order sum over the live links, the
// same number, bit for bit, whichever way the grouping was reached; a running sum stands in for it
// in the loop test wherever the two cannot disagree about the limit.
#pragma once
#include <stdint.h>

#include <cmath>
#include <limits>
#include <queue>
#include <vector>

namespace swift {

struct LoggingGroups {
  std::vector<int32_t> group_of;   // group index of every machine, groups numbered in pipeline order
  double storage = 0.0;            // T * bytes per iteration on the links between the final groups
  double recovery = 0.0;           // sum over groups of R(G) |G| / N (R(G) divided as above if parallel)
};

inline LoggingGroups plan_logging_groups(int64_t n, const double *R, const double *M, double T, double B,
                                         double m_max, bool parallel) {
  // A group is named by its first machine (its head).  Entries of machines that are not heads are dead.
  const int64_t kEnd = n;
  std::vector<double> r((size_t)n), link((size_t)n, 0.0);      // R(G) undivided; M(G, next group)
  std::vector<int64_t> size((size_t)n, 1), next((size_t)n), prev((size_t)n);
  std::vector<uint32_t> version((size_t)n, 0);                 // of the pair (head, next head)
  for (int64_t i = 0; i < n; ++i) {
    r[(size_t)i] = R[i];
    next[(size_t)i] = i + 1;                                   // kEnd behind the last group
    prev[(size_t)i] = i - 1;                                   // -1 in front of the first
    if (i + 1 < n) link[(size_t)i] = M[i];
  }
  const double N = (double)n;
  auto eff = [&](double rr, int64_t sz) { return parallel ? rr / (double)(n / sz) : rr; };
  auto ratio_of = [&](int64_t i) {                             // pair (group i, the group after it)
    const int64_t j = next[(size_t)i];
    const int64_t a = size[(size_t)i], b = size[(size_t)j];
    const double merged = r[(size_t)i] + r[(size_t)j] + link[(size_t)i] / B;
    const double dR = eff(merged, a + b) * (double)(a + b) / N - eff(r[(size_t)i], a) * (double)a / N -
                      eff(r[(size_t)j], b) * (double)b / N;
    const double dM = link[(size_t)i] * T;
    return dM > 0 ? dR / dM : std::numeric_limits<double>::infinity();
  };
  struct Candidate {
    double ratio;
    int64_t left;          // head of the left group: pairs are ordered like their left heads
    uint32_t version;
  };
  struct Later {           // priority_queue keeps the LARGEST on top: "a comes later than b"
    bool operator()(const Candidate &a, const Candidate &b) const {
      if (a.ratio != b.ratio) return a.ratio > b.ratio;
      return a.left > b.left;
    }
  };
  std::priority_queue<Candidate, std::vector<Candidate>, Later> queue;
  auto offer = [&](int64_t i) {
    if (i < 0 || next[(size_t)i] == kEnd) return;
    queue.push(Candidate{ratio_of(i), i, ++version[(size_t)i]});
  };
  for (int64_t i = 0; i + 1 < n; ++i) offer(i);
  int64_t n_groups = n;
  auto storage = [&]() {
    double sum = 0.0;
    for (int64_t i = 0; next[(size_t)i] != kEnd; i = next[(size_t)i]) sum += link[(size_t)i];
    return T * sum;
  };
  // The loop test is T * (in-order sum of the live links) > limit.  A running sum (one subtraction per merge)
  // answers it whenever it is further from the limit than its own worst-case rounding error; only then is
  // the in-order sum formed again, so the decisions are those of the in-order sum at O(1) per merge.
  double running = storage() / T;
  const double sum0 = running;
  double ops = (double)n;                                      // additions and subtractions behind `running`
  auto over_limit = [&]() {
    const double slack = T * (4.0 * ops * 2.220446049250313e-16 * sum0) + 8.0 * 2.220446049250313e-16 * std::fabs(m_max);
    const double s = T * running;
    if (std::fabs(s - m_max) > slack) return s > m_max;        // (also the answer for an infinite limit)
    return storage() > m_max;
  };
  while (n_groups > 1 && over_limit()) {
    // every live pair has one entry of its current version in the queue, so a current one surfaces
    Candidate c = queue.top();
    queue.pop();
    while (size[(size_t)c.left] == 0 || next[(size_t)c.left] == kEnd || c.version != version[(size_t)c.left]) {
      c = queue.top();
      queue.pop();
    }
    const int64_t i = c.left, j = next[(size_t)i];
    r[(size_t)i] = r[(size_t)i] + r[(size_t)j] + link[(size_t)i] / B;
    running -= link[(size_t)i];
    ops += 1.0;
    size[(size_t)i] += size[(size_t)j];
    link[(size_t)i] = link[(size_t)j];
    next[(size_t)i] = next[(size_t)j];
    if (next[(size_t)j] != kEnd) prev[(size_t)next[(size_t)j]] = i;
    size[(size_t)j] = 0;                                       // j is no head any more
    --n_groups;
    offer(prev[(size_t)i]);                                    // the two pairs whose ratio has changed
    offer(i);
  }
  LoggingGroups out;
  out.group_of.resize((size_t)n);
  int32_t k = 0;
  for (int64_t i = 0; i != kEnd; i = next[(size_t)i], ++k) {
    for (int64_t m = i; m < i + size[(size_t)i]; ++m) out.group_of[(size_t)m] = k;
    out.recovery += eff(r[(size_t)i], size[(size_t)i]) * (double)size[(size_t)i] / N;
  }
  out.storage = storage();
  return out;
}

}  // namespace swift
