// Channel clustering of the offline prologue (Section 3.1; Algorithm 1 Prologue,
// get_permutation_matrix): the host half of skvq_calibrate_reorder.  Pure host code; the steps
// are the ones listed at skvq_calibrate_reorder in skvq.h.  fp64 throughout, every operation
// rounded once (the file is compiled without contraction).
#include <algorithm>
#include <array>
#include <numeric>
#include <vector>

#include "skvq_internal.h"

namespace skvq {
namespace {

// One channel's feature: the smallest and the largest value seen in calibration.
struct Feature {
  double lo, hi;
  double span() const { return hi - lo; }
};

struct Clustering {
  std::vector<Feature> centre;  // one per cluster
  std::vector<int> owner;       // cluster of every channel, -1 before the first assignment

  // Gives every channel to its nearest centre; says whether any channel changed hands.
  bool assign(const std::array<Feature, kD> &x) {
    bool changed = false;
    for (int ch = 0; ch < kD; ++ch) {
      int nearest = 0;
      double nearest_d2 = 0.0;
      for (size_t j = 0; j < centre.size(); ++j) {
        const double dl = x[ch].lo - centre[j].lo, dh = x[ch].hi - centre[j].hi;
        const double d2 = dl * dl + dh * dh;
        if (j == 0 || d2 < nearest_d2) {  // strict: equal distances go to the lowest cluster
          nearest = (int)j;
          nearest_d2 = d2;
        }
      }
      changed |= owner[ch] != nearest;
      owner[ch] = nearest;
    }
    return changed;
  }

  // Moves every centre to the mean of its channels (one pass of running sums over the channels
  // in index order); a cluster without channels stays where it is.
  void recentre(const std::array<Feature, kD> &x) {
    struct Sum {
      double lo = 0.0, hi = 0.0;
      int n = 0;
    };
    std::vector<Sum> sum(centre.size());
    for (int ch = 0; ch < kD; ++ch) {
      Sum &s = sum[owner[ch]];
      s.lo += x[ch].lo;
      s.hi += x[ch].hi;
      ++s.n;
    }
    for (size_t j = 0; j < centre.size(); ++j)
      if (sum[j].n > 0) centre[j] = Feature{sum[j].lo / sum[j].n, sum[j].hi / sum[j].n};
  }
};

// The multiple of `step` nearest to x (halves go up).
int nearest_multiple(int x, int step) { return (x + step / 2) / step * step; }

void reorder_head(const float *stats, int G, int gran, int max_iter, int32_t *perm, int32_t *bounds) {
  const int n_clusters = kD / G;
  std::array<Feature, kD> x;
  for (int ch = 0; ch < kD; ++ch) x[ch] = Feature{(double)stats[2 * ch], (double)stats[2 * ch + 1]};

  // channels from the narrowest to the widest (equal spans: by index, which a stable sort keeps)
  std::vector<int> by_span(kD);
  std::iota(by_span.begin(), by_span.end(), 0);
  std::stable_sort(by_span.begin(), by_span.end(), [&](int a, int b) { return x[a].span() < x[b].span(); });

  // start: the mean feature of each run of G channels of that list
  Clustering km;
  km.owner.assign(kD, -1);
  for (int j = 0; j < n_clusters; ++j) {
    Feature mean{0.0, 0.0};
    for (auto it = by_span.begin() + j * G; it != by_span.begin() + (j + 1) * G; ++it) {
      mean.lo += x[*it].lo;
      mean.hi += x[*it].hi;
    }
    km.centre.push_back(Feature{mean.lo / G, mean.hi / G});
  }
  // Lloyd: at most max_iter moves of the centres, each followed by a new assignment
  bool changed = km.assign(x);
  for (int moves = 0; changed && moves < max_iter; ++moves) {
    km.recentre(x);
    changed = km.assign(x);
  }

  // clusters from the narrowest centre to the widest; members in by_span order
  std::vector<int> listed(n_clusters);
  std::iota(listed.begin(), listed.end(), 0);
  std::stable_sort(listed.begin(), listed.end(),
                   [&](int a, int b) { return km.centre[a].span() < km.centre[b].span(); });
  std::vector<std::vector<int>> members(n_clusters);
  for (int ch : by_span) members[km.owner[ch]].push_back(ch);
  int32_t *out = perm;
  bounds[0] = 0;
  for (int j = 0; j < n_clusters; ++j) {
    out = std::copy(members[listed[j]].begin(), members[listed[j]].end(), out);
    bounds[j + 1] = (int32_t)(out - perm);
  }
  // inner boundaries to the granularity, left to right; each group keeps `gran` positions and
  // leaves as many to every group after it
  for (int j = 1; j < n_clusters; ++j) {
    const int floor_j = bounds[j - 1] + gran, ceil_j = kD - (n_clusters - j) * gran;
    bounds[j] = std::clamp(nearest_multiple(bounds[j], gran), floor_j, ceil_j);
  }
}

}  // namespace

int reorder_channels(const float *stats, int Hk, int G, int gran, int max_iter, int32_t *perm, int32_t *bounds) {
  const int n_clusters = kD / G;
  for (int h = 0; h < Hk; ++h)
    reorder_head(stats + (size_t)h * kD * 2, G, gran, max_iter, perm + (size_t)h * kD,
                 bounds + (size_t)h * (n_clusters + 1));
  return 0;
}

}  // namespace skvq
