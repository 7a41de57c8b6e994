// Staleness gate of the rollout controller (host only).
//
// A generation request may be submitted, as the N-th since the start, only if
// floor((N - 1) / B) <= i + eta  (B = training batch size, i = current policy
// version, eta = maximum staleness of a training batch).  Since the left side
// grows with N, the requests admissible at version i are exactly those with
// N <= (i + eta + 1) * B: the gate keeps that bound as a budget instead of
// testing requests one by one.
#pragma once
#include <stdint.h>
#include <algorithm>
#include <vector>

namespace areal {

class StalenessGate {
 public:
  StalenessGate(int64_t batch_size, int64_t eta) : B_(batch_size), eta_(eta) {}
  // how many more requests may be submitted at the current version
  int64_t budget() const {
    // (i + eta + 1) * B can exceed int64 only for absurd arguments: saturate
    const __int128 lim = ((__int128)version_ + eta_ + 1) * B_;
    const __int128 left = lim - submitted_;
    if (left <= 0) return 0;
    return left > INT64_MAX ? INT64_MAX : (int64_t)left;
  }
  // submit up to n requests; returns how many were admitted
  int64_t submit(int64_t n) {
    const int64_t k = std::max<int64_t>(0, std::min(n, budget()));
    submitted_ += k;
    return k;
  }
  bool set_version(int64_t v) {
    if (v < version_) return false;
    version_ = v;
    return true;
  }
  int64_t submitted() const { return submitted_; }
  int64_t version() const { return version_; }

 private:
  int64_t B_, eta_;
  int64_t version_ = 0, submitted_ = 0;
};

// Dynamic batching: sequences longest first; a sequence opens a new micro-batch while
// fewer than k_min exist or when none has room (total length <= capacity), otherwise it
// joins, among those with room, the one holding the fewest sequences (first created on a
// tie).  Equal lengths keep their input order.  batch_of[i] = micro-batch of sequence i;
// returns the number of micro-batches.
inline int dynamic_batching(const int32_t* lens, int n, int64_t capacity, int k_min, int32_t* batch_of) {
  std::vector<int> order(n);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return lens[a] > lens[b]; });
  std::vector<int64_t> total;
  std::vector<int> count;
  for (int i : order) {
    int best = -1;
    if ((int)total.size() >= k_min)
      for (int b = 0; b < (int)total.size(); ++b)
        if (total[b] + lens[i] <= capacity && (best < 0 || count[b] < count[best])) best = b;
    if (best < 0) {
      best = (int)total.size();
      total.push_back(0);
      count.push_back(0);
    }
    total[best] += lens[i];
    ++count[best];
    batch_of[i] = best;
  }
  return (int)total.size();
}

}  // namespace areal
