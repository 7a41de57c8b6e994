// Host-side paged KV allocator: a pool of fixed-size blocks (16 tokens each,
// all layers) handed to sequences on demand, plus the chunk planner that cuts
// a set of (sequence, position range) spans into forward passes.  Pure C++,
// no GPU calls: unit-tested on the CPU through include/areal_host.h.
#pragma once
#include <stdint.h>

#include <algorithm>
#include <vector>

namespace areal {

class KvAllocator {
 public:
  KvAllocator(int64_t n_blocks, int max_seqs, int max_blocks_per_seq, int block_tokens)
      : n_blocks_(n_blocks), max_blocks_per_seq_(max_blocks_per_seq), block_tokens_(block_tokens),
        seq_blocks_(max_seqs), refcnt_(n_blocks, 0) {
    free_.reserve(n_blocks);
    for (int64_t b = n_blocks - 1; b >= 0; --b) free_.push_back((int32_t)b);   // pop() yields 0,1,2..
  }
  int64_t n_blocks() const { return n_blocks_; }
  int64_t n_free() const { return (int64_t)free_.size(); }
  int blocks_for(int64_t n_tokens) const { return (int)((n_tokens + block_tokens_ - 1) / block_tokens_); }
  const std::vector<int32_t>& blocks(int seq) const { return seq_blocks_[seq]; }

  // Extra blocks sequence `seq` needs to hold n_tokens; -1 if over the per-sequence limit.
  int64_t extra_needed(int seq, int64_t n_tokens) const {
    const int need = blocks_for(n_tokens);
    if (need > max_blocks_per_seq_) return -1;
    return std::max<int64_t>(0, need - (int64_t)seq_blocks_[seq].size());
  }
  // Grow `seq` to n_tokens.  All or nothing: false (and no change) if the pool is short.
  bool reserve(int seq, int64_t n_tokens) {
    const int64_t extra = extra_needed(seq, n_tokens);
    if (extra < 0 || extra > n_free()) return false;
    for (int64_t i = 0; i < extra; ++i) {
      seq_blocks_[seq].push_back(free_.back());
      refcnt_[free_.back()] = 1;
      free_.pop_back();
    }
    return true;
  }
  // Sequence `dst` (which must hold no blocks) starts out with the first n blocks of
  // `src`, shared: a block returns to the pool when its last holder releases it.
  bool share_prefix(int dst, int src, int n) {
    if (dst == src || !seq_blocks_[dst].empty() || n < 0 || n > (int)seq_blocks_[src].size() ||
        n > max_blocks_per_seq_)
      return false;
    for (int i = 0; i < n; ++i) {
      seq_blocks_[dst].push_back(seq_blocks_[src][i]);
      ++refcnt_[seq_blocks_[src][i]];
    }
    return true;
  }
  int refcount(int32_t block) const { return refcnt_[block]; }
  void release(int seq) {
    auto& v = seq_blocks_[seq];
    for (auto it = v.rbegin(); it != v.rend(); ++it)
      if (--refcnt_[*it] == 0) free_.push_back(*it);
    v.clear();
  }
  // Test hook: deterministic shuffle of the free list (placement must not matter).
  void shuffle_free(uint64_t seed) {
    uint64_t s = seed * 6364136223846793005ull + 1442695040888963407ull;
    for (size_t i = free_.size(); i > 1; --i) {
      s = s * 6364136223846793005ull + 1442695040888963407ull;
      std::swap(free_[i - 1], free_[(s >> 33) % i]);
    }
  }

 private:
  int64_t n_blocks_;
  int max_blocks_per_seq_, block_tokens_;
  std::vector<int32_t> free_;
  std::vector<std::vector<int32_t>> seq_blocks_;
  std::vector<int32_t> refcnt_;          // holders per block
};

// A span of one sequence to run through the decoder: positions [pos0, pos0+len).
struct Span {
  int32_t slot, pos0, len;
  int32_t out_index;      // row of the logits output this sequence's last position feeds, or -1
};
// One forward pass: consecutive pieces of spans, at most max_rows rows in total.
struct PassPiece {
  int32_t slot, pos0, len, row0;
  int32_t out_index;      // >= 0 when the piece ends its span (last row produces logits)
};
inline std::vector<std::vector<PassPiece>> plan_passes(const std::vector<Span>& spans, int max_rows) {
  std::vector<std::vector<PassPiece>> passes;
  std::vector<PassPiece> cur;
  int rows = 0;
  for (const Span& s : spans) {
    int done = 0;
    while (done < s.len) {
      if (rows == max_rows) {
        passes.push_back(cur);
        cur.clear();
        rows = 0;
      }
      const int take = std::min(s.len - done, max_rows - rows);
      PassPiece p{s.slot, s.pos0 + done, take, rows, -1};
      done += take;
      if (done == s.len) p.out_index = s.out_index;
      cur.push_back(p);
      rows += take;
    }
  }
  if (!cur.empty()) passes.push_back(cur);
  return passes;
}

}  // namespace areal
