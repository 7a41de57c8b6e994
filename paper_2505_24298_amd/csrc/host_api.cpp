// Host-only entry points of include/areal_host.h: the paged KV block allocator, the pass
// planner, the staleness gate and dynamic batching behind a C interface.  Plain C++ with no
// GPU call, so that it also builds on its own under the address and undefined-behaviour
// sanitizers (build.py build_host_sanitized) for the CPU tests.
#include <stdint.h>

#include <vector>

#include "../../include/areal.h"
#include "../../include/areal_host.h"
#include "gate.hpp"
#include "kv_alloc.hpp"

using namespace areal;

extern "C" {

struct areal_kvalloc { KvAllocator a; };

areal_kvalloc* areal_kvalloc_create(int64_t n_blocks, int32_t max_seqs, int32_t max_blocks_per_seq) {
  if (n_blocks < 0 || max_seqs <= 0 || max_blocks_per_seq <= 0) return nullptr;
  return new areal_kvalloc{KvAllocator(n_blocks, max_seqs, max_blocks_per_seq, AREAL_KV_BLOCK_TOKENS)};
}
void areal_kvalloc_destroy(areal_kvalloc* a) { delete a; }
int areal_kvalloc_reserve(areal_kvalloc* a, int32_t seq, int64_t n_tokens) { return a->a.reserve(seq, n_tokens) ? 0 : AREAL_E_NOMEM; }
void areal_kvalloc_release(areal_kvalloc* a, int32_t seq) { a->a.release(seq); }
int areal_kvalloc_share(areal_kvalloc* a, int32_t dst, int32_t src, int32_t n_blocks) {
  return a->a.share_prefix(dst, src, n_blocks) ? 0 : AREAL_E_INVAL;
}
int64_t areal_kvalloc_free_blocks(const areal_kvalloc* a) { return a->a.n_free(); }
int32_t areal_kvalloc_table(const areal_kvalloc* a, int32_t seq, int32_t* out, int32_t cap) {
  const auto& b = a->a.blocks(seq);
  for (size_t i = 0; i < b.size() && (int)i < cap; ++i) out[i] = b[i];
  return (int32_t)b.size();
}
void areal_kvalloc_shuffle(areal_kvalloc* a, uint64_t seed) { a->a.shuffle_free(seed); }

struct areal_gate { StalenessGate g; };
areal_gate* areal_gate_create(int64_t batch_size, int64_t eta) {
  if (batch_size < 1 || eta < 0) return nullptr;
  return new areal_gate{StalenessGate(batch_size, eta)};
}
void areal_gate_destroy(areal_gate* g) { delete g; }
int64_t areal_gate_submit(areal_gate* g, int64_t n) { return g ? g->g.submit(n) : 0; }
int64_t areal_gate_budget(const areal_gate* g) { return g ? g->g.budget() : 0; }
int areal_gate_set_version(areal_gate* g, int64_t version) {
  if (!g) return AREAL_E_INVAL;
  return g->g.set_version(version) ? AREAL_OK : AREAL_E_STATE;
}
int64_t areal_gate_submitted(const areal_gate* g) { return g ? g->g.submitted() : 0; }

int32_t areal_dynamic_batching(int32_t n, const int32_t* lens, int64_t capacity, int32_t k_min,
                               int32_t* batch_of) {
  if (n < 0 || capacity < 1 || k_min < 1 || (n > 0 && (!lens || !batch_of))) return AREAL_E_INVAL;
  for (int i = 0; i < n; ++i)
    if (lens[i] < 1) return AREAL_E_INVAL;
  return dynamic_batching(lens, n, capacity, k_min, batch_of);
}

int32_t areal_plan_passes(int32_t n_spans, const int32_t* lens, int32_t max_rows, int32_t* out, int32_t cap) {
  std::vector<Span> spans;
  for (int i = 0; i < n_spans; ++i) spans.push_back(Span{i, 0, lens[i], i});
  auto passes = plan_passes(spans, max_rows);
  int n = 0;
  for (size_t p = 0; p < passes.size(); ++p)
    for (auto& pc : passes[p]) {
      if (n < cap) {
        int32_t* o = out + (int64_t)n * 6;
        o[0] = (int32_t)p; o[1] = pc.slot; o[2] = pc.pos0; o[3] = pc.len; o[4] = pc.row0; o[5] = pc.out_index;
      }
      ++n;
    }
  return n;
}

}  // extern "C"
