// Expert-cache simulation for offloading (the paper's second motivation for chunk-level sparsity
// and expert selection stability, Sec. 1 and Sec. 4.1.2): how many expert loads a cache of
// `capacity` experts with least-recently-used replacement needs for a stream of union lists.
// Host code only: it reads the lists from host memory and launches nothing.
//
// With at most 256 experts the cache is two small arrays: a residency flag and the time of the
// last touch per expert; the victim of an eviction is the resident expert with the oldest touch.
#include "common.hpp"

namespace blockffn {

int offload_sim(const int32_t *active_idx, const int32_t *n_active, int64_t n_chunks, int E, int capacity,
                int64_t *loads_per_chunk, int64_t *totals) {
  bool resident[kMaxExperts] = {};
  int64_t last_touch[kMaxExperts] = {};
  int n_resident = 0;
  int64_t clock = 0, touches = 0, loads = 0, evictions = 0;
  for (int64_t c = 0; c < n_chunks; ++c) {
    const int n = n_active[c];
    if (n < 0 || n > E) return BLOCKFFN_ERR_INVALID;
    int64_t chunk_loads = 0;
    for (int s = 0; s < n; ++s) {
      const int e = active_idx[c * E + s];
      if (e < 0 || e >= E) return BLOCKFFN_ERR_INVALID;
      ++touches;
      ++clock;
      if (resident[e]) {
        last_touch[e] = clock;
        continue;
      }
      ++chunk_loads;
      if (capacity == 0) continue;
      if (n_resident >= capacity) {
        int victim = -1;
        for (int i = 0; i < E; ++i)
          if (resident[i] && (victim < 0 || last_touch[i] < last_touch[victim])) victim = i;
        resident[victim] = false;
        --n_resident;
        ++evictions;
      }
      resident[e] = true;
      last_touch[e] = clock;
      ++n_resident;
    }
    loads += chunk_loads;
    if (loads_per_chunk) loads_per_chunk[c] = chunk_loads;
  }
  totals[0] = touches;
  totals[1] = loads;
  totals[2] = evictions;
  return BLOCKFFN_OK;
}

}  // namespace blockffn
