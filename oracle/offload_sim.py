"""CPU oracle for the expert-cache (offloading) simulation: TEST INFRASTRUCTURE.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this file.
It shares no code with the library.

The paper motivates chunk-level sparsity and a high reuse ratio with offloading: expert weights
are brought into fast memory only when activated, so similar expert sets on consecutive tokens
save expert IO (Sec. 1, Sec. 4.1.2).  It gives no mechanism; the reading taken here is the
textbook one: a cache of ``capacity`` experts with least-recently-used replacement, driven by the
stream of union lists of one layer.  The experts of a chunk are touched one after the other in
the order of its list (ascending expert index); a touch of a resident expert is a hit and makes
it the most recently used; a touch of a non-resident expert is a load, which first evicts the
least recently used resident expert when the cache is full.  The cache starts empty.
"""

from __future__ import annotations

from collections import OrderedDict

import numpy as np


def lru_offload(active_idx: np.ndarray, n_active: np.ndarray, capacity: int):
    """Returns (loads_per_chunk int64 [n_chunks], totals int64 [3] = touches, loads, evictions)."""
    cache: "OrderedDict[int, None]" = OrderedDict()
    loads = np.zeros(len(n_active), dtype=np.int64)
    touches = evictions = 0
    for c in range(len(n_active)):
        for s in range(int(n_active[c])):
            e = int(active_idx[c, s])
            touches += 1
            if e in cache:
                cache.move_to_end(e)
                continue
            loads[c] += 1
            if capacity == 0:
                continue            # nothing can stay resident
            if len(cache) >= capacity:
                cache.popitem(last=False)
                evictions += 1
            cache[e] = None
    return loads, np.array([touches, loads.sum(), evictions], dtype=np.int64)
