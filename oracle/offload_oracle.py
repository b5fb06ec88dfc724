"""Oracle of the token-level offload tier (Section V-A, Algorithm 2: the GPU-memory -> CPU-memory
store of the tokens that leave the GPU cache, and the CPU-memory -> GPU-memory load of tokens that
are wanted back).  Plain numpy, one pair at a time, no blocking: a store is a list of rows per
(sequence, head) pair, in eviction order.

TEST INFRASTRUCTURE ONLY, like everything under oracle/: imported by the tests, never by the HIP
library or its binding.
"""
from __future__ import annotations

import numpy as np


class HostStore:
    """K, V [b,h,host_cap,d], score, pos [b,h,host_cap], len [b,h]: rows 0..len-1 of a pair are valid."""

    def __init__(self, b: int, h: int, d: int, host_cap: int, dtype=np.float64):
        self.K = np.zeros((b, h, host_cap, d), dtype=dtype)
        self.V = np.zeros((b, h, host_cap, d), dtype=dtype)
        self.score = np.zeros((b, h, host_cap), dtype=np.float64)
        self.pos = np.full((b, h, host_cap), -1, dtype=np.int32)
        self.len = np.zeros((b, h), dtype=np.int32)
        self.host_cap = host_cap


def offload_evicted(K, V, score, pos, kept_idx, kept_cnt, cache_len, store: HostStore):
    """The rows of slots [0, cache_len) that the kept list does not name go to the end of the pair's
    store, in ascending slot order (Algorithm 2: what leaves GPU memory is stored in CPU memory).
    A pair without room is left alone.  Returns the list of pairs that were skipped."""
    b, h = K.shape[:2]
    skipped = []
    for s in range(b):
        m, c = int(cache_len[s]), int(kept_cnt[s])
        for hd in range(h):
            kept = set(int(x) for x in kept_idx[s, hd, :c])
            evicted = [i for i in range(m) if i not in kept]
            L = int(store.len[s, hd])
            if L + len(evicted) > store.host_cap:
                skipped.append((s, hd))
                continue
            for k, i in enumerate(evicted):
                store.K[s, hd, L + k] = K[s, hd, i]
                store.V[s, hd, L + k] = V[s, hd, i]
                store.score[s, hd, L + k] = score[s, hd, i]
                store.pos[s, hd, L + k] = pos[s, hd, i]
            store.len[s, hd] = L + len(evicted)
    return skipped


def reload_tokens(store: HostStore, req_idx, req_cnt, K, V, score, pos, cache_len):
    """Rows req_idx[s, hd, :req_cnt[s]] of the pair's store are appended to its cache (Algorithm 2: what
    is needed again is loaded from CPU memory).  Returns the new lengths; a sequence without room
    keeps its length and nothing of it is written."""
    b, h, cap = K.shape[:3]
    new_len = np.array(cache_len, dtype=np.int32).copy()
    for s in range(b):
        L, r = int(cache_len[s]), int(req_cnt[s])
        if L + r > cap:
            continue
        for hd in range(h):
            for k in range(r):
                j = int(req_idx[s, hd, k])
                assert 0 <= j < store.len[s, hd], "the oracle is only asked for tokens the store holds"
                K[s, hd, L + k] = store.K[s, hd, j]
                V[s, hd, L + k] = store.V[s, hd, j]
                score[s, hd, L + k] = store.score[s, hd, j]
                pos[s, hd, L + k] = store.pos[s, hd, j]
        new_len[s] = L + r
    return new_len
