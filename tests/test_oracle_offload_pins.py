"""Pins of the offload-tier oracle (Section V-A, Algorithm 2, store and load of Phase II) against
what the bookkeeping must satisfy whatever the implementation: no token is ever lost or duplicated
between the cache and the store, stored rows are bit-exact copies, a load followed by a decode step
attends over exactly the union.  CPU only."""
import numpy as np
from scipy.special import softmax

from oracle import offload_oracle as OF


def _state(rng, b, h, cap, d, lens):
    K = np.zeros((b, h, cap, d))
    V = np.zeros((b, h, cap, d))
    pos = np.full((b, h, cap), -1, dtype=np.int32)
    for s, L in enumerate(lens):
        K[s, :, :L] = rng.standard_normal((h, L, d))
        V[s, :, :L] = rng.standard_normal((h, L, d))
        pos[s, :, :L] = np.arange(L)
    return K, V, pos, np.array(lens, dtype=np.int32)


def test_no_token_is_lost_or_duplicated_over_a_trajectory(oracle):
    O = oracle
    rng = np.random.default_rng(5)
    b, h, cap, d, w, sp = 2, 3, 64, 4, 3, 7000
    K, V, pos, lens = _state(rng, b, h, cap, d, [30, 11])
    K0, V0 = K.copy(), V.copy()
    score = np.zeros((b, h, cap))
    store = OF.HostStore(b, h, d, 64)
    n = lens.copy()
    cl = lens.copy()
    new_rows = {}
    score_at = {}
    for t in range(12):
        n = n + 1
        q, kn, vn = (rng.standard_normal((b, h, d)) for _ in range(3))
        for s in range(b):
            new_rows[(s, int(n[s]) - 1)] = (kn[s].copy(), vn[s].copy())
        kept, cnt, out, p = O.decode_step(q, kn, vn, K, V, score, pos, cl, n, w, sp, 0.5)
        before = store.len.copy()
        # the importance every token has right now, by position: what a token evicted now must carry
        for s in range(b):
            for hd in range(h):
                for i in range(int(cl[s])):
                    score_at[(s, hd, int(pos[s, hd, i]))] = score[s, hd, i]
        assert OF.offload_evicted(K, V, score, pos, kept, cnt, cl, store) == []
        for s in range(b):
            for hd in range(h):
                for j in range(int(before[s, hd]), int(store.len[s, hd])):
                    assert store.score[s, hd, j] == score_at[(s, hd, int(store.pos[s, hd, j]))] > 0
        for s in range(b):
            assert np.all(store.len[s] - before[s] == cl[s] - cnt[s])          # exactly the evicted tokens
        O.compact(K, V, score, pos, kept, cnt, cl)
        for s in range(b):
            for hd in range(h):
                cached = pos[s, hd, :cl[s]].tolist()
                stored = store.pos[s, hd, :store.len[s, hd]].tolist()
                assert sorted(cached + stored) == list(range(int(n[s])))      # a partition of all tokens
                for j, tpos in enumerate(stored):                             # stored rows are exact copies
                    ref_k = K0[s, hd, tpos] if tpos < lens[s] else new_rows[(s, tpos)][0][hd]
                    ref_v = V0[s, hd, tpos] if tpos < lens[s] else new_rows[(s, tpos)][1][hd]
                    assert np.array_equal(store.K[s, hd, j], ref_k) and np.array_equal(store.V[s, hd, j], ref_v)
    # the importance stored with a token is the value it had when it was evicted: never above the
    # smallest kept one at that time is not guaranteed later, but it is positive and finite
    assert np.all(np.isfinite(store.score)) and np.all(store.score >= 0)


def test_the_newest_token_is_offloaded_too_when_it_loses(oracle):
    # no local window (w = 0): the token of the current step is a candidate like any other, has the
    # smallest importance (one attention weight against the others' sums) and is evicted at once
    O = oracle
    rng = np.random.default_rng(8)
    b, h, cap, d = 1, 2, 16, 4
    K, V, pos, lens = _state(rng, b, h, cap, d, [8])
    score = np.full((b, h, cap), 5.0)
    store = OF.HostStore(b, h, d, 8)
    cl, n = lens.copy(), lens + 1
    q, kn, vn = (rng.standard_normal((b, h, d)) for _ in range(3))
    kept, cnt, out, p = O.decode_step(q, kn, vn, K, V, score, pos, cl, n, 0, 2000, 0.5)   # keeps 7 of 9
    assert cnt[0] == 7 and cl[0] == 9
    OF.offload_evicted(K, V, score, pos, kept, cnt, cl, store)
    for hd in range(h):
        assert store.len[0, hd] == 2 and 8 in store.pos[0, hd, :2].tolist()        # position 8 = the new token
        j = store.pos[0, hd, :2].tolist().index(8)
        assert np.array_equal(store.K[0, hd, j], kn[0, hd]) and np.array_equal(store.V[0, hd, j], vn[0, hd])
        assert store.pos[0, hd, 0] < store.pos[0, hd, 1]                           # ascending slot order


def test_a_full_store_skips_the_pair_and_writes_nothing(oracle):
    O = oracle
    rng = np.random.default_rng(6)
    K, V, pos, lens = _state(rng, 1, 2, 32, 4, [20])
    score = rng.random((1, 2, 32))
    store = OF.HostStore(1, 2, 4, 5)                       # room for 5 tokens per pair
    cl = lens.copy()
    kept, cnt = O.select(score, cl, cl, 2, 5000)           # keeps 10 of 20: 10 evicted > 5
    assert OF.offload_evicted(K, V, score, pos, kept, cnt, cl, store) == [(0, 0), (0, 1)]
    assert np.all(store.len == 0) and np.all(store.pos == -1)


def test_loading_everything_back_restores_dense_attention(oracle):
    # evict, store, load every stored token back: attention over the cache (as a set) is again the
    # dense attention of Eq. 1-2 over all tokens
    O = oracle
    rng = np.random.default_rng(7)
    b, h, cap, d = 1, 2, 48, 5
    K, V, pos, lens = _state(rng, b, h, cap, d, [24])
    Kall, Vall = K.copy(), V.copy()
    score = np.zeros((b, h, cap))
    cl, n = lens.copy(), lens + 1
    q, kn, vn = (rng.standard_normal((b, h, d)) for _ in range(3))
    kept, cnt, out, p = O.decode_step(q, kn, vn, K, V, score, pos, cl, n, 2, 6000, 0.5)
    Kall[:, :, 24], Vall[:, :, 24] = kn, vn
    store = OF.HostStore(b, h, d, 32)
    OF.offload_evicted(K, V, score, pos, kept, cnt, cl, store)
    O.compact(K, V, score, pos, kept, cnt, cl)
    r = int(store.len[0, 0])
    req = np.tile(np.arange(r, dtype=np.int32), (b, h, 1))
    new_len = OF.reload_tokens(store, req, np.array([r], dtype=np.int32), K, V, score, pos, cl)
    assert new_len[0] == 25
    q2 = rng.standard_normal((b, h, d))
    for hd in range(h):
        L = new_len[0]
        z = K[0, hd, :L] @ q2[0, hd] * 0.5
        got = softmax(z) @ V[0, hd, :L]
        ref = softmax(Kall[0, hd, :25] @ q2[0, hd] * 0.5) @ Vall[0, hd, :25]
        np.testing.assert_allclose(got, ref, rtol=1e-12)
        assert sorted(pos[0, hd, :L].tolist()) == list(range(25))
    # no room: the sequence keeps its length
    assert OF.reload_tokens(store, req, np.array([40], dtype=np.int32), K, V, score, pos, new_len)[0] == 25
