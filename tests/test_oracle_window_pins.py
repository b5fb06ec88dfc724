"""Pins of the oracle's strict local attention sum (Algorithm 1 line 2 taken literally: the sum of
the R most recent attention-weight rows) against library routines, the already pinned running-sum
path, exact special cases and an independent per-token bookkeeping.  CPU only."""
import numpy as np
from scipy.special import softmax


def _state(rng, b, h, cap, d, lens):
    K = np.zeros((b, h, cap, d))
    V = np.zeros((b, h, cap, d))
    pos = np.full((b, h, cap), -1, dtype=np.int32)
    for s, L in enumerate(lens):
        K[s, :, :L] = rng.standard_normal((h, L, d))
        V[s, :, :L] = rng.standard_normal((h, L, d))
        pos[s, :, :L] = np.arange(L)
    return K, V, pos, np.array(lens, dtype=np.int32)


def test_prefill_rows_are_the_last_rows_of_the_causal_softmax(oracle):
    O = oracle
    rng = np.random.default_rng(11)
    b, h, cap, d, R = 2, 3, 20, 5, 4
    K, V, pos, lens = _state(rng, b, h, cap, d, [13, 3])          # second prompt shorter than R
    q_tail = rng.standard_normal((b, h, R, d))
    ring = O.prefill_rows(q_tail, K, lens, 0.4)
    for s in range(b):
        L = lens[s]
        for hd in range(h):
            for r in range(R):
                t = L - R + r
                if t < 0:
                    assert np.all(ring[s, hd, r] == 0)
                    continue
                ref = softmax(K[s, hd, :t + 1] @ q_tail[s, hd, r] * 0.4)
                np.testing.assert_allclose(ring[s, hd, r, :t + 1], ref, rtol=1e-12)
                assert np.all(ring[s, hd, r, t + 1:] == 0)
    # their sum is the importance seed of the running-sum path
    np.testing.assert_allclose(ring.sum(axis=2), O.prefill_scores(q_tail, K, lens, 0.4), rtol=1e-12, atol=1e-15)


def _run(O, rng, window_R, steps, sparsity_bp, w, seed_rows, ring_rows):
    """Runs the running-sum path and the window path side by side from the same prompt."""
    b, h, cap, d = 2, 2, 48, 6
    K, V, pos, lens = _state(rng, b, h, cap, d, [17, 9])
    q_tail = rng.standard_normal((b, h, seed_rows, d))
    A = dict(K=K.copy(), V=V.copy(), pos=pos.copy(), len=lens.copy(), score=O.prefill_scores(q_tail, K, lens, 0.5))
    Bw = dict(K=K.copy(), V=V.copy(), pos=pos.copy(), len=lens.copy(), score=np.zeros((b, h, cap)))
    ring = np.zeros((b, h, ring_rows, cap))
    ring[:, :, :seed_rows] = O.prefill_rows(q_tail, K, lens, 0.5)
    n = lens.copy()
    hist = []
    for t in range(steps):
        n = n + 1
        q = rng.standard_normal((b, h, d))
        kn, vn = rng.standard_normal((b, h, d)), rng.standard_normal((b, h, d))
        ra = O.decode_step(q, kn, vn, A["K"], A["V"], A["score"], A["pos"], A["len"], n, w, sparsity_bp, 0.5)
        row = (seed_rows + t) % ring_rows
        rb = O.decode_step_window(q, kn, vn, Bw["K"], Bw["V"], ring, row, Bw["score"], Bw["pos"], Bw["len"], n,
                                  w, sparsity_bp, 0.5)
        hist.append((ra, rb, {k: v.copy() for k, v in A.items()}, {k: v.copy() for k, v in Bw.items()}, ring.copy()))
        O.compact(A["K"], A["V"], A["score"], A["pos"], ra[0], ra[1], A["len"])
        O.compact_ring(ring, rb[0], rb[1])
        O.compact(Bw["K"], Bw["V"], Bw["score"], Bw["pos"], rb[0], rb[1], Bw["len"])
    return hist


def test_a_window_that_holds_every_row_is_the_running_sum(oracle):
    O = oracle
    rng = np.random.default_rng(12)
    steps, seed_rows = 9, 3
    hist = _run(O, rng, None, steps, 6000, 2, seed_rows, seed_rows + steps)
    evicted = 0
    for (ra, rb, A, Bw, ring) in hist:
        assert np.array_equal(ra[0], rb[0]) and np.array_equal(ra[1], rb[1])        # same kept sets
        np.testing.assert_allclose(rb[2], ra[2], rtol=1e-12, atol=1e-14)             # same outputs
        for s, m in enumerate(A["len"]):
            np.testing.assert_allclose(Bw["score"][s, :, :m], A["score"][s, :, :m], rtol=1e-12, atol=1e-14)
            evicted += m - ra[1][s]
    assert evicted > 0


def test_a_one_row_window_is_the_current_attention_row(oracle):
    O = oracle
    rng = np.random.default_rng(13)
    hist = _run(O, rng, None, 5, 5000, 1, 1, 1)
    for (ra, rb, A, Bw, ring) in hist:
        for s, m in enumerate(Bw["len"]):
            assert np.array_equal(Bw["score"][s, :, :m], rb[3][s, :, :m])
            assert np.array_equal(ring[s, :, 0, :m], rb[3][s, :, :m])


def test_window_sum_matches_per_token_bookkeeping(oracle):
    """Independent statement: remember, per step, the weight every token POSITION received; the
    importance of a cached token is the sum over the last R steps (prompt rows included)."""
    O = oracle
    rng = np.random.default_rng(14)
    b, h, cap, d, R, steps = 1, 2, 40, 4, 3, 10
    K, V, pos, lens = _state(rng, b, h, cap, d, [12])
    q_tail = rng.standard_normal((b, h, R, d))
    ring = O.prefill_rows(q_tail, K, lens, 0.7)
    rows = [[{int(p): ring[0, hd, r, p] for p in range(lens[0])} for r in range(R)] for hd in range(h)]
    score = np.zeros((b, h, cap))
    n = lens.copy()
    dropped = False
    for t in range(steps):
        n = n + 1
        q, kn, vn = (rng.standard_normal((b, h, d)) for _ in range(3))
        kept, cnt, out, p = O.decode_step_window(q, kn, vn, K, V, ring, t % R, score, pos, lens, n, 2, 5000, 0.7)
        m = lens[0]
        for hd in range(h):
            rows[hd].append({int(pos[0, hd, i]): p[0, hd, i] for i in range(m)})
            last = rows[hd][-R:]
            for i in range(m):
                tok = int(pos[0, hd, i])
                ref = sum(r.get(tok, 0.0) for r in last)
                assert abs(score[0, hd, i] - ref) <= 1e-12 * max(1.0, ref)
                older = sum(r.get(tok, 0.0) for r in rows[hd][:-R])
                dropped |= older > 1e-3
            # rows sum to one, so the kept mass before eviction is the number of rows held
            assert abs(score[0, hd, :m].sum() - sum(sum(v for k, v in r.items() if k in
                       {int(x) for x in pos[0, hd, :m]}) for r in last)) < 1e-12
        O.compact_ring(ring, kept, cnt)
        O.compact(K, V, score, pos, kept, cnt, lens)
    assert dropped          # some cached token did lose weight that a running sum would have kept


def test_window_mass_without_eviction_is_the_number_of_rows(oracle):
    O = oracle
    rng = np.random.default_rng(15)
    b, h, cap, d, R = 1, 1, 32, 4, 4
    K, V, pos, lens = _state(rng, b, h, cap, d, [6])
    ring = np.zeros((b, h, R, cap))
    ring[..., lens[0]:] = 7.0              # unused slots may hold anything: a new token starts with no history
    score = np.zeros((b, h, cap))
    n = lens.copy()
    for t in range(7):
        n = n + 1
        q, kn, vn = (rng.standard_normal((b, h, d)) for _ in range(3))
        kept, cnt, out, p = O.decode_step_window(q, kn, vn, K, V, ring, t % R, score, pos, lens, n, 3, 0, 0.5)
        assert cnt[0] == lens[0]                                   # sparsity 0: nothing leaves
        np.testing.assert_allclose(score[0, 0, :lens[0]].sum(), min(t + 1, R), rtol=1e-12)


def test_prefill_attention_is_causal_dense_attention(oracle):
    """Eq. 1-2 with the causal mask: every row against the library softmax; the last row against the
    oracle's own decode step at sparsity 0 (an independent path); no dependence on later tokens."""
    O = oracle
    rng = np.random.default_rng(16)
    b, h, cap, d = 2, 2, 24, 5
    K, V, pos, lens = _state(rng, b, h, cap, d, [19, 7])
    Q = rng.standard_normal((b, h, cap, d))
    out = O.prefill_attention(Q, K, V, lens, 0.45)
    for s in range(b):
        L = lens[s]
        assert np.all(out[s, :, L:] == 0)
        for hd in range(h):
            np.testing.assert_allclose(out[s, hd, 0], V[s, hd, 0], rtol=1e-13)     # one visible token
            for t in range(L):
                a = softmax(K[s, hd, :t + 1] @ Q[s, hd, t] * 0.45)
                np.testing.assert_allclose(out[s, hd, t], a @ V[s, hd, :t + 1], rtol=1e-12, atol=1e-14)
    # the last prompt row is a decode step over the first s-1 tokens plus the last one, nothing evicted
    Kc, Vc = K.copy(), V.copy()
    score = np.zeros((b, h, cap))
    pc = pos.copy()
    lm1 = lens - 1
    kn = np.stack([K[s, :, lens[s] - 1] for s in range(b)])
    vn = np.stack([V[s, :, lens[s] - 1] for s in range(b)])
    qn = np.stack([Q[s, :, lens[s] - 1] for s in range(b)])
    _, _, o_dec, _ = O.decode_step(qn, kn, vn, Kc, Vc, score, pc, lm1.copy(), lens, 3, 0, 0.45)
    for s in range(b):
        np.testing.assert_allclose(out[s, :, lens[s] - 1], o_dec[s], rtol=1e-12, atol=1e-14)
    # causality: changing everything from position 5 on leaves rows 0..4 alone
    K2, V2, Q2 = K.copy(), V.copy(), Q.copy()
    K2[:, :, 5:] += 1.0
    V2[:, :, 5:] -= 2.0
    Q2[:, :, 5:] *= 3.0
    out2 = O.prefill_attention(Q2, K2, V2, lens, 0.45)
    assert np.array_equal(out2[:, :, :5], out[:, :, :5])
    assert not np.allclose(out2[0, :, 5:19], out[0, :, 5:19])


def test_window_step_with_the_head_reduced_token_set(oracle):
    # Algorithm 1's header note on top of its line 2: the window sums of the heads are added and every
    # head of a sequence keeps the same tokens.  Pinned against the separately pinned pieces: the
    # window sums of the per-head step, summed over the heads with numpy, ranked by brute force.
    O = oracle
    rng = np.random.default_rng(23)
    b, h, cap, d, R, w, sp = 2, 3, 40, 5, 3, 2, 5000
    K, V, pos, lens = _state(rng, b, h, cap, d, [21, 12])
    ring = np.zeros((b, h, R, cap))
    ring[:, :, :R] = O.prefill_rows(rng.standard_normal((b, h, R, d)), K, lens, 0.5)
    A = dict(K=K.copy(), V=V.copy(), pos=pos.copy(), len=lens.copy(), score=np.zeros((b, h, cap)), ring=ring.copy())
    Bs = dict(K=K.copy(), V=V.copy(), pos=pos.copy(), len=lens.copy(), score=np.zeros((b, h, cap)), ring=ring.copy())
    n = lens.copy()
    for t in range(6):
        n = n + 1
        q, kn, vn = (rng.standard_normal((b, h, d)) for _ in range(3))
        # per-head step on a copy: gives the window sums (they do not depend on the selection)
        tmp = {k: v.copy() for k, v in A.items()}
        O.decode_step_window(q, kn, vn, tmp["K"], tmp["V"], tmp["ring"], t % R, tmp["score"], tmp["pos"], tmp["len"],
                             n, w, sp, 0.5)
        kept, cnt, out, p = O.decode_step_window(q, kn, vn, Bs["K"], Bs["V"], Bs["ring"], t % R, Bs["score"],
                                                 Bs["pos"], Bs["len"], n, w, sp, 0.5, head_shared=True)
        np.testing.assert_array_equal(Bs["score"], tmp["score"])
        for s in range(b):
            m = Bs["len"][s]
            keep, nl, ng = O.budget(int(n[s]), int(m), w, sp)
            assert cnt[s] == keep
            tot = Bs["score"][s].sum(axis=0)[:m - nl]
            order = sorted(range(m - nl), key=lambda i: (-tot[i], i))[:ng]
            want = sorted(order) + list(range(m - nl, m))
            for hd in range(h):
                assert kept[s, hd, :keep].tolist() == want
            # the output is the renormalised attention over that set
            for hd in range(h):
                z = Bs["K"][s, hd, want] @ q[s, hd] * 0.5
                np.testing.assert_allclose(out[s, hd], softmax(z) @ Bs["V"][s, hd, want], rtol=1e-10, atol=1e-12)
        O.compact_ring(Bs["ring"], kept, cnt)
        O.compact(Bs["K"], Bs["V"], Bs["score"], Bs["pos"], kept, cnt, Bs["len"])
        # keep the per-head reference state in step with the shared one
        A = {k: v.copy() for k, v in Bs.items()}
    # a single head: the shared rule is the per-head rule
    K1, V1, pos1, lens1 = _state(rng, 1, 1, 30, 4, [15])
    r1 = np.zeros((1, 1, 2, 30))
    q, kn, vn = (rng.standard_normal((1, 1, 4)) for _ in range(3))
    a = O.decode_step_window(q, kn, vn, K1.copy(), V1.copy(), r1.copy(), 0, np.zeros((1, 1, 30)), pos1.copy(),
                             lens1.copy(), lens1 + 1, 3, 6000, 0.5)
    b_ = O.decode_step_window(q, kn, vn, K1.copy(), V1.copy(), r1.copy(), 0, np.zeros((1, 1, 30)), pos1.copy(),
                              lens1.copy(), lens1 + 1, 3, 6000, 0.5, head_shared=True)
    np.testing.assert_array_equal(a[0], b_[0])
    np.testing.assert_array_equal(a[2], b_[2])
