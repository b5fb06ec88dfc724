"""Pins of the oracle's KV-compression routines (Section V-B) against what the paper's formulas and
plain arithmetic fix: a hand-worked channel, the half-step error bound, exact recovery of data
that already lies on an 8-bit affine grid, channel-wise independence, saturation of late tokens.
CPU only."""
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    rows = []
    with open(os.path.join(HERE, "golden", "kv_quant.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            x, t, code, xhat, kind = line.split()
            rows.append((float(x), float(t), int(code), float(xhat), kind))
    return rows


def test_hand_worked_channel(oracle):
    O = oracle
    rows = _golden()
    cached = [r for r in rows if r[4] == "cached"]
    late = [r for r in rows if r[4] == "late"]
    # channel 0 is the worked one; channel 1 is there so that a transposed layout would show
    X = np.zeros((1, 1, len(cached), 2))
    X[0, 0, :, 0] = [r[0] for r in cached]
    X[0, 0, :, 1] = np.linspace(3.0, 5.0, len(cached))
    cnt = np.array([len(cached)], dtype=np.int32)
    lam, zero = O.kv_qparams(X, cnt)
    assert lam[0, 0, 0] == np.float32(1.0 / 128.0) and zero[0, 0, 0] == 128.0
    codes = O.kv_quantize(X, cnt, lam, zero)
    assert codes[0, 0, :, 0].tolist() == [r[2] for r in cached]
    back = O.kv_dequantize(codes, cnt, lam, zero)
    assert back[0, 0, :, 0].tolist() == [r[3] for r in cached]
    # tokens that arrive later reuse the parameters and saturate
    Y = np.zeros((1, 1, len(late), 2))
    Y[0, 0, :, 0] = [r[0] for r in late]
    Y[0, 0, :, 1] = 4.0
    cl = np.array([len(late)], dtype=np.int32)
    c2 = O.kv_quantize(Y, cl, lam, zero)
    assert c2[0, 0, :, 0].tolist() == [r[2] for r in late]
    assert O.kv_dequantize(c2, cl, lam, zero)[0, 0, :, 0].tolist() == [r[3] for r in late]


def _rand(rng, b, h, rows, d):
    X = rng.standard_normal((b, h, rows, d)) * rng.uniform(0.2, 4.0, size=(b, h, 1, d)) \
        + rng.uniform(-3, 3, size=(b, h, 1, d))
    return X.astype(np.float16).astype(np.float64)


def test_round_trip_error_is_at_most_half_a_step(oracle):
    O = oracle
    rng = np.random.default_rng(5)
    X = _rand(rng, 2, 3, 37, 16)
    cnt = np.array([37, 21], dtype=np.int32)
    lam, zero = O.kv_qparams(X, cnt)
    assert np.array_equal(zero, np.rint(zero))        # the zero point is itself a rounded integer
    assert not np.all(np.abs(zero) < 1)
    codes = O.kv_quantize(X, cnt, lam, zero)
    back = O.kv_dequantize(codes, cnt, lam, zero)
    for s in range(2):
        L = cnt[s]
        x, y = X[s, :, :L], back[s, :, :L]
        step = lam[s][:, None, :].astype(np.float64)
        assert np.all(np.abs(x - y) <= 0.5 * step * (1 + 1e-5) + 1e-7)
        # the range is used: the smallest value takes code 0, the largest 254 or 255
        assert np.all(codes[s, :, :L].min(axis=1) == 0)
        assert np.all(codes[s, :, :L].max(axis=1) >= 254)
        # lambda is the range over 255 steps
        rngc = x.max(axis=1) - x.min(axis=1)
        np.testing.assert_allclose(lam[s], rngc / 255.0, rtol=1e-6)
        # min maps to code 0: -min/lambda within half a step of the zero point
        assert np.all(np.abs(-x.min(axis=1) / lam[s] - zero[s]) <= 0.5 + 1e-3)
    # rows past the count are neither read for the range nor written
    assert np.all(codes[1, :, 21:] == 0) and np.all(back[1, :, 21:] == 0)
    X2 = X.copy()
    X2[1, :, 21:] = 1e4
    lam2, zero2 = O.kv_qparams(X2, cnt)
    assert np.array_equal(lam, lam2) and np.array_equal(zero, zero2)


def test_codes_are_monotone_in_the_value(oracle):
    O = oracle
    rng = np.random.default_rng(6)
    X = _rand(rng, 1, 2, 64, 8)
    cnt = np.array([64], dtype=np.int32)
    lam, zero = O.kv_qparams(X, cnt)
    codes = O.kv_quantize(X, cnt, lam, zero)
    for hd in range(2):
        for c in range(8):
            order = np.argsort(X[0, hd, :, c], kind="stable")
            assert np.all(np.diff(codes[0, hd, order, c].astype(np.int32)) >= 0)


def test_data_on_an_8_bit_affine_grid_is_recovered_exactly(oracle):
    O = oracle
    rng = np.random.default_rng(7)
    b, h, rows, d = 1, 2, 300, 4
    k = rng.integers(0, 256, size=(b, h, rows, d))
    k[:, :, 0, :] = 0
    k[:, :, 1, :] = 255
    step = np.array([2.0 ** -6, 2.0 ** -9, 2.0 ** -3, 2.0 ** -7])
    k0 = np.array([17, 128, 255, 0])
    X = (k - k0) * step                       # exactly representable in fp16
    assert np.array_equal(X.astype(np.float16).astype(np.float64), X)
    cnt = np.array([rows], dtype=np.int32)
    lam, zero = O.kv_qparams(X, cnt)
    assert np.array_equal(lam[0, 0], step.astype(np.float32)) and np.array_equal(zero[0, 1], k0)
    codes = O.kv_quantize(X, cnt, lam, zero)
    assert np.array_equal(codes, k)
    assert np.array_equal(O.kv_dequantize(codes, cnt, lam, zero), X)


def test_parameters_are_per_channel_and_per_pair(oracle):
    O = oracle
    rng = np.random.default_rng(8)
    X = _rand(rng, 2, 2, 40, 6)
    cnt = np.array([40, 40], dtype=np.int32)
    lam, zero = O.kv_qparams(X, cnt)
    codes = O.kv_quantize(X, cnt, lam, zero)
    Y = X.copy()
    Y[1, 0, :, 3] *= 2.0                       # exact in fp16/fp32: scale doubles, codes stay
    lam2, zero2 = O.kv_qparams(Y, cnt)
    codes2 = O.kv_quantize(Y, cnt, lam2, zero2)
    assert lam2[1, 0, 3] == 2 * lam[1, 0, 3] and zero2[1, 0, 3] == zero[1, 0, 3]
    lam2[1, 0, 3] = lam[1, 0, 3]
    assert np.array_equal(lam, lam2) and np.array_equal(zero, zero2) and np.array_equal(codes, codes2)


def test_flat_channel_takes_the_minimum_range(oracle):
    O = oracle
    X = np.full((1, 1, 9, 3), 0.75)
    X[0, 0, :, 1] = -6.5
    X[0, 0, :, 2] = np.linspace(0, 1, 9)
    cnt = np.array([9], dtype=np.int32)
    lam, zero = O.kv_qparams(X, cnt)
    floor = np.float32(2.0 ** -7) / np.float32(255.0)
    assert lam[0, 0, 0] == floor and lam[0, 0, 1] == floor and lam[0, 0, 2] > floor
    back = O.kv_dequantize(O.kv_quantize(X, cnt, lam, zero), cnt, lam, zero)
    assert np.all(np.abs(back[..., :2] - X[..., :2]) <= 1.5 * float(floor))
    # an empty cache still gives usable parameters
    lam0, zero0 = O.kv_qparams(X, np.array([0], dtype=np.int32))
    assert np.all(lam0 == floor) and np.all(zero0 == 0)


def test_attention_over_a_compressed_cache_is_attention_over_the_dequantised_values(oracle):
    """Sparsity 0: the step on the de-quantised cache is dense attention (Eq. 1-2) on those values."""
    O = oracle
    from scipy.special import softmax
    rng = np.random.default_rng(9)
    b, h, cap, d, L = 1, 2, 24, 8, 11
    K = np.zeros((b, h, cap, d))
    V = np.zeros((b, h, cap, d))
    K[:, :, :L] = _rand(rng, b, h, L, d)
    V[:, :, :L] = _rand(rng, b, h, L, d)
    cnt = np.array([L], dtype=np.int32)
    Kq = O.kv_dequantize(O.kv_quantize(K, cnt, *O.kv_qparams(K, cnt)), cnt, *O.kv_qparams(K, cnt))
    Vq = O.kv_dequantize(O.kv_quantize(V, cnt, *O.kv_qparams(V, cnt)), cnt, *O.kv_qparams(V, cnt))
    q = rng.standard_normal((b, h, d))
    kn, vn = Kq[:, :, L - 1].copy(), Vq[:, :, L - 1].copy()
    Kc, Vc = Kq.copy(), Vq.copy()
    score = np.zeros((b, h, cap))
    pos = np.full((b, h, cap), -1, dtype=np.int32)
    pos[:, :, :L - 1] = np.arange(L - 1)
    clen = np.array([L - 1], dtype=np.int32)
    _, _, out, _ = O.decode_step(q, kn, vn, Kc, Vc, score, pos, clen, np.array([L], dtype=np.int32),
                                 4, 0, 0.3)
    for hd in range(h):
        a = softmax(Kq[0, hd, :L] @ q[0, hd] * 0.3)
        np.testing.assert_allclose(out[0, hd], a @ Vq[0, hd, :L], rtol=1e-12, atol=1e-14)
