"""Pins for the CPU oracle: facts fixed by the mathematics of the cell grid, not by the oracle.

Each test checks the oracle (oracle/rnn_oracle.c) against something written independently of
it: a closed form, a scalar recursion in pure Python, an invariant of the unrolled cell grid
(Section 2.2 of the paper: cell (l, t) depends on (l, t-1) and (l-1, t) only), a brute-force
evaluation with a different loop structure, or an fp64 library RNN.
"""
import math

import numpy as np
import pytest

LSTM, GRU = 0, 1


def sig(a):
    return 1.0 / (1.0 + math.exp(-a))


def rand_weights(rng, cell, L, D, I, H, scale=None, bias=True):
    G = 4 if cell == LSTM else 3
    k = scale if scale is not None else 1.0 / math.sqrt(H)
    ws = []
    for l in range(L):
        il = I if l == 0 else D * H
        for _ in range(D):
            ws.append(rng.uniform(-k, k, size=(G * H, il)))
            ws.append(rng.uniform(-k, k, size=(G * H, H)))
            ws.append(rng.uniform(-k, k, size=(G * H,)) if bias else None)
            ws.append(rng.uniform(-k, k, size=(G * H,)) if bias else None)
    return ws


# ---------------------------------------------------------------- P1 / P2: zero weights
def test_zero_weight_lstm_closed_form(oracle):
    # all W = 0, b = 0: i = f = o = 1/2, g = 0, so c_t = c0 / 2^t and h_t = tanh(c_t) / 2
    L, D, I, H, T, B = 1, 1, 3, 5, 7, 2
    ws = [np.zeros((4 * H, I)), np.zeros((4 * H, H)), None, None]
    rng = np.random.default_rng(1)
    x = rng.standard_normal((T, B, I))
    c0 = rng.standard_normal((1, B, H))
    h0 = rng.standard_normal((1, B, H))
    y, hT, cT = oracle.forward(LSTM, L, D, I, H, ws, x, h0=h0, c0=c0)
    for t in range(T):
        ct = c0[0] * 2.0 ** (-(t + 1))
        np.testing.assert_allclose(y[t], 0.5 * np.tanh(ct), rtol=0, atol=1e-15)
    np.testing.assert_allclose(cT[0], c0[0] * 2.0 ** (-T), rtol=0, atol=1e-15)
    y0, _, _ = oracle.forward(LSTM, L, D, I, H, ws, x)
    assert np.all(y0 == 0.0)


def test_zero_weight_gru_closed_form(oracle):
    # r = z = 1/2, n = tanh(0) = 0, so h_t = h0 / 2^t
    L, D, I, H, T, B = 1, 1, 2, 4, 6, 3
    ws = [np.zeros((3 * H, I)), np.zeros((3 * H, H)), None, None]
    rng = np.random.default_rng(2)
    x = rng.standard_normal((T, B, I))
    h0 = rng.standard_normal((1, B, H))
    for variant in (0, 1):
        y, hT, _ = oracle.forward(GRU, L, D, I, H, ws, x, h0=h0, gru_variant=variant)
        for t in range(T):
            np.testing.assert_allclose(y[t], h0[0] * 2.0 ** (-(t + 1)), rtol=0, atol=1e-15)
        np.testing.assert_allclose(hT[0], h0[0] * 2.0 ** (-T), rtol=0, atol=1e-15)


# ---------------------------------------------------------------- P3 / P4: hidden size 1
def test_hidden_size_one_single_step(oracle):
    rng = np.random.default_rng(3)
    for _ in range(5):
        wi, wh = rng.uniform(-1, 1, (4, 1)), rng.uniform(-1, 1, (4, 1))
        bi, bh = rng.uniform(-1, 1, 4), rng.uniform(-1, 1, 4)
        x = rng.standard_normal((1, 1, 1))
        xv = float(x[0, 0, 0])
        y, _, cT = oracle.forward(LSTM, 1, 1, 1, 1, [wi, wh, bi, bh], x)
        b = bi + bh
        c1 = sig(wi[0, 0] * xv + b[0]) * math.tanh(wi[2, 0] * xv + b[2])
        h1 = sig(wi[3, 0] * xv + b[3]) * math.tanh(c1)
        assert abs(y[0, 0, 0] - h1) < 1e-15 and abs(cT[0, 0, 0] - c1) < 1e-15

        wi, wh = rng.uniform(-1, 1, (3, 1)), rng.uniform(-1, 1, (3, 1))
        bi, bh = rng.uniform(-1, 1, 3), rng.uniform(-1, 1, 3)
        y, _, _ = oracle.forward(GRU, 1, 1, 1, 1, [wi, wh, bi, bh], x)
        r = sig(wi[0, 0] * xv + bi[0] + bh[0])
        z = sig(wi[1, 0] * xv + bi[1] + bh[1])
        h1 = (1 - z) * math.tanh(wi[2, 0] * xv + bi[2] + r * bh[2])
        assert abs(y[0, 0, 0] - h1) < 1e-15
        # variant 1 from zero state: r * h = 0, so the candidate sees b_hn unscaled
        y1, _, _ = oracle.forward(GRU, 1, 1, 1, 1, [wi, wh, bi, bh], x, gru_variant=1)
        h1b = (1 - z) * math.tanh(wi[2, 0] * xv + bi[2] + bh[2])
        assert abs(y1[0, 0, 0] - h1b) < 1e-15


def test_hidden_size_one_multi_step(oracle):
    rng = np.random.default_rng(4)
    T = 4
    x = rng.standard_normal((T, 1, 1))
    h0v, c0v = 0.3, -0.7
    # LSTM, scalar recursion unrolled by hand
    wi, wh = rng.uniform(-1, 1, (4, 1)), rng.uniform(-1, 1, (4, 1))
    bi, bh = rng.uniform(-1, 1, 4), rng.uniform(-1, 1, 4)
    y, hT, cT = oracle.forward(LSTM, 1, 1, 1, 1, [wi, wh, bi, bh], x,
                               h0=np.full((1, 1, 1), h0v), c0=np.full((1, 1, 1), c0v))
    h, c = h0v, c0v
    for t in range(T):
        xv = float(x[t, 0, 0])
        a = [wi[g, 0] * xv + bi[g] + wh[g, 0] * h + bh[g] for g in range(4)]
        c = sig(a[1]) * c + sig(a[0]) * math.tanh(a[2])
        h = sig(a[3]) * math.tanh(c)
        assert abs(y[t, 0, 0] - h) < 1e-14
    assert abs(hT[0, 0, 0] - h) < 1e-14 and abs(cT[0, 0, 0] - c) < 1e-14
    # GRU, both variants
    wi, wh = rng.uniform(-1, 1, (3, 1)), rng.uniform(-1, 1, (3, 1))
    bi, bh = rng.uniform(-1, 1, 3), rng.uniform(-1, 1, 3)
    for variant in (0, 1):
        y, hT, _ = oracle.forward(GRU, 1, 1, 1, 1, [wi, wh, bi, bh], x,
                                  h0=np.full((1, 1, 1), h0v), gru_variant=variant)
        h = h0v
        for t in range(T):
            xv = float(x[t, 0, 0])
            r = sig(wi[0, 0] * xv + bi[0] + wh[0, 0] * h + bh[0])
            z = sig(wi[1, 0] * xv + bi[1] + wh[1, 0] * h + bh[1])
            if variant == 0:
                n = math.tanh(wi[2, 0] * xv + bi[2] + r * (wh[2, 0] * h + bh[2]))
            else:
                n = math.tanh(wi[2, 0] * xv + bi[2] + wh[2, 0] * (r * h) + bh[2])
            h = (1 - z) * n + z * h
            assert abs(y[t, 0, 0] - h) < 1e-14
        assert abs(hT[0, 0, 0] - h) < 1e-14


# ---------------------------------------------------------------- P5: saturated gates
def _lstm_saturated(rng, I, H, b_i, b_f, b_o, zero_hh):
    """Weights whose i / f / o gates are pinned by a large bias (None = leave the gate free)."""
    wi = rng.uniform(-0.5, 0.5, (4 * H, I))
    wh = rng.uniform(-0.5, 0.5, (4 * H, H))
    bi = rng.uniform(-0.5, 0.5, 4 * H)
    bh = np.zeros(4 * H)
    for blk, val in ((0, b_i), (1, b_f), (3, b_o)):
        if val is not None:
            wi[blk * H:(blk + 1) * H] = 0
            wh[blk * H:(blk + 1) * H] = 0
            bi[blk * H:(blk + 1) * H] = val
    if zero_hh:
        wh[:] = 0
    return wi, wh, bi, bh


def test_saturated_lstm_identities(oracle):
    rng = np.random.default_rng(5)
    I, H, T, B = 3, 4, 6, 2
    x = rng.standard_normal((T, B, I))
    c0 = rng.uniform(-1, 1, (1, B, H))
    # forget = 1, input = 0: the cell state never changes; h_t = sigma(a_o) tanh(c0)
    wi, wh, bi, bh = _lstm_saturated(rng, I, H, -40.0, 40.0, None, zero_hh=True)
    y, hT, cT = oracle.forward(LSTM, 1, 1, I, H, [wi, wh, bi, bh], x, c0=c0)
    np.testing.assert_allclose(cT[0], c0[0], rtol=0, atol=1e-15)
    for t in range(T):
        ao = x[t] @ wi[3 * H:].T + bi[3 * H:]
        np.testing.assert_allclose(y[t], 1 / (1 + np.exp(-ao)) * np.tanh(c0[0]), atol=1e-14)
    # input = forget = 1, no recurrence: the cell state is a running sum of tanh(W_g x_t + b_g)
    wi, wh, bi, bh = _lstm_saturated(rng, I, H, 40.0, 40.0, None, zero_hh=True)
    _, _, cT = oracle.forward(LSTM, 1, 1, I, H, [wi, wh, bi, bh], x, c0=c0)
    acc = c0[0] + sum(np.tanh(x[t] @ wi[2 * H:3 * H].T + bi[2 * H:3 * H]) for t in range(T))
    np.testing.assert_allclose(cT[0], acc, rtol=0, atol=1e-13)
    # input = output = 1, forget = 0, no recurrence: memoryless, h_t = tanh(tanh(W_g x_t + b_g))
    wi, wh, bi, bh = _lstm_saturated(rng, I, H, 40.0, -40.0, 40.0, zero_hh=True)
    y, _, _ = oracle.forward(LSTM, 1, 1, I, H, [wi, wh, bi, bh], x, c0=c0)
    dense = np.tanh(np.tanh(x.reshape(T * B, I) @ wi[2 * H:3 * H].T + bi[2 * H:3 * H]))
    np.testing.assert_allclose(y.reshape(T * B, H), dense, rtol=0, atol=1e-14)


def test_saturated_lstm_recurrent_term(oracle):
    # input = output = 1, forget = 0, W_hh kept for the candidate: h_t = tanh(tanh(W_g x + U_g h + b_g)),
    # a plain nonlinear recurrence evaluated here with matrix products
    rng = np.random.default_rng(6)
    I, H, T, B = 2, 3, 5, 2
    x = rng.standard_normal((T, B, I))
    wi, wh, bi, bh = _lstm_saturated(rng, I, H, 40.0, -40.0, 40.0, zero_hh=False)
    bh[2 * H:3 * H] = rng.uniform(-0.5, 0.5, H)
    h0 = rng.uniform(-0.5, 0.5, (1, B, H))
    y, _, _ = oracle.forward(LSTM, 1, 1, I, H, [wi, wh, bi, bh], x, h0=h0)
    h = h0[0]
    for t in range(T):
        h = np.tanh(np.tanh(x[t] @ wi[2 * H:3 * H].T + h @ wh[2 * H:3 * H].T
                            + bi[2 * H:3 * H] + bh[2 * H:3 * H]))
        np.testing.assert_allclose(y[t], h, rtol=0, atol=1e-14)


def test_saturated_gru_identities(oracle):
    rng = np.random.default_rng(7)
    I, H, T, B = 3, 4, 5, 2
    x = rng.standard_normal((T, B, I))
    h0 = rng.uniform(-1, 1, (1, B, H))
    wi = rng.uniform(-0.5, 0.5, (3 * H, I))
    wh = rng.uniform(-0.5, 0.5, (3 * H, H))
    bi = rng.uniform(-0.5, 0.5, 3 * H)
    bh = rng.uniform(-0.5, 0.5, 3 * H)
    # update gate = 1: the state is copied forever
    wi1, wh1, bi1, bh1 = wi.copy(), wh.copy(), bi.copy(), bh.copy()
    wi1[H:2 * H] = 0; wh1[H:2 * H] = 0; bi1[H:2 * H] = 40.0; bh1[H:2 * H] = 0
    y, hT, _ = oracle.forward(GRU, 1, 1, I, H, [wi1, wh1, bi1, bh1], x, h0=h0)
    np.testing.assert_allclose(hT[0], h0[0], rtol=0, atol=1e-14)
    # update gate = 0, no recurrence: h_t = tanh(W_in x + b_in + sigma(W_ir x + b_ir + b_hr) b_hn)
    wi2, wh2, bi2, bh2 = wi.copy(), np.zeros_like(wh), bi.copy(), bh.copy()
    wi2[H:2 * H] = 0; bi2[H:2 * H] = -40.0; bh2[H:2 * H] = 0
    y, _, _ = oracle.forward(GRU, 1, 1, I, H, [wi2, wh2, bi2, bh2], x, h0=h0)
    r = 1 / (1 + np.exp(-(x @ wi2[:H].T + bi2[:H] + bh2[:H])))
    ref = np.tanh(x @ wi2[2 * H:].T + bi2[2 * H:] + r * bh2[2 * H:])
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- P6: split sequence
@pytest.mark.parametrize("cell", [LSTM, GRU])
def test_split_sequence_equals_whole(oracle, cell):
    rng = np.random.default_rng(8)
    L, D, I, H, T, B = 2, 1, 3, 4, 7, 2
    ws = rand_weights(rng, cell, L, D, I, H)
    x = rng.standard_normal((T, B, I))
    h0 = rng.uniform(-1, 1, (L, B, H))
    c0 = rng.uniform(-1, 1, (L, B, H)) if cell == LSTM else None
    y, hT, cT = oracle.forward(cell, L, D, I, H, ws, x, h0=h0, c0=c0)
    for k in (1, 3, 6):
        ya, ha, ca = oracle.forward(cell, L, D, I, H, ws, x[:k], h0=h0, c0=c0)
        yb, hb, cb = oracle.forward(cell, L, D, I, H, ws, x[k:], h0=ha, c0=ca)
        assert np.array_equal(np.concatenate([ya, yb]), y)
        assert np.array_equal(hb, hT)
        if cell == LSTM:
            assert np.array_equal(cb, cT)
    # one step at a time
    h, c = h0, c0
    for t in range(T):
        yt, h, c = oracle.forward(cell, L, D, I, H, ws, x[t:t + 1], h0=h, c0=c)
        assert np.array_equal(yt[0], y[t])


# ---------------------------------------------------------------- P7: layer composition
@pytest.mark.parametrize("cell,D", [(LSTM, 1), (LSTM, 2), (GRU, 1), (GRU, 2)])
def test_layers_compose(oracle, cell, D):
    rng = np.random.default_rng(9)
    L, I, H, T, B = 3, 3, 4, 5, 2
    ws = rand_weights(rng, cell, L, D, I, H)
    x = rng.standard_normal((T, B, I))
    lengths = np.array([5, 3], dtype=np.int32)
    h0 = rng.uniform(-1, 1, (L * D, B, H))
    c0 = rng.uniform(-1, 1, (L * D, B, H))
    y, hT, cT, layers = oracle.forward(cell, L, D, I, H, ws, x, lengths, h0, c0, return_layers=True)
    cur = x
    for l in range(L):
        il = I if l == 0 else D * H
        sl = slice(l * D, (l + 1) * D)
        yl, hl, cl = oracle.forward(cell, 1, D, il, H, ws[l * D * 4:(l + 1) * D * 4], cur, lengths,
                                    h0[sl], c0[sl])
        assert np.array_equal(yl, layers[l])
        assert np.array_equal(hl, hT[sl])
        if cell == LSTM:
            assert np.array_equal(cl, cT[sl])
        cur = yl
    assert np.array_equal(cur, y)


# ---------------------------------------------------------------- P8: direction symmetry
@pytest.mark.parametrize("cell", [LSTM, GRU])
def test_backward_direction_is_time_reversed_forward(oracle, cell):
    rng = np.random.default_rng(10)
    I, H, T, B = 3, 4, 6, 3
    ws = rand_weights(rng, cell, 1, 2, I, H)
    x = rng.standard_normal((T, B, I))
    lengths = np.array([6, 2, 4], dtype=np.int32)
    h0 = rng.uniform(-1, 1, (2, B, H))
    c0 = rng.uniform(-1, 1, (2, B, H))
    y, hT, cT = oracle.forward(cell, 1, 2, I, H, ws, x, lengths, h0, c0)
    # forward half == unidirectional model with the forward weights
    yf, hf, cf = oracle.forward(cell, 1, 1, I, H, ws[:4], x, lengths, h0[:1], c0[:1])
    assert np.array_equal(y[:, :, :H], yf) and np.array_equal(hT[:1], hf)
    # backward half == forward model with the backward weights on each sequence reversed in time
    xr = np.zeros_like(x)
    for b in range(B):
        n = lengths[b]
        xr[:n, b] = x[:n, b][::-1]
    yb, hb, cb = oracle.forward(cell, 1, 1, I, H, ws[4:], xr, lengths, h0[1:], c0[1:])
    for b in range(B):
        n = lengths[b]
        assert np.array_equal(y[:n, b, H:], yb[:n, b][::-1])
        assert np.all(y[n:, b, :] == 0.0)
    assert np.array_equal(hT[1:], hb)
    if cell == LSTM:
        assert np.array_equal(cT[1:], cb)


# ---------------------------------------------------------------- P9: batch independence, padding
@pytest.mark.parametrize("cell", [LSTM, GRU])
def test_batch_independence_and_padding(oracle, cell):
    rng = np.random.default_rng(11)
    L, D, I, H, T, B = 2, 2, 3, 4, 6, 4
    ws = rand_weights(rng, cell, L, D, I, H)
    x = rng.standard_normal((T, B, I))
    lengths = np.array([6, 1, 4, 3], dtype=np.int32)
    h0 = rng.uniform(-1, 1, (L * D, B, H))
    c0 = rng.uniform(-1, 1, (L * D, B, H))
    y, hT, cT = oracle.forward(cell, L, D, I, H, ws, x, lengths, h0, c0)
    for b in range(B):
        n = int(lengths[b])
        # alone, without any padding
        y1, h1, c1 = oracle.forward(cell, L, D, I, H, ws, x[:n, b:b + 1], None, h0[:, b:b + 1],
                                    c0[:, b:b + 1])
        assert np.array_equal(y[:n, b], y1[:, 0])
        assert np.array_equal(hT[:, b], h1[:, 0])
        if cell == LSTM:
            assert np.array_equal(cT[:, b], c1[:, 0])
        # padded positions are +0.0 bit patterns
        assert np.all(y[n:, b].view(np.uint64) == 0)
        # final states of the top layer are the outputs at the sequence's ends
        assert np.array_equal(hT[(L - 1) * D + 0, b], y[n - 1, b, :H])
        assert np.array_equal(hT[(L - 1) * D + 1, b], y[0, b, H:])
    # padding content must not matter
    x2 = x.copy()
    for b in range(B):
        x2[lengths[b]:, b] = 123.0
    y2, hT2, _ = oracle.forward(cell, L, D, I, H, ws, x2, lengths, h0, c0)
    assert np.array_equal(y, y2) and np.array_equal(hT, hT2)
    # permuting the batch permutes the outputs
    perm = np.array([2, 0, 3, 1])
    yp, hp, _ = oracle.forward(cell, L, D, I, H, ws, x[:, perm], lengths[perm], h0[:, perm], c0[:, perm])
    assert np.array_equal(yp, y[:, perm]) and np.array_equal(hp, hT[:, perm])


# ---------------------------------------------------------------- P10: bounds
def test_bounds(oracle):
    rng = np.random.default_rng(12)
    I, H, T, B = 4, 6, 20, 3
    x = 3 * rng.standard_normal((T, B, I))
    ws = rand_weights(rng, LSTM, 1, 1, I, H, scale=2.0)
    c0 = rng.uniform(-2, 2, (1, B, H))
    prev = np.abs(c0[0])
    for t in range(1, T + 1):
        y, hT, cT = oracle.forward(LSTM, 1, 1, I, H, ws, x[:t], c0=c0)
        assert np.all(np.isfinite(y)) and np.all(np.abs(y) < 1.0)
        assert np.all(np.abs(cT[0]) <= prev + 1.0)
        prev = np.abs(cT[0])
    ws = rand_weights(rng, GRU, 1, 1, I, H, scale=2.0)
    h0 = rng.uniform(-3, 3, (1, B, H))
    y, hT, _ = oracle.forward(GRU, 1, 1, I, H, ws, x, h0=h0)
    bound = np.maximum(np.abs(h0[0]), 1.0)
    for t in range(T):
        assert np.all(np.abs(y[t]) <= bound + 1e-15)


# ---------------------------------------------------------------- P11: brute force, tiny
def _brute(cell, L, D, I, H, ws, x, lengths, h0, c0, gru_variant=0):
    """Whole network with Python floats; time is the outer loop and every product is spelled out.
    gru_variant 1: the candidate's recurrent product runs over r_k * h_k, with the reset gate of
    every unit k computed first (each unit's own r multiplies that unit's own previous state)."""
    T, B, _ = x.shape
    G = 4 if cell == LSTM else 3
    cur = [[[float(v) for v in x[t, b]] for b in range(B)] for t in range(T)]
    hT = {}
    cT = {}
    for l in range(L):
        il = I if l == 0 else D * H
        nxt = [[[0.0] * (D * H) for _ in range(B)] for _ in range(T)]
        for d in range(D):
            Wi, Wh, bi, bh = ws[(l * D + d) * 4:(l * D + d) * 4 + 4]
            hs = [[float(h0[l * D + d, b, j]) for j in range(H)] for b in range(B)]
            cs = [[float(c0[l * D + d, b, j]) for j in range(H)] for b in range(B)]
            order = range(T) if d == 0 else range(T - 1, -1, -1)
            for t in order:
                for b in range(B):
                    if t >= lengths[b]:
                        continue
                    a = []
                    ah = []
                    for row in range(G * H):
                        sx = float(bi[row])
                        for k in range(il):
                            sx = sx + float(Wi[row, k]) * cur[t][b][k]
                        sh = float(bh[row])
                        for k in range(H):
                            sh = sh + float(Wh[row, k]) * hs[b][k]
                        a.append(sx)
                        ah.append(sh)
                    hn = [0.0] * H
                    if cell != LSTM and gru_variant == 1:
                        # reset gates of all units first, then W_hn (r * h) term by term
                        r_all = [sig(a[k] + ah[k]) for k in range(H)]
                        for j in range(H):
                            sh = float(bh[2 * H + j])
                            for k in range(H):
                                sh = sh + float(Wh[2 * H + j, k]) * (r_all[k] * hs[b][k])
                            z_ = sig(a[H + j] + ah[H + j])
                            n_ = math.tanh(a[2 * H + j] + sh)
                            hn[j] = (1 - z_) * n_ + z_ * hs[b][j]
                    for j in range(H):
                        if cell != LSTM and gru_variant == 1:
                            break
                        if cell == LSTM:
                            i_ = sig(a[j] + ah[j]); f_ = sig(a[H + j] + ah[H + j])
                            g_ = math.tanh(a[2 * H + j] + ah[2 * H + j]); o_ = sig(a[3 * H + j] + ah[3 * H + j])
                            cs[b][j] = f_ * cs[b][j] + i_ * g_
                            hn[j] = o_ * math.tanh(cs[b][j])
                        else:
                            r_ = sig(a[j] + ah[j]); z_ = sig(a[H + j] + ah[H + j])
                            n_ = math.tanh(a[2 * H + j] + r_ * ah[2 * H + j])
                            hn[j] = (1 - z_) * n_ + z_ * hs[b][j]
                    hs[b] = hn
                    for j in range(H):
                        nxt[t][b][d * H + j] = hn[j]
            hT[l * D + d] = hs
            cT[l * D + d] = cs
        cur = nxt
    return np.array(cur), np.array([hT[i] for i in range(L * D)]), np.array([cT[i] for i in range(L * D)])


@pytest.mark.parametrize("cell,variant,H", [(LSTM, 0, 2), (GRU, 0, 2), (GRU, 1, 2), (GRU, 1, 3)])
def test_brute_force_tiny(oracle, cell, variant, H):
    rng = np.random.default_rng(13)
    L, D, I, T, B = 2, 2, 2, 3, 2
    ws = rand_weights(rng, cell, L, D, I, H, scale=1.0)
    x = rng.standard_normal((T, B, I))
    lengths = np.array([3, 2], dtype=np.int32)
    h0 = rng.uniform(-1, 1, (L * D, B, H))
    c0 = rng.uniform(-1, 1, (L * D, B, H))
    y, hT, cT = oracle.forward(cell, L, D, I, H, ws, x, lengths, h0, c0, gru_variant=variant)
    yb, hb, cb = _brute(cell, L, D, I, H, ws, x, lengths, h0, c0, gru_variant=variant)
    np.testing.assert_allclose(y, yb, rtol=0, atol=1e-13)
    np.testing.assert_allclose(hT, hb, rtol=0, atol=1e-13)
    if cell == LSTM:
        np.testing.assert_allclose(cT, cb, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- P12: fp64 library RNN (secondary)
@pytest.mark.parametrize("cell,D", [(LSTM, 1), (LSTM, 2), (GRU, 1), (GRU, 2)])
def test_against_library_rnn_fp64(oracle, cell, D):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(14)
    L, I, H, T, B = 2, 5, 7, 9, 3
    ws = rand_weights(rng, cell, L, D, I, H)
    x = rng.standard_normal((T, B, I))
    h0 = rng.uniform(-1, 1, (L * D, B, H))
    c0 = rng.uniform(-1, 1, (L * D, B, H))
    mod = (torch.nn.LSTM if cell == LSTM else torch.nn.GRU)(I, H, num_layers=L, bidirectional=(D == 2)).double()
    with torch.no_grad():
        for l in range(L):
            for d in range(D):
                sfx = "_l%d%s" % (l, "_reverse" if d == 1 else "")
                w = ws[(l * D + d) * 4:(l * D + d) * 4 + 4]
                for name, arr in zip(("weight_ih", "weight_hh", "bias_ih", "bias_hh"), w):
                    getattr(mod, name + sfx).copy_(torch.from_numpy(arr))
        xt = torch.from_numpy(x)
        if cell == LSTM:
            yt, (ht, ct) = mod(xt, (torch.from_numpy(h0), torch.from_numpy(c0)))
        else:
            yt, ht = mod(xt, torch.from_numpy(h0))
    y, hT, cT = oracle.forward(cell, L, D, I, H, ws, x, None, h0, c0)
    np.testing.assert_allclose(y, yt.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(hT, ht.numpy(), rtol=0, atol=1e-12)
    if cell == LSTM:
        np.testing.assert_allclose(cT, ct.numpy(), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- misc: threads, arguments
def test_threads_do_not_change_results(oracle):
    rng = np.random.default_rng(15)
    L, D, I, H, T, B = 2, 2, 8, 16, 5, 3
    for cell in (LSTM, GRU):
        ws = rand_weights(rng, cell, L, D, I, H)
        x = rng.standard_normal((T, B, I))
        a = oracle.forward(cell, L, D, I, H, ws, x, nthreads=1)
        b = oracle.forward(cell, L, D, I, H, ws, x, nthreads=4)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_rejects_bad_lengths(oracle):
    ws = [np.zeros((4, 1)), np.zeros((4, 1)), None, None]
    x = np.zeros((3, 2, 1))
    for bad in ([0, 1], [4, 1]):
        with pytest.raises(ValueError):
            oracle.forward(LSTM, 1, 1, 1, 1, ws, x, lengths=np.array(bad, dtype=np.int32))


def test_projection_is_a_matrix_product(oracle):
    rng = np.random.default_rng(16)
    a = rng.standard_normal((7, 5))
    w = rng.standard_normal((6, 5))
    np.testing.assert_allclose(oracle.projection(a, w), a @ w.T, rtol=0, atol=1e-14)
    # the projection plus the recurrent part is what the cell sees: a one-step LSTM from zero
    # state with o, i saturated open and f closed gives h = tanh(tanh(P_g))
    H, I = 3, 5
    wi = np.zeros((4 * H, I)); wi[2 * H:3 * H] = w[:H]
    bi = np.zeros(4 * H); bi[:H] = 40; bi[H:2 * H] = -40; bi[3 * H:] = 40
    y, _, _ = oracle.forward(LSTM, 1, 1, I, H, [wi, np.zeros((4 * H, H)), bi, None], a[:, None, :])
    np.testing.assert_allclose(y[:, 0], np.tanh(np.tanh(oracle.projection(a, w[:H]))), atol=1e-14)


# ---------------------------------------------------------------- peepholes and clipping (the ONNX operator's optional terms)
def _clamp(a, c):
    return max(-c, min(c, a))


def test_peephole_scalar_recursion(oracle):
    # hidden size 1, two layers, unrolled by hand: i and f see c_{t-1}, o sees the new c_t
    rng = np.random.default_rng(31)
    T = 5
    x = rng.standard_normal((T, 1, 1))
    ws, ps = [], []
    for _ in range(2):
        ws += [rng.uniform(-1, 1, (4, 1)), rng.uniform(-1, 1, (4, 1)), rng.uniform(-1, 1, 4), rng.uniform(-1, 1, 4)]
        ps.append(rng.uniform(-2, 2, (3, 1)))
    h0 = rng.uniform(-1, 1, (2, 1, 1))
    c0 = rng.uniform(-2, 2, (2, 1, 1))
    y, hT, cT = oracle.forward(LSTM, 2, 1, 1, 1, ws, x, h0=h0, c0=c0, peepholes=ps)
    seq = [float(v) for v in x[:, 0, 0]]
    for l in range(2):
        wi, wh, bi, bh = ws[4 * l:4 * l + 4]
        pi, pf, po = (float(v) for v in ps[l][:, 0])
        h, c = float(h0[l, 0, 0]), float(c0[l, 0, 0])
        out = []
        for xv in seq:
            a = [wi[g, 0] * xv + bi[g] + wh[g, 0] * h + bh[g] for g in range(4)]
            i_ = sig(a[0] + pi * c)
            f_ = sig(a[1] + pf * c)
            c = f_ * c + i_ * math.tanh(a[2])
            h = sig(a[3] + po * c) * math.tanh(c)
            out.append(h)
        assert abs(hT[l, 0, 0] - h) < 1e-14 and abs(cT[l, 0, 0] - c) < 1e-14
        seq = out
    np.testing.assert_allclose(y[:, 0, 0], seq, rtol=0, atol=1e-14)


def test_peephole_closed_form_and_identities(oracle):
    rng = np.random.default_rng(32)
    I, H, T, B = 3, 4, 6, 2
    x = rng.standard_normal((T, B, I))
    c0 = rng.uniform(-1, 1, (1, B, H))
    # all W = 0, b = 0: only the peepholes drive the gates, g = tanh(0) = 0, so
    # c_t = sigma(p_f c_{t-1}) c_{t-1} and h_t = sigma(p_o c_t) tanh(c_t), whatever p_i is
    ws = [np.zeros((4 * H, I)), np.zeros((4 * H, H)), None, None]
    p = rng.uniform(-3, 3, (3, H))
    y, hT, cT = oracle.forward(LSTM, 1, 1, I, H, ws, x, c0=c0, peepholes=[p])
    c = c0[0].copy()
    for t in range(T):
        c = c / (1.0 + np.exp(-p[1] * c))
        np.testing.assert_allclose(y[t], np.tanh(c) / (1.0 + np.exp(-p[2] * c)), rtol=0, atol=1e-15)
    np.testing.assert_allclose(cT[0], c, rtol=0, atol=1e-15)
    # zero peepholes, a missing entry and "no peepholes" are the same network, bit for bit
    ws = rand_weights(rng, LSTM, 2, 2, I, H)
    ref = oracle.forward(LSTM, 2, 2, I, H, ws, x)
    for ps in ([np.zeros((3, H))] * 4, [None] * 4, [np.zeros((3, H)), None, None, np.zeros((3, H))]):
        got = oracle.forward(LSTM, 2, 2, I, H, ws, x, peepholes=ps)
        for a, b in zip(ref, got):
            assert np.array_equal(a, b)
    # each of the three weights matters, and only in its own layer and direction
    for k in range(3):
        q = np.zeros((3, H)); q[k] = 0.7
        got = oracle.forward(LSTM, 2, 2, I, H, ws, x, peepholes=[None, q, None, None])
        assert np.max(np.abs(got[1][1] - ref[1][1])) > 1e-4          # hT of (layer 0, backward) changes
        assert np.array_equal(got[1][0], ref[1][0])                  # (layer 0, forward) does not
    with pytest.raises(ValueError):
        oracle.forward(GRU, 1, 1, I, H, rand_weights(rng, GRU, 1, 1, I, H), x, peepholes=[np.zeros((3, H))])


def test_peephole_input_gate_per_unit(oracle):
    # f = 0 and o = 1 by bias, W_hh = 0, the i/f/o rows of W_ih zero: every unit j runs the scalar recursion
    # c_t = sigma(b_i[j] + p_i[j] c_{t-1}) tanh(W_g[j] x_t + b_g[j]),  h_t = tanh(c_t), with g far from zero,
    # so a p_i taken from another unit (or applied to another unit's c) changes the result
    rng = np.random.default_rng(35)
    I, H, T, B = 2, 4, 6, 2
    x = rng.standard_normal((T, B, I))
    wi = np.zeros((4 * H, I)); wi[2 * H:3 * H] = rng.uniform(-2, 2, (H, I))
    bi = np.zeros(4 * H)
    bi[0:H] = rng.uniform(-1, 1, H); bi[H:2 * H] = -40.0; bi[2 * H:3 * H] = rng.uniform(-1, 1, H); bi[3 * H:] = 40.0
    p = np.zeros((3, H)); p[0] = [2.5, -1.5, 0.75, -3.0]
    c0 = rng.uniform(-1, 1, (1, B, H))
    y, hT, cT = oracle.forward(LSTM, 1, 1, I, H, [wi, np.zeros((4 * H, H)), bi, None], x, c0=c0, peepholes=[p])
    for b in range(B):
        for j in range(H):
            c = float(c0[0, b, j])
            for t in range(T):
                g = math.tanh(sum(float(wi[2 * H + j, k]) * float(x[t, b, k]) for k in range(I)) + float(bi[2 * H + j]))
                c = sig(float(bi[j]) + float(p[0, j]) * c) * g
                assert abs(y[t, b, j] - math.tanh(c)) < 1e-14
            assert abs(cT[0, b, j] - c) < 1e-14
    # the units really differ: with p_i rotated by one unit the result moves
    q = p.copy(); q[0] = np.roll(p[0], 1)
    y2, _, _ = oracle.forward(LSTM, 1, 1, I, H, [wi, np.zeros((4 * H, H)), bi, None], x, c0=c0, peepholes=[q])
    assert np.max(np.abs(y2 - y)) > 1e-3


def test_peephole_all_gates_active_matrix_form(oracle):
    # every term alive, distinct weights per unit, 3 units, two directions: the cell written with
    # matrix-vector products over all units at once (a different routine from the oracle's scalar dots)
    rng = np.random.default_rng(36)
    I, H, T, B, D = 3, 3, 5, 2, 2
    ws = rand_weights(rng, LSTM, 1, D, I, H, scale=1.0)
    ps = [rng.uniform(-2, 2, (3, H)) for _ in range(D)]
    x = rng.standard_normal((T, B, I))
    h0 = rng.uniform(-1, 1, (D, B, H)); c0 = rng.uniform(-1, 1, (D, B, H))
    lengths = np.array([5, 3], dtype=np.int32)
    y, hT, cT = oracle.forward(LSTM, 1, D, I, H, ws, x, lengths, h0, c0, peepholes=ps)
    s = lambda v: 1.0 / (1.0 + np.exp(-v))
    for d in range(D):
        Wi, Wh, bi, bh = ws[4 * d:4 * d + 4]
        for b in range(B):
            n = int(lengths[b])
            h, c = h0[d, b].copy(), c0[d, b].copy()
            for t in (range(n) if d == 0 else range(n - 1, -1, -1)):
                a = Wi @ x[t, b] + bi + Wh @ h + bh
                i_ = s(a[:H] + ps[d][0] * c); f_ = s(a[H:2 * H] + ps[d][1] * c)
                c = f_ * c + i_ * np.tanh(a[2 * H:3 * H])
                h = s(a[3 * H:] + ps[d][2] * c) * np.tanh(c)
                np.testing.assert_allclose(y[t, b, d * H:(d + 1) * H], h, rtol=0, atol=1e-14)
            np.testing.assert_allclose(hT[d, b], h, rtol=0, atol=1e-14)
            np.testing.assert_allclose(cT[d, b], c, rtol=0, atol=1e-14)


def test_clip_scalar_recursion(oracle):
    rng = np.random.default_rng(33)
    T, clip = 6, 0.8
    x = 2 * rng.standard_normal((T, 1, 1))
    h0v, c0v = 0.4, 5.0      # f >= sigma(-clip) keeps the first new c above the threshold
    wi, wh = rng.uniform(-2, 2, (4, 1)), rng.uniform(-2, 2, (4, 1))
    bi, bh = rng.uniform(-1, 1, 4), rng.uniform(-1, 1, 4)
    p = rng.uniform(-2, 2, (3, 1))
    y, hT, cT = oracle.forward(LSTM, 1, 1, 1, 1, [wi, wh, bi, bh], x, h0=np.full((1, 1, 1), h0v),
                               c0=np.full((1, 1, 1), c0v), peepholes=[p], clip=clip)
    h, c = h0v, c0v
    hit, cmax = 0, 0.0
    for t in range(T):
        xv = float(x[t, 0, 0])
        a = [wi[g, 0] * xv + bi[g] + wh[g, 0] * h + bh[g] for g in range(4)]
        args = [a[0] + p[0, 0] * c, a[1] + p[1, 0] * c, a[2]]
        hit += sum(abs(v) > clip for v in args)
        c = sig(_clamp(args[1], clip)) * c + sig(_clamp(args[0], clip)) * math.tanh(_clamp(args[2], clip))
        h = sig(_clamp(a[3] + p[2, 0] * c, clip)) * math.tanh(c)     # the cell state inside tanh(c) is not clipped
        cmax = max(cmax, abs(c))
        assert abs(y[t, 0, 0] - h) < 1e-14
    assert hit >= 3 and cmax > clip          # the threshold was active, and a new c went beyond it
    assert abs(cT[0, 0, 0] - c) < 1e-14
    # GRU, both variants: r, z and the whole argument of n are clipped
    wi, wh = rng.uniform(-2, 2, (3, 1)), rng.uniform(-2, 2, (3, 1))
    bi, bh = rng.uniform(-1, 1, 3), rng.uniform(-1, 1, 3)
    for variant in (0, 1):
        y, hT, _ = oracle.forward(GRU, 1, 1, 1, 1, [wi, wh, bi, bh], x, h0=np.full((1, 1, 1), h0v),
                                  gru_variant=variant, clip=clip)
        h = h0v
        for t in range(T):
            xv = float(x[t, 0, 0])
            r = sig(_clamp(wi[0, 0] * xv + bi[0] + wh[0, 0] * h + bh[0], clip))
            z = sig(_clamp(wi[1, 0] * xv + bi[1] + wh[1, 0] * h + bh[1], clip))
            if variant == 0:
                n = math.tanh(_clamp(wi[2, 0] * xv + bi[2] + r * (wh[2, 0] * h + bh[2]), clip))
            else:
                n = math.tanh(_clamp(wi[2, 0] * xv + bi[2] + wh[2, 0] * (r * h) + bh[2], clip))
            h = (1 - z) * n + z * h
            assert abs(y[t, 0, 0] - h) < 1e-14


def test_clip_closed_forms_and_identities(oracle):
    rng = np.random.default_rng(34)
    I, H, T, B = 3, 5, 7, 2
    x = rng.standard_normal((T, B, I))
    # biases of +-40 on every gate and a threshold of 1: every gate sits at its clipped value,
    # i = f = o = sigma(1), g = tanh(1), so c_t = s c_{t-1} + s tanh(1), a geometric series
    s, g = sig(1.0), math.tanh(1.0)
    ws = [rng.uniform(-1, 1, (4 * H, I)), rng.uniform(-1, 1, (4 * H, H)), np.full(4 * H, 40.0), None]
    c0 = rng.uniform(-1, 1, (1, B, H))
    y, hT, cT = oracle.forward(LSTM, 1, 1, I, H, ws, x, c0=c0, clip=1.0)
    c = c0[0].copy()
    for t in range(T):
        c = s * c + s * g
        np.testing.assert_allclose(y[t], s * np.tanh(c), rtol=0, atol=1e-15)
    np.testing.assert_allclose(cT[0], s ** T * c0[0] + s * g * (1 - s ** T) / (1 - s), rtol=0, atol=1e-14)
    # the same with -40: i = f = o = sigma(-1), g = -tanh(1)
    ws[2] = np.full(4 * H, -40.0)
    s2 = sig(-1.0)
    y, hT, cT = oracle.forward(LSTM, 1, 1, I, H, ws, x, c0=c0, clip=1.0)
    np.testing.assert_allclose(cT[0], s2 ** T * c0[0] - s2 * g * (1 - s2 ** T) / (1 - s2), rtol=0, atol=1e-14)
    # GRU with +40 everywhere and threshold 1: z = sigma(1), n = tanh(1): h_t = (1 - z) n + z h_{t-1}
    wg = [rng.uniform(-1, 1, (3 * H, I)), rng.uniform(-1, 1, (3 * H, H)), np.full(3 * H, 40.0), None]
    h0 = rng.uniform(-1, 1, (1, B, H))
    for variant in (0, 1):
        y, hT, _ = oracle.forward(GRU, 1, 1, I, H, wg, x, h0=h0, gru_variant=variant, clip=1.0)
        np.testing.assert_allclose(hT[0], s ** T * h0[0] + (1 - s) * g * (1 - s ** T) / (1 - s), rtol=0, atol=1e-14)
    # a threshold beyond every argument changes nothing, bit for bit; a tight one does
    for cell in (LSTM, GRU):
        ws = rand_weights(rng, cell, 2, 2, I, H)
        ref = oracle.forward(cell, 2, 2, I, H, ws, x)
        same = oracle.forward(cell, 2, 2, I, H, ws, x, clip=1e6)
        tight = oracle.forward(cell, 2, 2, I, H, ws, x, clip=0.05)
        assert np.array_equal(ref[0], same[0]) and np.array_equal(ref[1], same[1])
        assert np.max(np.abs(ref[0] - tight[0])) > 1e-3
