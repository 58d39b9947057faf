"""Pins for the CPU oracle: each test fixes the oracle to something that is not the oracle.

The paper prints no LSTM equations and no worked example, so the pins are mathematical:
finite differences, closed forms, invariants, an independent library implementation
(torch.nn.LSTM on the CPU in float64) and a scalar case in 50-digit arithmetic.
"""
import numpy as np
import pytest
import torch

from oracle import lstm_oracle as O

RNG = np.random.default_rng(1805)


def rand_case(T=5, B=3, n_in=4, n=5, lens=None, scale=0.5, rng=RNG, D=1):
    lens = np.array([5, 0, 3] if lens is None else lens, dtype=np.int64)
    c = dict(
        x=rng.standard_normal((T, B, n_in)),
        W_x=rng.uniform(-scale, scale, (D, n_in, 4 * n)),
        W_h=rng.uniform(-scale, scale, (D, n, 4 * n)),
        b=rng.uniform(-scale, scale, (D, 4 * n)),
        h0=rng.standard_normal((D, B, n)) * 0.5,
        c0=rng.standard_normal((D, B, n)) * 0.5,
        lens=lens,
        dy=rng.standard_normal((T, B, D * n)),
        dhT=rng.standard_normal((D, B, n)),
        dcT=rng.standard_normal((D, B, n)),
    )
    return c


def loss(c, direction, **over):
    a = dict(c)
    a.update(over)
    y, cs, hT, cT = O.lstm_fwd(a["x"], a["W_x"][0], a["W_h"][0], a["b"][0], a["h0"][0], a["c0"][0], a["lens"], direction)
    return (c["dy"] * y).sum() + (c["dhT"][0] * hT).sum() + (c["dcT"][0] * cT).sum()


def grads(c, direction):
    return O.lstm_bwd(c["x"], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], c["lens"], direction,
                      c["dy"], c["dhT"][0], c["dcT"][0])


# ---- P1: finite differences -------------------------------------------------------------------
@pytest.mark.parametrize("direction", [1, -1])
def test_fd_all_coordinates_tiny(direction):
    c = rand_case()
    dx, dWx, dWh, db, dh0, dc0 = grads(c, direction)
    eps = 1e-5
    for name, g in (("x", dx), ("W_x", dWx[None]), ("W_h", dWh[None]), ("b", db[None]), ("h0", dh0[None]), ("c0", dc0[None])):
        base = c[name]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            p = base.copy(); p[idx] += eps
            m = base.copy(); m[idx] -= eps
            num[idx] = (loss(c, direction, **{name: p}) - loss(c, direction, **{name: m})) / (2 * eps)
        ana = g.reshape(base.shape)
        err = np.abs(num - ana).max() / max(np.abs(ana).max(), 1e-30)
        assert err < 1e-6, (name, err)
    # padded frames and the empty row get exactly zero input gradient
    assert (dx[3:, 2] == 0).all() and (dx[:, 1] == 0).all()


def test_fd_random_coordinates_config1_shape():
    rng = np.random.default_rng(7)
    c = rand_case(T=20, B=4, n_in=32, n=64, lens=[20, 20, 20, 20], scale=0.1, rng=rng)
    g = dict(zip(("x", "W_x", "W_h", "b", "h0", "c0"), grads(c, 1)))
    eps = 1e-5
    worst = 0.0
    for name in g:
        base = c[name]
        ana = g[name].reshape(base.shape)
        scale = np.abs(ana).max()
        for _ in range(90):
            idx = tuple(rng.integers(0, s) for s in base.shape)
            p = base.copy(); p[idx] += eps
            m = base.copy(); m[idx] -= eps
            num = (loss(c, 1, **{name: p}) - loss(c, 1, **{name: m})) / (2 * eps)
            worst = max(worst, abs(num - ana[idx]) / scale)
    assert worst < 1e-6, worst


# ---- P2 / P3: closed forms with zero weights ---------------------------------------------------
def test_zero_weight_closed_form():
    T, B, n_in, n = 7, 3, 4, 6
    lens = np.array([7, 4, 0])
    c0 = RNG.standard_normal((B, n))
    x = RNG.standard_normal((T, B, n_in))
    y, cs, hT, cT = O.lstm_fwd(x, np.zeros((n_in, 4 * n)), np.zeros((n, 4 * n)), None, None, c0, lens, 1)
    for b in range(B):
        for t in range(T):
            if t < lens[b]:
                ck = c0[b] * 0.5 ** (t + 1)
                np.testing.assert_allclose(cs[t, b], ck, rtol=1e-14)
                np.testing.assert_allclose(y[t, b], 0.5 * np.tanh(ck), rtol=1e-14)
            else:
                assert (y[t, b] == 0).all()
        np.testing.assert_allclose(cT[b], c0[b] * 0.5 ** lens[b], rtol=1e-14)
    y0 = O.lstm_fwd(x, np.zeros((n_in, 4 * n)), np.zeros((n, 4 * n)), None, None, None, lens, -1)[0]
    assert (y0 == 0).all()


@pytest.mark.parametrize("direction", [1, -1])
def test_constant_gate_closed_form(direction):
    T, B, n_in, n = 9, 2, 3, 4
    lens = np.array([9, 5])
    bias = np.concatenate([np.full(n, 0.3), np.full(n, -0.7), np.full(n, 1.1), np.full(n, 0.2)]) + 0.01 * np.arange(4 * n)
    sig = lambda u: 1 / (1 + np.exp(-u))
    ib, fb, gb, ob = sig(bias[:n]), sig(bias[n:2 * n]), np.tanh(bias[2 * n:3 * n]), sig(bias[3 * n:])
    c0 = RNG.standard_normal((B, n))
    x = RNG.standard_normal((T, B, n_in))
    W_x0 = np.zeros((n_in, 4 * n))
    y, cs, hT, cT = O.lstm_fwd(x, W_x0, np.zeros((n, 4 * n)), bias, None, c0, lens, direction)
    for b in range(B):
        k = lens[b]
        ck = fb ** k * c0[b] + ib * gb * (1 - fb ** k) / (1 - fb)     # geometric series
        np.testing.assert_allclose(cT[b], ck, rtol=1e-13)
        np.testing.assert_allclose(hT[b], ob * np.tanh(ck), rtol=1e-13)
        # the j-th processed frame holds the j-step value, whatever x is
        for j in range(1, k + 1):
            t = j - 1 if direction == 1 else k - j
            cj = fb ** j * c0[b] + ib * gb * (1 - fb ** j) / (1 - fb)
            np.testing.assert_allclose(cs[t, b], cj, rtol=1e-13)
    # backward: W_h = 0, W_x = 0 => dx = 0 and dW_x = X^T DZ with DZ from a scalar recursion
    dy = RNG.standard_normal((T, B, n))
    dx, dWx, dWh, db, dh0, dc0 = O.lstm_bwd(x, W_x0, np.zeros((n, 4 * n)), bias, None, c0, lens, direction, dy)
    assert (dx == 0).all()
    assert (dh0 == 0).all()                                     # W_h = 0: nothing flows into h0
    DZ = np.zeros((T, B, 4 * n))
    for b in range(B):
        k = lens[b]
        Dc = np.zeros(n)
        for j in range(k, 0, -1):
            t = j - 1 if direction == 1 else k - j
            cj = fb ** j * c0[b] + ib * gb * (1 - fb ** j) / (1 - fb)
            cjm = fb ** (j - 1) * c0[b] + ib * gb * (1 - fb ** (j - 1)) / (1 - fb)
            tc = np.tanh(cj)
            dc = Dc + dy[t, b] * ob * (1 - tc ** 2)
            DZ[t, b] = np.concatenate([dc * gb * ib * (1 - ib), dc * cjm * fb * (1 - fb), dc * ib * (1 - gb ** 2),
                                       dy[t, b] * tc * ob * (1 - ob)])
            Dc = dc * fb
        np.testing.assert_allclose(dc0[b], Dc, rtol=1e-12)
    np.testing.assert_allclose(dWx, np.einsum("tbi,tbj->ij", x, DZ), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(db, DZ.sum((0, 1)), rtol=1e-11)


# ---- P4: padding invariance, NaN padding ---------------------------------------------------------
@pytest.mark.parametrize("direction", [1, -1])
def test_padding_invariance_nan(direction):
    c = rand_case(T=6, B=3, lens=[4, 0, 2])
    k = 3
    ref_f = O.lstm_fwd(c["x"][:4], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], c["lens"], direction)
    ref_b = O.lstm_bwd(c["x"][:4], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], c["lens"], direction,
                       c["dy"][:4], c["dhT"][0], c["dcT"][0])
    xp = np.full((4 + k, 3, 4), np.nan); dyp = np.full((4 + k, 3, 5), np.nan)
    for b, L in enumerate(c["lens"]):
        xp[:L, b] = c["x"][:L, b]; dyp[:L, b] = c["dy"][:L, b]
    got_f = O.lstm_fwd(xp, c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], c["lens"], direction)
    got_b = O.lstm_bwd(xp, c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], c["lens"], direction,
                       dyp, c["dhT"][0], c["dcT"][0])
    for b, L in enumerate(c["lens"]):
        assert np.array_equal(got_f[0][:L, b], ref_f[0][:L, b])
        assert (got_f[0][L:, b] == 0).all()
        assert (got_b[0][L:, b] == 0).all()
        # stored cell state at padded frames is the carried one: final state (+1) or c0 (-1)
        carried = got_f[3][b] if direction == 1 else c["c0"][0][b]
        assert (got_f[1][L:, b] == carried).all()
        assert np.array_equal(got_b[0][:L, b], ref_b[0][:L, b])
    assert np.array_equal(got_f[2], ref_f[2]) and np.array_equal(got_f[3], ref_f[3])
    for a, r in zip(got_b[1:], ref_b[1:]):
        assert np.array_equal(a, r)
    # empty row: state and incoming gradient pass straight through
    assert np.array_equal(got_f[2][1], c["h0"][0][1]) and np.array_equal(got_b[4][1], c["dhT"][0][1])
    assert np.array_equal(got_f[3][1], c["c0"][0][1]) and np.array_equal(got_b[5][1], c["dcT"][0][1])


# ---- P5: batch independence ----------------------------------------------------------------------
@pytest.mark.parametrize("direction", [1, -1])
def test_batch_independence(direction):
    c = rand_case(T=6, B=4, lens=[6, 2, 5, 1])
    full_f = O.lstm_fwd(c["x"], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], c["lens"], direction)
    full_b = grads(c, direction)
    sW = [np.zeros_like(full_b[1]), np.zeros_like(full_b[2]), np.zeros_like(full_b[3])]
    for r in range(4):
        s = slice(r, r + 1)
        f = O.lstm_fwd(c["x"][:, s], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0][s], c["c0"][0][s], c["lens"][s], direction)
        g = O.lstm_bwd(c["x"][:, s], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0][s], c["c0"][0][s], c["lens"][s],
                       direction, c["dy"][:, s], c["dhT"][0][s], c["dcT"][0][s])
        np.testing.assert_allclose(f[0][:, 0], full_f[0][:, r], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(f[1][:, 0], full_f[1][:, r], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(g[0][:, 0], full_b[0][:, r], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(g[4][0], full_b[4][r], rtol=1e-12, atol=1e-14)
        for k in range(3):
            sW[k] += g[1 + k]
    for k in range(3):
        np.testing.assert_allclose(sW[k], full_b[1 + k], rtol=1e-11, atol=1e-13)
    perm = np.array([2, 0, 3, 1])
    pf = O.lstm_fwd(c["x"][:, perm], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0][perm], c["c0"][0][perm], c["lens"][perm], direction)
    np.testing.assert_allclose(pf[0], full_f[0][:, perm], rtol=1e-13, atol=1e-15)


# ---- P6: reversal identity -----------------------------------------------------------------------
def _rev_prefix(a, lens):
    out = a.copy()
    for b, L in enumerate(lens):
        out[:L, b] = a[:L, b][::-1]
    return out


def test_reversal_identity():
    c = rand_case(T=7, B=4, lens=[7, 3, 0, 5])
    args = (c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], c["lens"])
    yb, csb, hTb, cTb = O.lstm_fwd(c["x"], *args, -1)
    yf, csf, hTf, cTf = O.lstm_fwd(_rev_prefix(c["x"], c["lens"]), *args, 1)
    np.testing.assert_allclose(yb, _rev_prefix(yf, c["lens"]), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(hTb, hTf, rtol=1e-13); np.testing.assert_allclose(cTb, cTf, rtol=1e-13)
    gb = O.lstm_bwd(c["x"], *args, -1, c["dy"], c["dhT"][0], c["dcT"][0])
    gf = O.lstm_bwd(_rev_prefix(c["x"], c["lens"]), *args, 1, _rev_prefix(c["dy"], c["lens"]), c["dhT"][0], c["dcT"][0])
    np.testing.assert_allclose(gb[0], _rev_prefix(gf[0], c["lens"]), rtol=1e-12, atol=1e-14)
    for a, r in zip(gb[1:], gf[1:]):
        np.testing.assert_allclose(a, r, rtol=1e-12, atol=1e-14)


# ---- P7: BLSTM composition -----------------------------------------------------------------------
def test_blstm_composition():
    c = rand_case(T=6, B=3, lens=[6, 0, 4], D=2)
    n = 5
    y, cs, hT, cT = O.blstm_fwd(c["x"], c["W_x"], c["W_h"], c["b"], c["h0"], c["c0"], c["lens"])
    g = O.blstm_bwd(c["x"], c["W_x"], c["W_h"], c["b"], c["h0"], c["c0"], c["lens"], c["dy"], c["dhT"], c["dcT"])
    dx_sum = 0
    for d, direction in enumerate((1, -1)):
        f1 = O.lstm_fwd(c["x"], c["W_x"][d], c["W_h"][d], c["b"][d], c["h0"][d], c["c0"][d], c["lens"], direction)
        assert np.array_equal(y[:, :, d * n:(d + 1) * n], f1[0]) and np.array_equal(cs[d], f1[1])
        assert np.array_equal(hT[d], f1[2]) and np.array_equal(cT[d], f1[3])
        g1 = O.lstm_bwd(c["x"], c["W_x"][d], c["W_h"][d], c["b"][d], c["h0"][d], c["c0"][d], c["lens"], direction,
                        c["dy"][:, :, d * n:(d + 1) * n], c["dhT"][d], c["dcT"][d])
        dx_sum = dx_sum + g1[0]
        for k in range(1, 6):
            assert np.array_equal(g[k][d], g1[k])
    np.testing.assert_allclose(g[0], dx_sum, rtol=1e-14)
    # and the whole thing against finite differences through both directions at once
    def L(x):
        yy, _, h, cc = O.blstm_fwd(x, c["W_x"], c["W_h"], c["b"], c["h0"], c["c0"], c["lens"])
        return (c["dy"] * yy).sum() + (c["dhT"] * h).sum() + (c["dcT"] * cc).sum()
    eps = 1e-5
    for idx in [(0, 0, 1), (3, 2, 0), (5, 0, 3), (4, 2, 2), (2, 1, 1)]:
        p = c["x"].copy(); p[idx] += eps
        m = c["x"].copy(); m[idx] -= eps
        assert abs((L(p) - L(m)) / (2 * eps) - g[0][idx]) < 1e-7 * max(1, np.abs(g[0]).max())


# ---- P8: time splitting and stepping ---------------------------------------------------------------
def test_time_splitting_and_stepping():
    c = rand_case(T=8, B=3, lens=[8, 8, 8])
    W = (c["W_x"][0], c["W_h"][0], c["b"][0])
    y, cs, hT, cT = O.lstm_fwd(c["x"], *W, c["h0"][0], c["c0"][0], c["lens"], 1)
    h, cc = c["h0"][0], c["c0"][0]
    ys = []
    for t in range(8):                                         # T calls with T = 1 (decoder stepping)
        y1, _, h, cc = O.lstm_fwd(c["x"][t:t + 1], *W, h, cc, None, 1)
        ys.append(y1[0])
    np.testing.assert_allclose(np.stack(ys), y, rtol=1e-14)
    np.testing.assert_allclose(h, hT, rtol=1e-14); np.testing.assert_allclose(cc, cT, rtol=1e-14)
    # two chunks forward, chained backward through dhT/dcT
    T1 = 3
    ya, _, ha, ca = O.lstm_fwd(c["x"][:T1], *W, c["h0"][0], c["c0"][0], None, 1)
    g2 = O.lstm_bwd(c["x"][T1:], *W, ha, ca, None, 1, c["dy"][T1:], c["dhT"][0], c["dcT"][0])
    g1 = O.lstm_bwd(c["x"][:T1], *W, c["h0"][0], c["c0"][0], None, 1, c["dy"][:T1], g2[4], g2[5])
    gf = grads(c, 1)
    np.testing.assert_allclose(np.concatenate([g1[0], g2[0]]), gf[0], rtol=1e-12, atol=1e-14)
    for k in (1, 2, 3):
        np.testing.assert_allclose(g1[k] + g2[k], gf[k], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g1[4], gf[4], rtol=1e-12); np.testing.assert_allclose(g1[5], gf[5], rtol=1e-12)


# ---- P9: scalar case in 50-digit arithmetic --------------------------------------------------------
def test_scalar_case_high_precision():
    import mpmath as mp
    mp.mp.dps = 50
    with open(__file__.rsplit("/", 1)[0] + "/golden/scalar_case.txt") as fh:
        vals = {}
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = mp.mpf(v)
    wx, wh = [vals[f"wx_{q}"] for q in "ifgo"], [vals[f"wh_{q}"] for q in "ifgo"]
    bb = [vals[f"b_{q}"] for q in "ifgo"]
    xs = [vals["x0"], vals["x1"]]
    h, c = vals["h0"], vals["c0"]
    sg = lambda u: 1 / (1 + mp.e ** (-u))
    for xt in xs:                                              # two steps of the scalar cell, n = n_in = B = 1
        zi, zf, zg, zo = (xt * wx[q] + h * wh[q] + bb[q] for q in range(4))
        c = sg(zf) * c + sg(zi) * mp.tanh(zg)
        h = sg(zo) * mp.tanh(c)
    f = lambda k: np.array(float(vals[k]))
    y, cs, hT, cT = O.lstm_fwd(np.array([f("x0"), f("x1")]).reshape(2, 1, 1),
                               np.array([float(v) for v in wx]).reshape(1, 4), np.array([float(v) for v in wh]).reshape(1, 4),
                               np.array([float(v) for v in bb]), f("h0").reshape(1, 1), f("c0").reshape(1, 1), None, 1)
    assert abs(hT[0, 0] - float(h)) < 1e-15 and abs(cT[0, 0] - float(c)) < 1e-15
    assert abs(y[1, 0, 0] - float(h)) < 1e-15


# ---- P10: hoisting the input projection is exact ---------------------------------------------------
def test_hoisting_is_exact():
    c = rand_case(T=6, B=3, lens=[6, 6, 6])
    y, cs, hT, cT = O.lstm_fwd(c["x"], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], None, 1)
    Zx = c["x"].reshape(-1, 4) @ c["W_x"][0] + c["b"][0]      # all time steps at once (Sec. 3: moved out of the loop)
    Zx = Zx.reshape(6, 3, 20)
    # feed Zx through an identity input projection with zero bias
    y2, cs2, hT2, cT2 = O.lstm_fwd(Zx, np.eye(20), c["W_h"][0], None, c["h0"][0], c["c0"][0], None, 1)
    np.testing.assert_allclose(y2, y, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(cT2, cT, rtol=1e-13)


# ---- P11: independent library implementation ---------------------------------------------------------
def test_against_torch_nn_lstm_bidirectional():
    T, B, n_in, n = 9, 5, 6, 7
    rng = np.random.default_rng(11)
    c = rand_case(T=T, B=B, n_in=n_in, n=n, lens=[9, 4, 1, 7, 9], rng=rng, D=2)
    m = torch.nn.LSTM(n_in, n, bidirectional=True).double()
    with torch.no_grad():
        for d, suf in enumerate(("", "_reverse")):
            getattr(m, "weight_ih_l0" + suf).copy_(torch.from_numpy(c["W_x"][d].T.copy()))
            getattr(m, "weight_hh_l0" + suf).copy_(torch.from_numpy(c["W_h"][d].T.copy()))
            getattr(m, "bias_ih_l0" + suf).copy_(torch.from_numpy(c["b"][d]))
            getattr(m, "bias_hh_l0" + suf).zero_()
    x = torch.from_numpy(c["x"]).requires_grad_(True)
    h0 = torch.from_numpy(c["h0"]).requires_grad_(True)
    c0 = torch.from_numpy(c["c0"]).requires_grad_(True)
    packed = torch.nn.utils.rnn.pack_padded_sequence(x, torch.from_numpy(c["lens"]), enforce_sorted=False)
    out, (hn, cn) = m(packed, (h0, c0))
    yt, _ = torch.nn.utils.rnn.pad_packed_sequence(out, total_length=T)
    L = (torch.from_numpy(c["dy"]) * yt).sum() + (torch.from_numpy(c["dhT"]) * hn).sum() + (torch.from_numpy(c["dcT"]) * cn).sum()
    L.backward()
    y, cs, hT, cT = O.blstm_fwd(c["x"], c["W_x"], c["W_h"], c["b"], c["h0"], c["c0"], c["lens"])
    g = O.blstm_bwd(c["x"], c["W_x"], c["W_h"], c["b"], c["h0"], c["c0"], c["lens"], c["dy"], c["dhT"], c["dcT"])
    tol = dict(rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(y, yt.detach().numpy(), **tol)
    np.testing.assert_allclose(hT, hn.detach().numpy(), **tol)
    np.testing.assert_allclose(cT, cn.detach().numpy(), **tol)
    np.testing.assert_allclose(g[0], x.grad.numpy(), **tol)
    for d, suf in enumerate(("", "_reverse")):
        np.testing.assert_allclose(g[1][d], getattr(m, "weight_ih_l0" + suf).grad.numpy().T, **tol)
        np.testing.assert_allclose(g[2][d], getattr(m, "weight_hh_l0" + suf).grad.numpy().T, **tol)
        np.testing.assert_allclose(g[3][d], getattr(m, "bias_ih_l0" + suf).grad.numpy(), **tol)
    np.testing.assert_allclose(g[4], h0.grad.numpy(), **tol)
    np.testing.assert_allclose(g[5], c0.grad.numpy(), **tol)


def test_cell_states_against_torch_lstmcell():
    T, B, n_in, n = 5, 3, 4, 6
    c = rand_case(T=T, B=B, n_in=n_in, n=n, lens=[5, 5, 5], rng=np.random.default_rng(3))
    cell = torch.nn.LSTMCell(n_in, n).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(c["W_x"][0].T.copy())); cell.weight_hh.copy_(torch.from_numpy(c["W_h"][0].T.copy()))
        cell.bias_ih.copy_(torch.from_numpy(c["b"][0])); cell.bias_hh.zero_()
        h, cc = torch.from_numpy(c["h0"][0]), torch.from_numpy(c["c0"][0])
        y, cs, _, _ = O.lstm_fwd(c["x"], c["W_x"][0], c["W_h"][0], c["b"][0], c["h0"][0], c["c0"][0], None, 1)
        for t in range(T):
            h, cc = cell(torch.from_numpy(c["x"][t]), (h, cc))
            np.testing.assert_allclose(cs[t], cc.numpy(), rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(y[t], h.numpy(), rtol=1e-12, atol=1e-13)


# ---- P12: W_h = 0 degenerates to a frame-wise formula --------------------------------------------------
def test_zero_recurrent_weight_first_frame():
    c = rand_case(T=4, B=3, lens=[4, 4, 4])
    W_h0 = np.zeros_like(c["W_h"][0])
    y, cs, _, _ = O.lstm_fwd(c["x"], c["W_x"][0], W_h0, c["b"][0], c["h0"][0], None, None, 1)
    sig = lambda u: 1 / (1 + np.exp(-u))
    z = np.einsum("tbi,ij->tbj", c["x"], c["W_x"][0]) + c["b"][0]
    i, f, g, o = sig(z[..., :5]), sig(z[..., 5:10]), np.tanh(z[..., 10:15]), sig(z[..., 15:])
    cc = np.zeros((3, 5))
    for t in range(4):                                          # only c recurs; every gate is frame-wise
        cc = f[t] * cc + i[t] * g[t]
        np.testing.assert_allclose(cs[t], cc, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(y[t], o[t] * np.tanh(cc), rtol=1e-13, atol=1e-15)


# ---- stacks ----------------------------------------------------------------------------------------------
def test_stack_matches_manual_chain_and_fd():
    rng = np.random.default_rng(5)
    T, B, n_in, n = 5, 2, 3, 4
    lens = np.array([5, 3])
    layers = [dict(W_x=rng.uniform(-.5, .5, (2, n_in if l == 0 else 2 * n, 4 * n)), W_h=rng.uniform(-.5, .5, (2, n, 4 * n)),
                   b=rng.uniform(-.5, .5, (2, 4 * n))) for l in range(2)]
    x = rng.standard_normal((T, B, n_in)); dy = rng.standard_normal((T, B, 2 * n))
    acts, y = O.blstm_stack_fwd(x, layers, lens)
    dx, grads_ = O.blstm_stack_bwd(acts, layers, lens, dy)
    def L(xx=x, ll=layers):
        return (O.blstm_stack_fwd(xx, ll, lens)[1] * dy).sum()
    eps = 1e-5
    for idx in [(0, 0, 0), (4, 0, 2), (2, 1, 1), (4, 1, 0)]:
        p = x.copy(); p[idx] += eps; m = x.copy(); m[idx] -= eps
        assert abs((L(p) - L(m)) / (2 * eps) - dx[idx]) < 1e-7 * max(1.0, np.abs(dx).max())
    for (l, key, gi, idx) in [(0, "W_x", 0, (1, 2, 5)), (0, "W_h", 1, (0, 3, 9)), (1, "W_x", 0, (1, 7, 15)), (1, "b", 2, (0, 6))]:
        def pert(s):
            ll = [dict(d) for d in layers]; a = ll[l][key].copy(); a[idx] += s; ll[l][key] = a; return ll
        num = (L(ll=pert(eps)) - L(ll=pert(-eps))) / (2 * eps)
        assert abs(num - grads_[l][gi][idx]) < 1e-7 * max(1.0, np.abs(grads_[l][gi]).max())


def _mixed_layers(rng, n_in, n, n_uni):
    layers = [dict(W_x=rng.uniform(-.5, .5, (2, n_in, 4 * n)), W_h=rng.uniform(-.5, .5, (2, n, 4 * n)), b=rng.uniform(-.5, .5, (2, 4 * n)))]
    for l in range(n_uni):
        layers.append(dict(W_x=rng.uniform(-.5, .5, (1, 2 * n if l == 0 else n, 4 * n)), W_h=rng.uniform(-.5, .5, (1, n, 4 * n)),
                           b=rng.uniform(-.5, .5, (1, 4 * n))))
    return layers


def test_mixed_stack_against_torch_modules():
    """One bidirectional layer below two unidirectional ones (Sec. 3, caption of Table 1, the training-speed table) against
    torch.nn.LSTM modules chained over packed sequences: outputs and every gradient."""
    rng = np.random.default_rng(21)
    T, B, n_in, n = 7, 4, 3, 5
    lens = np.array([7, 2, 5, 1])
    layers = _mixed_layers(rng, n_in, n, 2)
    x = rng.standard_normal((T, B, n_in)); dy = rng.standard_normal((T, B, n))
    acts, y = O.encoder_stack_fwd(x, layers, lens)
    dx, grads_ = O.encoder_stack_bwd(acts, layers, lens, dy)
    assert y.shape == (T, B, n) and acts[1].shape == (T, B, 2 * n) and acts[2].shape == (T, B, n)
    mods = [torch.nn.LSTM(n_in, n, bidirectional=True).double(), torch.nn.LSTM(2 * n, n).double(), torch.nn.LSTM(n, n).double()]
    with torch.no_grad():
        for m, L in zip(mods, layers):
            for d, suf in enumerate(("", "_reverse")[:L["W_x"].shape[0]]):
                getattr(m, "weight_ih_l0" + suf).copy_(torch.from_numpy(L["W_x"][d].T.copy()))
                getattr(m, "weight_hh_l0" + suf).copy_(torch.from_numpy(L["W_h"][d].T.copy()))
                getattr(m, "bias_ih_l0" + suf).copy_(torch.from_numpy(L["b"][d]))
                getattr(m, "bias_hh_l0" + suf).zero_()
    xt = torch.from_numpy(x).requires_grad_(True)
    cur = torch.nn.utils.rnn.pack_padded_sequence(xt, torch.from_numpy(lens), enforce_sorted=False)
    for m in mods:
        cur, _ = m(cur)
    yt, _ = torch.nn.utils.rnn.pad_packed_sequence(cur, total_length=T)
    (torch.from_numpy(dy) * yt).sum().backward()
    tol = dict(rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(y, yt.detach().numpy(), **tol)
    np.testing.assert_allclose(dx, xt.grad.numpy(), **tol)
    for m, L, g in zip(mods, layers, grads_):
        assert g[0].shape == L["W_x"].shape and g[1].shape == L["W_h"].shape and g[2].shape == L["b"].shape
        for d, suf in enumerate(("", "_reverse")[:L["W_x"].shape[0]]):
            np.testing.assert_allclose(g[0][d], getattr(m, "weight_ih_l0" + suf).grad.numpy().T, **tol)
            np.testing.assert_allclose(g[1][d], getattr(m, "weight_hh_l0" + suf).grad.numpy().T, **tol)
            np.testing.assert_allclose(g[2][d], getattr(m, "bias_ih_l0" + suf).grad.numpy(), **tol)


def test_mixed_stack_reduces_to_its_parts_and_fd():
    """An all-bidirectional list gives the bidirectional stack; a unidirectional layer on top never looks ahead
    (its output at frame t does not change when later frames of its input change); central differences."""
    rng = np.random.default_rng(22)
    T, B, n_in, n = 6, 3, 3, 4
    lens = np.array([6, 4, 0])
    bl = [dict(W_x=rng.uniform(-.5, .5, (2, n_in if l == 0 else 2 * n, 4 * n)), W_h=rng.uniform(-.5, .5, (2, n, 4 * n)),
               b=rng.uniform(-.5, .5, (2, 4 * n))) for l in range(2)]
    x = rng.standard_normal((T, B, n_in))
    np.testing.assert_array_equal(O.encoder_stack_fwd(x, bl, lens)[1], O.blstm_stack_fwd(x, bl, lens)[1])
    layers = _mixed_layers(rng, n_in, n, 3)
    dy = rng.standard_normal((T, B, n))
    acts, y = O.encoder_stack_fwd(x, layers, lens)
    top_in = acts[-1].copy(); top_in[4:] += 1.0                 # change the last layer's input from frame 4 on
    y2 = O.lstm_fwd(top_in, layers[-1]["W_x"][0], layers[-1]["W_h"][0], layers[-1]["b"][0], None, None, lens, direction=1)[0]
    np.testing.assert_array_equal(y2[:4], y[:4])
    assert np.abs(y2[4:, 0] - y[4:, 0]).max() > 1e-3
    dx, grads_ = O.encoder_stack_bwd(acts, layers, lens, dy)
    assert np.all(dx[:, 2] == 0) and np.all(dx[4:, 1] == 0)
    def L(xx=x, ll=layers):
        return (O.encoder_stack_fwd(xx, ll, lens)[1] * dy).sum()
    eps = 1e-5
    for idx in [(0, 0, 0), (5, 0, 2), (3, 1, 1)]:
        p = x.copy(); p[idx] += eps; m = x.copy(); m[idx] -= eps
        assert abs((L(p) - L(m)) / (2 * eps) - dx[idx]) < 1e-7 * max(1.0, np.abs(dx).max())
    for (l, key, gi, idx) in [(0, "W_x", 0, (1, 2, 5)), (1, "W_x", 0, (0, 7, 3)), (2, "W_h", 1, (0, 3, 9)), (3, "b", 2, (0, 6)), (3, "W_x", 0, (0, 1, 15))]:
        def pert(s):
            ll = [dict(d) for d in layers]; a = ll[l][key].copy(); a[idx] += s; ll[l][key] = a; return ll
        num = (L(ll=pert(eps)) - L(ll=pert(-eps))) / (2 * eps)
        assert abs(num - grads_[l][gi][idx]) < 1e-7 * max(1.0, np.abs(grads_[l][gi]).max())


# ---- max-pooling in time (the speech encoder's pooling between layers) -----------------------------------------
def _pool_case(T=9, B=4, F=6, lens=(9, 4, 0, 7), seed=5):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((T, B, F)), np.array(lens, dtype=np.int64)


def test_maxpool_hand_worked_example():
    """tests/golden/maxpool_case.txt: a case small enough to do by hand, ties and short last windows included."""
    import os
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "maxpool_case.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = v
    T, B, pool = int(vals["T"][0]), int(vals["T"][2]), int(vals["T"][4])
    lens = np.array(vals["lens"], dtype=np.int64)
    row_major = lambda k, n: np.array(vals[k], dtype=np.float64).reshape(B, n).T[:, :, None]     # file lists row after row
    y, out_ref, dout, dy_ref = row_major("y", T), row_major("out", 3), row_major("dout", 3), row_major("dy", T)
    out, lens_out, arg = O.time_maxpool_fwd(y, lens, pool)
    assert np.array_equal(out, out_ref)
    assert np.array_equal(lens_out, np.array(vals["lens_out"], dtype=np.int64))
    assert np.array_equal(arg[:, :, 0].T.reshape(-1), np.array(vals["arg"], dtype=np.int64))
    assert np.array_equal(O.time_maxpool_bwd(dout, arg, lens, pool, T), dy_ref)


@pytest.mark.parametrize("pool", [2, 3])
def test_maxpool_against_torch_on_full_length_rows(pool):
    """An independent library: torch max_pool1d with ceil_mode on rows without padding, forward and gradient."""
    T, B, F = 11, 3, 4
    y, _ = _pool_case(T, B, F, (T,) * B)
    out, lens_out, arg = O.time_maxpool_fwd(y, None, pool)
    yt = torch.tensor(y, dtype=torch.float64).permute(1, 2, 0).clone().requires_grad_(True)      # [B, F, T]
    ot = torch.nn.functional.max_pool1d(yt, pool, pool, ceil_mode=True)
    assert np.array_equal(out, ot.detach().permute(2, 0, 1).numpy())
    assert np.all(lens_out == -(-T // pool))
    dout = np.random.default_rng(3).standard_normal(out.shape)
    ot.backward(torch.tensor(dout).permute(1, 2, 0))
    assert np.array_equal(O.time_maxpool_bwd(dout, arg, None, pool, T), yt.grad.permute(2, 0, 1).numpy())


def test_maxpool_brute_force_padding_and_identities():
    y, lens = _pool_case()
    T, B, F = y.shape
    for pool in (1, 2, 4):
        out, lens_out, arg = O.time_maxpool_fwd(y, lens, pool)
        # brute force, element by element, straight from the definition
        for b in range(B):
            assert lens_out[b] == -(-lens[b] // pool)
            for tp in range(out.shape[0]):
                for f in range(F):
                    window = [y[t, b, f] for t in range(pool * tp, min(pool * tp + pool, lens[b]))]
                    assert out[tp, b, f] == (max(window) if window else 0.0)
                    if window:
                        assert arg[tp, b, f] == window.index(max(window))        # list.index: the earliest maximum
        # padded frames are never read
        ynan = y.copy()
        for b in range(B):
            ynan[lens[b]:, b, :] = np.nan
        out2, _, arg2 = O.time_maxpool_fwd(ynan, lens, pool)
        assert np.array_equal(out, out2) and np.array_equal(arg, arg2)
        # the gradient is moved, not changed: same sum, one non-zero per window and feature, nothing at padded frames
        dout = np.random.default_rng(9).standard_normal(out.shape)
        dy = O.time_maxpool_bwd(dout, arg, lens, pool, T)
        valid = np.arange(out.shape[0])[:, None] < lens_out[None, :]
        assert np.isclose(dy.sum(), (dout * valid[:, :, None]).sum())
        assert np.count_nonzero(dy) == int(valid.sum()) * F
        for b in range(B):
            assert not dy[lens[b]:, b, :].any()
        if pool == 1:                                           # windows of one frame: the identity on valid frames
            mask = (np.arange(T)[:, None] < lens[None, :])[:, :, None]
            assert np.array_equal(out, y * mask) and np.array_equal(dy, dout * mask)


def test_maxpool_gradient_is_the_derivative():
    """Central differences of L = sum(dout * out) away from ties."""
    y, lens = _pool_case(T=6, B=2, F=3, lens=(6, 5), seed=11)
    pool = 2
    out, _, arg = O.time_maxpool_fwd(y, lens, pool)
    dout = np.random.default_rng(4).standard_normal(out.shape)
    dy = O.time_maxpool_bwd(dout, arg, lens, pool, y.shape[0])
    eps = 1e-6
    for idx in [(0, 0, 0), (1, 0, 2), (4, 1, 1), (5, 0, 0), (3, 1, 2)]:
        yp, ym = y.copy(), y.copy()
        yp[idx] += eps
        ym[idx] -= eps
        num = ((O.time_maxpool_fwd(yp, lens, pool)[0] - O.time_maxpool_fwd(ym, lens, pool)[0]) * dout).sum() / (2 * eps)
        assert abs(num - dy[idx]) < 1e-8
