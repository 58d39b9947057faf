"""CPU oracle for the masked, variable-length LSTM / BLSTM layer, forward and backward.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it.  It shares nothing with the HIP path and never
imports it.  All arithmetic is numpy float64; the only library primitives used as steps are
`@` (matrix product), `np.exp` and `np.tanh`.

What it computes.  The paper (Sec. 3 "Speed comparison", Sec. 7 "features", Listing 1) names
its native LSTM layer (`unit: nativelstm2`, `direction: +1 / -1`, two such layers on the same
input concatenated into one bidirectional layer, stepped `rnn_cell` LSTM in the decoder) and
states that the input projection can be moved out of the recurrent loop, but prints no cell
equations.  The definition below is therefore the textbook peephole-free LSTM, with these
readings (all are conventions of this repository, none is the paper's):

  * gate blocks along the 4n axis are ordered  i | f | g | o ;
  * one bias vector b[4n], no forget-gate offset;
  * a frame t of row b is *valid* iff t < seq_lens[b].  At a padded frame the state (h, c) is
    carried unchanged, the output y is zero, the stored cell state is the carried c, and the
    frame contributes no gradient.  Values stored in x or dy at padded frames are never read;
  * direction -1 walks t = T-1 .. 0 over the same end-padded tensors, so padded frames are met
    first and skipped with the state still at (h0, c0);
  * hT, cT are the state after the last *processed* valid frame of each row;
  * rows with seq_lens[b] == 0 are allowed.

Because the method is exact (hoisting the input projection only reorders work), the oracle is
the plain definition, evaluated time step by time step with no blocking, fusion or reordering.

Pins (tests/test_oracle_pins.py): central finite differences of the scalar
L = sum(dy*y) + sum(dhT*hT) + sum(dcT*cT); zero-weight and constant-gate closed forms; padding
invariance with NaN padding; batch independence; reversal identity for direction -1; BLSTM
composition; time splitting; hoisting exactness; agreement with torch.nn.LSTM (CPU, float64,
packed sequences) as an independent library implementation; a scalar case evaluated in
50-digit arithmetic.

Second function pair, time_maxpool_fwd / time_maxpool_bwd (max-pooling in time between encoder layers, see the
comment above them): pinned by a hand-worked example (tests/golden/maxpool_case.txt), torch's max_pool1d and its
gradient on unpadded rows, brute force from the definition, NaN-padding invariance and central differences.

encoder_stack_fwd / encoder_stack_bwd (one bidirectional layer below unidirectional ones): pinned by chained
torch.nn.LSTM modules over packed sequences (outputs and every gradient), by its reduction to the bidirectional stack,
by causality of the top layer and by central differences.
"""
import numpy as np

F64 = np.float64


def _sigmoid(u):
    """Logistic function 1/(1+exp(-u)), evaluated without overflow on either side."""
    u = np.asarray(u, dtype=F64)
    out = np.empty_like(u)
    pos = u >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-u[pos]))
    e = np.exp(u[~pos])
    out[~pos] = e / (1.0 + e)
    return out


def _time_order(T, direction):
    """Frame index visited at processing step tau = 0..T-1 (Listing 1: `direction` +1 / -1)."""
    if direction == 1:
        return list(range(T))
    if direction == -1:
        return list(range(T - 1, -1, -1))
    raise ValueError("direction must be +1 or -1")


def _prep(x, W_x, W_h, b, h0, c0, seq_lens):
    x = np.asarray(x, dtype=F64)
    W_x = np.asarray(W_x, dtype=F64)
    W_h = np.asarray(W_h, dtype=F64)
    T, B, n_in = x.shape
    n = W_h.shape[0]
    assert W_x.shape == (n_in, 4 * n) and W_h.shape == (n, 4 * n)
    b = np.zeros(4 * n, F64) if b is None else np.asarray(b, dtype=F64)
    h0 = np.zeros((B, n), F64) if h0 is None else np.asarray(h0, dtype=F64)
    c0 = np.zeros((B, n), F64) if c0 is None else np.asarray(c0, dtype=F64)
    if seq_lens is None:
        seq_lens = np.full(B, T, np.int64)
    seq_lens = np.asarray(seq_lens, dtype=np.int64)
    assert seq_lens.shape == (B,) and (seq_lens >= 0).all() and (seq_lens <= T).all()
    return x, W_x, W_h, b, h0, c0, seq_lens, T, B, n_in, n


def lstm_fwd(x, W_x, W_h, b=None, h0=None, c0=None, seq_lens=None, direction=1, want_trace=False):
    """One masked LSTM layer over a whole batch of sequences, one direction.

    x[T,B,n_in], W_x[n_in,4n], W_h[n,4n], b[4n], h0/c0[B,n], seq_lens[B]
    -> y[T,B,n], cs[T,B,n], hT[B,n], cT[B,n]  (+ trace dict when want_trace).
    Follows the layer the paper names in Listing 1 (`rec` / `nativelstm2`, `direction`).
    """
    x, W_x, W_h, b, h0, c0, seq_lens, T, B, n_in, n = _prep(x, W_x, W_h, b, h0, c0, seq_lens)
    h = h0.copy()
    c = c0.copy()
    y = np.zeros((T, B, n), F64)
    cs = np.zeros((T, B, n), F64)
    tr = None
    if want_trace:
        tr = {k: np.zeros((T, B, n), F64) for k in ("i", "f", "g", "o", "tanh_c", "h_prev", "c_prev")}
    for t in _time_order(T, direction):
        v = np.nonzero(t < seq_lens)[0]          # valid rows at this frame
        cs[t] = c                                # padded rows store the carried cell state
        if v.size == 0:
            continue
        z = x[t, v] @ W_x + h[v] @ W_h + b       # [len(v), 4n], blocks i|f|g|o
        i = _sigmoid(z[:, 0 * n:1 * n])
        f = _sigmoid(z[:, 1 * n:2 * n])
        g = np.tanh(z[:, 2 * n:3 * n])
        o = _sigmoid(z[:, 3 * n:4 * n])
        c_new = f * c[v] + i * g
        tc = np.tanh(c_new)
        h_new = o * tc
        if want_trace:
            tr["i"][t, v], tr["f"][t, v], tr["g"][t, v], tr["o"][t, v] = i, f, g, o
            tr["tanh_c"][t, v] = tc
            tr["h_prev"][t, v] = h[v]
            tr["c_prev"][t, v] = c[v]
        c[v] = c_new
        h[v] = h_new
        y[t, v] = h_new
        cs[t, v] = c_new
    if want_trace:
        return y, cs, h, c, tr
    return y, cs, h, c


def lstm_bwd(x, W_x, W_h, b, h0, c0, seq_lens, direction, dy, dhT=None, dcT=None):
    """Exact gradient (back-propagation through time) of
    L = sum(dy*y) + sum(dhT*hT) + sum(dcT*cT) for the layer of `lstm_fwd`.

    -> dx[T,B,n_in], dW_x[n_in,4n], dW_h[n,4n], db[4n], dh0[B,n], dc0[B,n].
    The forward pass is re-run to obtain the gate activations.
    """
    x, W_x, W_h, b, h0, c0, seq_lens, T, B, n_in, n = _prep(x, W_x, W_h, b, h0, c0, seq_lens)
    dy = np.asarray(dy, dtype=F64)
    assert dy.shape == (T, B, n)
    _, _, _, _, tr = lstm_fwd(x, W_x, W_h, b, h0, c0, seq_lens, direction, want_trace=True)
    Dh = np.zeros((B, n), F64) if dhT is None else np.asarray(dhT, dtype=F64).copy()
    Dc = np.zeros((B, n), F64) if dcT is None else np.asarray(dcT, dtype=F64).copy()
    dx = np.zeros((T, B, n_in), F64)
    dW_x = np.zeros((n_in, 4 * n), F64)
    dW_h = np.zeros((n, 4 * n), F64)
    db = np.zeros(4 * n, F64)
    for t in reversed(_time_order(T, direction)):
        v = np.nonzero(t < seq_lens)[0]
        if v.size == 0:
            continue                              # padded rows: Dh, Dc pass through, dx stays 0
        i, f, g, o = tr["i"][t, v], tr["f"][t, v], tr["g"][t, v], tr["o"][t, v]
        tc = tr["tanh_c"][t, v]
        dh = dy[t, v] + Dh[v]
        do = dh * tc
        dc = Dc[v] + dh * o * (1.0 - tc * tc)
        di = dc * g
        dg = dc * i
        df = dc * tr["c_prev"][t, v]
        Dc[v] = dc * f
        dz = np.concatenate([di * i * (1.0 - i), df * f * (1.0 - f), dg * (1.0 - g * g), do * o * (1.0 - o)], axis=1)
        dx[t, v] = dz @ W_x.T
        Dh[v] = dz @ W_h.T
        dW_x += x[t, v].T @ dz
        dW_h += tr["h_prev"][t, v].T @ dz
        db += dz.sum(axis=0)
    return dx, dW_x, dW_h, db, Dh, Dc


def _opt(a, d):
    return None if a is None else a[d]


def blstm_fwd(x, W_x, W_h, b=None, h0=None, c0=None, seq_lens=None):
    """Bidirectional layer: a direction +1 and a direction -1 layer on the same input, outputs
    concatenated along the feature axis (Listing 1: enc*_fw, enc*_bw, `copy`).

    W_x[2,n_in,4n], W_h[2,n,4n], b[2,4n], h0/c0[2,B,n]  (index 0 = forward, 1 = backward)
    -> y[T,B,2n], cs[2,T,B,n], hT[2,B,n], cT[2,B,n].
    """
    outs = [lstm_fwd(x, W_x[d], W_h[d], _opt(b, d), _opt(h0, d), _opt(c0, d), seq_lens, 1 if d == 0 else -1)
            for d in (0, 1)]
    y = np.concatenate([outs[0][0], outs[1][0]], axis=2)
    return y, np.stack([outs[0][1], outs[1][1]]), np.stack([outs[0][2], outs[1][2]]), np.stack([outs[0][3], outs[1][3]])


def blstm_bwd(x, W_x, W_h, b, h0, c0, seq_lens, dy, dhT=None, dcT=None):
    """Gradient of the bidirectional layer: dy[T,B,2n] is split by column halves, dx is the sum of
    the two directions' dx, everything else is stacked with a leading [2]."""
    n = np.asarray(W_h).shape[1]
    dy = np.asarray(dy, dtype=F64)
    outs = [lstm_bwd(x, W_x[d], W_h[d], _opt(b, d), _opt(h0, d), _opt(c0, d), seq_lens, 1 if d == 0 else -1,
                     dy[:, :, d * n:(d + 1) * n], _opt(dhT, d), _opt(dcT, d)) for d in (0, 1)]
    dx = outs[0][0] + outs[1][0]
    return (dx,) + tuple(np.stack([outs[0][k], outs[1][k]]) for k in range(1, 6))


def blstm_stack_fwd(x, layers, seq_lens):
    """Stack of bidirectional layers (Sec. 4: every encoder layer is bidirectional, so layer k>1
    sees 2n inputs).  layers = list of dicts with W_x[2,n_in_k,4n], W_h[2,n,4n], b[2,4n] (or None).
    Initial states are zero.  -> list of per-layer inputs, final y."""
    acts = []
    cur = np.asarray(x, dtype=F64)
    for L in layers:
        acts.append(cur)
        cur = blstm_fwd(cur, L["W_x"], L["W_h"], L.get("b"), None, None, seq_lens)[0]
    return acts, cur


def blstm_stack_bwd(acts, layers, seq_lens, dy_top):
    """Back-propagate dy_top (w.r.t. the top layer's y) through the stack.
    -> dx of the bottom layer, list of (dW_x, dW_h, db) per layer (bottom first)."""
    grads = [None] * len(layers)
    d = np.asarray(dy_top, dtype=F64)
    for k in range(len(layers) - 1, -1, -1):
        L = layers[k]
        dx, dW_x, dW_h, db, _, _ = blstm_bwd(acts[k], L["W_x"], L["W_h"], L.get("b"), None, None, seq_lens, d)
        grads[k] = (dW_x, dW_h, db)
        d = dx
    return d, grads


# ---- encoders that mix bidirectional and unidirectional layers --------------------------------------------------
# The translation encoder of the paper's speed comparison (Sec. 3, caption of Table 1, the training-speed table; Sec. 4 for the
# comparison system) has one bidirectional layer at the bottom and 3 or 5 unidirectional layers above it.  A layer is
# bidirectional here when its weights carry two directions (W_x[2, n_in, 4n]) and runs forward in time when they carry
# one (W_x[1, n_in, 4n]); the layer above a bidirectional one sees 2n inputs, the layer above a unidirectional one n.
def encoder_stack_fwd(x, layers, seq_lens):
    """layers = list of dicts with W_x[D,n_in_k,4n], W_h[D,n,4n], b[D,4n] (or None), D in {1, 2}; zero initial
    states.  -> list of per-layer inputs, final y ([T,B,D_top*n])."""
    acts = []
    cur = np.asarray(x, dtype=F64)
    for L in layers:
        acts.append(cur)
        D = np.asarray(L["W_x"]).shape[0]
        b = L.get("b")
        if D == 2:
            cur = blstm_fwd(cur, L["W_x"], L["W_h"], b, None, None, seq_lens)[0]
        else:
            cur = lstm_fwd(cur, L["W_x"][0], L["W_h"][0], None if b is None else b[0], None, None, seq_lens, direction=1)[0]
    return acts, cur


def encoder_stack_bwd(acts, layers, seq_lens, dy_top):
    """Back-propagate dy_top through the mixed stack.  -> dx of the bottom layer, list of (dW_x, dW_h, db) per
    layer, bottom first, each with the leading direction axis of its layer."""
    grads = [None] * len(layers)
    d = np.asarray(dy_top, dtype=F64)
    for k in range(len(layers) - 1, -1, -1):
        L = layers[k]
        b = L.get("b")
        if np.asarray(L["W_x"]).shape[0] == 2:
            dx, dW_x, dW_h, db, _, _ = blstm_bwd(acts[k], L["W_x"], L["W_h"], b, None, None, seq_lens, d)
        else:
            dx, dW_x, dW_h, db, _, _ = lstm_bwd(acts[k], L["W_x"][0], L["W_h"][0], None if b is None else b[0], None, None,
                                                seq_lens, 1, d)
            dW_x, dW_h, db = dW_x[None], dW_h[None], db[None]
        grads[k] = (dW_x, dW_h, db)
        d = dx
    return d, grads


# ---- max-pooling in time between encoder layers ---------------------------------------------------------------
# The paper's attention-based speech encoder (Sec. 4, the attention model on Switchboard)
# takes a maximum over time between its six bidirectional layers, which shortens the input by a factor of 8 in
# total; window, stride and the treatment of padding are not given.  Reading of this repository:
# non-overlapping windows of `pool` consecutive frames (stride = window; 2 after each of three layers gives the
# factor 8), windows are taken inside every sequence separately:
#     T' = ceil(T / pool),  lens'[b] = ceil(lens[b] / pool),
#     out[t', b, :] = max over the VALID frames t in [pool t', pool t' + pool), t < lens[b], of y[t, b, :]
# for t' < lens'[b] and 0 at padded output frames; the last window of a sequence may be short.  Values stored at
# padded input frames are never read.  The gradient of an output element goes to the frame that supplied the maximum,
# to the earliest one when several are equal; every other element of dy, padded frames included, is 0.

def time_maxpool_fwd(y, seq_lens, pool):
    """Returns (out [T', B, F], lens' [B], arg [T', B, F]) with arg = offset of the chosen frame inside its window."""
    y = np.asarray(y, dtype=F64)
    T, B, F = y.shape
    lens = np.full(B, T, dtype=np.int64) if seq_lens is None else np.clip(np.asarray(seq_lens, dtype=np.int64), 0, T)
    assert pool >= 1
    Tp = -(-T // pool)
    lens_out = -(-lens // pool)
    out = np.zeros((Tp, B, F), dtype=F64)
    arg = np.zeros((Tp, B, F), dtype=np.int64)
    for b in range(B):
        for tp in range(int(lens_out[b])):
            t0 = pool * tp
            t1 = min(t0 + pool, int(lens[b]))
            best = y[t0, b, :].copy()
            which = np.zeros(F, dtype=np.int64)
            for t in range(t0 + 1, t1):
                better = y[t, b, :] > best          # strictly greater: ties keep the earliest frame
                best = np.where(better, y[t, b, :], best)
                which = np.where(better, t - t0, which)
            out[tp, b, :] = best
            arg[tp, b, :] = which
    return out, lens_out, arg


def time_maxpool_bwd(dout, arg, seq_lens, pool, T):
    """dy [T, B, F] from dout [T', B, F] and the arg of the forward pass."""
    dout = np.asarray(dout, dtype=F64)
    Tp, B, F = dout.shape
    lens = np.full(B, T, dtype=np.int64) if seq_lens is None else np.clip(np.asarray(seq_lens, dtype=np.int64), 0, T)
    dy = np.zeros((T, B, F), dtype=F64)
    cols = np.arange(F)
    for b in range(B):
        for tp in range(int(-(-lens[b] // pool))):
            dy[pool * tp + arg[tp, b, :], b, cols] = dout[tp, b, :]
    return dy
