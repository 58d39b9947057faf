"""Seeded synthetic inputs for the benchmark configurations (1-5, the mixed encoder 7, and the decoder step).

This module only draws random numbers and rounds them to the storage type; it holds none of
the LSTM arithmetic.  Both the CPU oracle's tests and the HIP path's tests take their inputs
from here, so the two sides always see identical values.

The inputs stand in for the paper's WMT 2017 and Switchboard workloads (Sec. 3-4), which are
not available: only their shapes are used - embedding width 620, 1000 units per direction,
six bidirectional encoder layers, decoder cell input 620 + 2000, beam 12 (Listing 1; Sec. 3, Table 2).

Draw order for configuration k, from torch.Generator(cpu) seeded with 18050522500 + k:
seq_lens, x, then per layer and per direction W_x, W_h, b, then h0, c0, dy.
Padded frames of x and dy are filled with N(0,1) noise (not zeros) so a missing mask shows.
"""
import numpy as np
import torch

SEED_BASE = 18050522500

# kind: "lstm" (one direction), "blstm", or "mixed" (first layer bidirectional, the others forward in time).
# len range is inclusive.  dtype "f32" or "bf16".
CONFIGS = {
    1: dict(kind="lstm", dtype="f32", n_in=32, n=64, B=4, layers=1, len_lo=20, len_hi=20, w=0.1),
    2: dict(kind="blstm", dtype="f32", n_in=620, n=1000, B=64, layers=1, len_lo=10, len_hi=50, w=0.08),
    3: dict(kind="blstm", dtype="bf16", n_in=620, n=1000, B=64, layers=6, len_lo=20, len_hi=80, w=0.08),
    4: dict(kind="blstm", dtype="bf16", n_in=40, n=1024, B=32, layers=6, len_lo=200, len_hi=1500, w=0.08),
    5: dict(kind="lstm", dtype="bf16", n_in=2620, n=1000, B=768, layers=1, len_lo=1, len_hi=1, w=0.08, steps=100),
    # the translation encoder of the speed comparison: one bidirectional layer below `layers - 1` unidirectional ones
    7: dict(kind="mixed", dtype="bf16", n_in=620, n=1000, B=64, layers=6, len_lo=20, len_hi=80, w=0.08),
}


def round_to(a, dtype):
    """Round a float32 torch tensor to the storage type and return it as float32 (exact)."""
    if dtype == "bf16":
        return a.to(torch.bfloat16).to(torch.float32)
    return a


def make(k, **override):
    """Build configuration k (optionally with overridden sizes, e.g. len_hi=40, layers=2, B=8).

    Returns a dict of numpy arrays (float32 values, already rounded to bf16 where the config
    stores bf16): seq_lens int32 [B]; x [T,B,n_in]; layers = list of {W_x [D,n_in_k,4n],
    W_h [D,n,4n], b [D,4n]} with D = 2 for "blstm" and D = 1 for "lstm" ("mixed": 2 for the first layer, 1 above,
    and the second layer sees 2n inputs); h0, c0 [D,B,n]
    (zeros, as every configuration prescribes); dy [T,B,D*n] for the top layer's output.
    """
    cfg = dict(CONFIGS[k])
    cfg.update(override)
    g = torch.Generator(device="cpu")
    g.manual_seed(SEED_BASE + k)
    B, n, n_in, dt = cfg["B"], cfg["n"], cfg["n_in"], cfg["dtype"]
    mixed = cfg["kind"] == "mixed"
    D = 2 if cfg["kind"] == "blstm" else 1             # directions of the top layer (and of every layer unless mixed)
    lens = torch.randint(cfg["len_lo"], cfg["len_hi"] + 1, (B,), generator=g, dtype=torch.int64)
    T = int(lens.max())
    x = round_to(torch.randn(T, B, n_in, generator=g), dt)
    layers = []
    for l in range(cfg["layers"]):
        Dl = 2 if (mixed and l == 0) else D
        ni = n_in if l == 0 else (2 * n if (mixed and l == 1) else D * n)
        Wx, Wh, bb = [], [], []
        for d in range(Dl):
            Wx.append(round_to((torch.rand(ni, 4 * n, generator=g) * 2 - 1) * cfg["w"], dt))
            Wh.append(round_to((torch.rand(n, 4 * n, generator=g) * 2 - 1) * cfg["w"], dt))
            bb.append(torch.zeros(4 * n))
        layers.append(dict(W_x=torch.stack(Wx).numpy(), W_h=torch.stack(Wh).numpy(), b=torch.stack(bb).numpy()))
    h0 = torch.zeros(D, B, n)
    c0 = torch.zeros(D, B, n)
    dy = round_to(torch.randn(T, B, D * n, generator=g), dt)
    return dict(cfg=cfg, k=k, T=T, D=D, seq_lens=lens.to(torch.int32).numpy(), x=x.numpy(), layers=layers,
                h0=h0.numpy(), c0=c0.numpy(), dy=dy.numpy())


def real_frames(inp):
    return int(inp["seq_lens"].astype(np.int64).sum())


def flops_fwd_bwd(inp):
    """Useful floating-point operations of one forward + backward pass over the stack:
    24*n*(n_in+n) per real frame, per direction, per layer (matrix products only)."""
    cfg = inp["cfg"]
    n, D = cfg["n"], inp["D"]
    tot = 0
    for l, L in enumerate(inp["layers"]):
        Dl, ni = L["W_x"].shape[0], L["W_x"].shape[1]
        tot += Dl * 24 * n * (ni + n)
    return tot * real_frames(inp)


# ---- one step of the attention decoder (Listing 1: 620-wide target embedding, 1000-wide cell, attention and readout,
# 2000-wide encoder states; Table 2: beam 12) ------------------------------------------------------------------------
DECODER = dict(Q=64, beam=12, len_lo=20, len_hi=80, A=1000, E=2000, n=1000, n_trg=620, R=1000, w=0.05)


def make_decoder(**override):
    """Seeded inputs of one decoder step, every bfloat16-stored tensor already rounded (float32 numpy arrays):
    src_lens int32 [Q]; H [S,Q,E] encoder states and ctx [S,Q,A] their projection, both drawn directly (the step takes
    ctx as an input); s [B,n] cell output, trg [B,n_trg] previous target embedding, accum [B,S] accumulated weights
    (zero at padded positions); W_s [A,n], b_s, w_fb, b_fb, v [A], b_e; W_r [R, n+n_trg+E], b_r [R].  B = Q*beam.
    Draw order: src_lens, H, ctx, s, trg, accum, W_s, b_s, w_fb, b_fb, v, b_e, W_r, b_r."""
    cfg = dict(DECODER)
    cfg.update(override)
    g = torch.Generator(device="cpu")
    g.manual_seed(SEED_BASE + 8)
    Q, beam, A, E, n, nt, R, w = cfg["Q"], cfg["beam"], cfg["A"], cfg["E"], cfg["n"], cfg["n_trg"], cfg["R"], cfg["w"]
    B = Q * beam
    lens = torch.randint(cfg["len_lo"], cfg["len_hi"] + 1, (Q,), generator=g, dtype=torch.int64)
    S = max(int(lens.max()), 1) if Q > 0 else 1
    bf = lambda a: round_to(a, "bf16")
    u = lambda *shape: torch.rand(*shape, generator=g) * 2 - 1
    H = bf(u(S, Q, E))
    ctx = bf(torch.randn(S, Q, A, generator=g))
    s = bf(u(B, n))
    trg = bf(torch.randn(B, nt, generator=g) * 0.5)
    accum = torch.rand(B, S, generator=g) * 1.5
    valid = torch.arange(S)[None, :] < lens.repeat_interleave(beam)[:, None]
    accum = accum * valid
    out = dict(cfg=cfg, S=S, B=B, src_lens=lens.to(torch.int32).numpy(), H=H.numpy(), ctx=ctx.numpy(), s=s.numpy(), trg=trg.numpy(),
               accum=accum.numpy(), W_s=bf(u(A, n) * w).numpy(), b_s=(u(A) * 0.1).numpy(), w_fb=(u(A) * 0.5).numpy(),
               b_fb=(u(A) * 0.1).numpy(), v=(u(A) * 0.2).numpy(), b_e=float(u(1)[0]) * 0.1,
               W_r=bf(u(R, n + nt + E) * w).numpy(), b_r=(u(R) * 0.1).numpy())
    return out
