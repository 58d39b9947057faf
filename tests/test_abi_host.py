"""Host-side tests of the C ABI: the library loads, exports every declared symbol, and reports
every argument error before touching the HIP runtime (so they all run without a GPU)."""
import ctypes
import os
import re

import pytest
import torch

from paper_1805_05225_amd import binding as Bn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x10000  # an aligned fake device pointer: validation must fail before anything dereferences it


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lstm_abi.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(?:int|const char\*)\s+(\w+)\s*\(", hdr))
    assert declared == set(Bn.EXPORTS)
    for name in declared:
        assert hasattr(Bn.lib, name)


def test_desc_layout_matches_header():
    assert ctypes.sizeof(Bn.LstmDesc) == 8 * 4 + 2 * 8


def _fwd(desc, fn=None, **over):
    a = dict(x=P, W_x=P, W_h=P, b=None, h0=None, c0=None, lens=None, y=P, c=P, hT=None, cT=None, reserve=P, ws=P)
    a.update(over)
    fn = fn or Bn.lib.lstm_fwd
    return fn(ctypes.byref(desc) if desc is not None else None, a["x"], a["W_x"], a["W_h"], a["b"], a["h0"], a["c0"], a["lens"],
              a["y"], a["c"], a["hT"], a["cT"], a["reserve"], a["ws"], None)


def _bwd(desc, fn=None, **over):
    a = dict(x=P, W_x=P, W_h=P, h0=None, c0=None, lens=None, y=P, c=P, reserve=P, dy=P, dhT=None, dcT=None, dx=P, dW_x=P,
             dW_h=P, db=P, dh0=None, dc0=None, ws=P)
    a.update(over)
    fn = fn or Bn.lib.lstm_bwd
    return fn(ctypes.byref(desc) if desc is not None else None, *[a[k] for k in (
        "x", "W_x", "W_h", "h0", "c0", "lens", "y", "c", "reserve", "dy", "dhT", "dcT", "dx", "dW_x", "dW_h", "db", "dh0",
        "dc0", "ws")], None)


def good_desc(**kw):
    d = Bn.make_desc(kw.pop("T", 5), kw.pop("B", 3), kw.pop("n_in", 4), kw.pop("n", 6), kw.pop("dtype", 0),
                     kw.pop("direction", 1), kw.pop("flags", 0))
    r, w = Bn.query(d, kw.pop("bidir", False))
    d.reserve_bytes, d.workspace_bytes = r, w
    return d


def test_query_sizes_grow_and_cover_bidirectional():
    d = Bn.make_desc(10, 4, 8, 16, 0)
    r1, w1 = Bn.query(d, False)
    r2, w2 = Bn.query(d, True)
    assert r2 > r1 > 10 * 4 * 4 * 16 * 4 and w2 > w1 > 0
    d0 = Bn.make_desc(0, 0, 8, 16, 1)
    r0, w0 = Bn.query(d0, True)
    assert r0 > 0 and w0 > 0


def test_null_and_dim_errors():
    assert _fwd(None) == -1
    for field, val in (("T", -1), ("B", -2), ("n", 0), ("n_in", 0)):
        d = good_desc()
        setattr(d, field, val)
        assert _fwd(d) == -2 and _bwd(d) == -2
    d = good_desc()
    assert _fwd(d, x=None) == -1 and _fwd(d, y=None) == -1 and _fwd(d, reserve=None) == -1 and _fwd(d, ws=None) == -1
    assert _bwd(d, dy=None) == -1 and _bwd(d, dW_h=None) == -1 and _bwd(d, c=None) == -1
    big = Bn.make_desc(1 << 20, 1 << 20, 4, 4, 0)
    assert _fwd(big) == -2


def test_direction_dtype_flag_errors():
    d = good_desc()
    d.direction = 0
    assert _fwd(d) == -3 and _bwd(d) == -3
    assert _fwd(d, fn=Bn.lib.blstm_fwd) in (-6, -7)          # blstm ignores direction; sizes are the uni ones
    d = good_desc(); d.dtype = 7
    assert _fwd(d) == -4
    d = good_desc(); d.flags = 64
    assert _fwd(d) == -4
    d = good_desc(flags=Bn.FLAG_PLAIN_LAUNCH)                  # a known flag: the sizes are those without it
    assert (d.reserve_bytes, d.workspace_bytes) == (good_desc().reserve_bytes, good_desc().workspace_bytes)
    d = good_desc(); d.reserved = 1
    assert _fwd(d) == -4
    d = good_desc(flags=Bn.FLAG_INFERENCE)
    assert _bwd(d) == -4                                       # nothing was saved: backward is impossible


def test_alignment_and_size_errors():
    d = good_desc()
    assert _fwd(d, x=P + 4) == -5 and _fwd(d, hT=P + 8) == -5 and _bwd(d, dcT=P + 2) == -5
    d.workspace_bytes -= 1
    assert _fwd(d) == -6 and _bwd(d) == -6
    d = good_desc(); d.reserve_bytes = 16
    assert _fwd(d) == -6
    d = good_desc(bidir=False)
    assert _fwd(d, fn=Bn.lib.blstm_fwd) == -6                  # bidirectional needs more than the uni sizes


def test_empty_batch_is_a_noop_and_inference_needs_no_reserve():
    d = good_desc(B=0)
    assert _fwd(d) == 0
    d = good_desc(flags=Bn.FLAG_INFERENCE)
    r, w = Bn.query(d, False)
    assert r == 0
    if not torch.cuda.is_available():
        assert _fwd(d, reserve=None, c=None) == -7             # valid call, but no gfx950 device here


def test_time_pool_argument_errors():
    f, b = Bn.lib.lstm_time_pool_fwd, Bn.lib.lstm_time_pool_bwd
    ok = dict(dtype=1, T=8, B=2, F=16, pool=2)
    fwd = lambda y=P, out=P, ldy=16, ldo=16, **o: f(*[{**ok, **o}[k] for k in ("dtype", "T", "B", "F", "pool")], y, ldy, None, out, ldo, None, None, None)
    bwd = lambda dout=P, dy=P, arg=P, ldo=16, ldy=16, **o: b(*[{**ok, **o}[k] for k in ("dtype", "T", "B", "F", "pool")], dout, ldo, arg, None, dy, ldy, None)
    assert fwd(y=None) == -1 and fwd(out=None) == -1 and bwd(dout=None) == -1 and bwd(dy=None) == -1 and bwd(arg=None) == -1
    for bad in (dict(T=-1), dict(B=-1), dict(F=0), dict(pool=0), dict(pool=256), dict(B=70000)):
        assert fwd(**bad) == -2 and bwd(**bad) == -2
    assert fwd(ldy=15) == -2 and fwd(ldo=8) == -2 and bwd(ldy=3) == -2
    assert fwd(dtype=7) == -4 and bwd(dtype=-1) == -4
    assert fwd(y=P + 1) == -5 and bwd(dy=P + 1) == -5 and fwd(dtype=0, out=P + 2) == -5


def test_attention_and_readout_argument_errors():
    import ctypes
    q = ctypes.c_uint64(0)
    mk = lambda **o: Bn.AttDesc(*[{**dict(S=8, Q=2, beam=3, A=16, E=32, n=24), **o}[k] for k in ("S", "Q", "beam", "A", "E", "n")], 1 << 30)
    query = lambda **o: Bn.lib.lstm_attention_query(ctypes.byref(mk(**o)), ctypes.byref(q))
    assert query() == 0 and q.value > 0
    assert Bn.lib.lstm_attention_query(None, ctypes.byref(q)) == -1 and Bn.lib.lstm_attention_query(ctypes.byref(mk()), None) == -1
    for bad in (dict(S=0), dict(Q=-1), dict(beam=0), dict(A=0), dict(E=0), dict(n=0), dict(Q=70000)):
        assert query(**bad) == -2
    for bad in (dict(beam=17), dict(S=1025), dict(E=33)):
        assert query(**bad) == -4
    names = ("enc", "ctx", "lens", "s", "ld_s", "W_s", "b_s", "w_fb", "b_fb", "v", "b_e", "acc_in", "acc_out", "a", "att", "ld_att", "ws")
    base = dict(enc=P, ctx=P, lens=None, s=P, ld_s=24, W_s=P, b_s=P, w_fb=P, b_fb=P, v=P, b_e=0.0, acc_in=P, acc_out=P, a=None, att=P, ld_att=32, ws=P)
    step = lambda d=None, **o: Bn.lib.lstm_attention_step(ctypes.byref(d or mk()), *[{**base, **o}[k] for k in names], None)
    for k in ("enc", "ctx", "s", "W_s", "b_s", "w_fb", "b_fb", "v", "acc_in", "acc_out", "att", "ws"):
        assert step(**{k: None}) == -1, k
    assert step(ld_s=23) == -2 and step(ld_att=30) == -2
    assert step(ld_att=33) == -5 and step(att=P + 2) == -5 and step(b_s=P + 2) == -5 and step(s=P + 1) == -5
    small = mk(); small.workspace_bytes = 16
    assert step(small) == -6
    assert step(mk(Q=0)) == 0                                   # nothing to do, nothing launched
    # readout
    rq = lambda B=4, R=8, n=16, nt=4, E=6: Bn.lib.lstm_readout_query(B, R, n, nt, E, ctypes.byref(q))
    assert rq() == 0 and q.value > 0 and rq(B=-1) == -2 and rq(R=0) == -2 and rq(n=0) == -2 and rq(nt=-1) == -2
    assert Bn.lib.lstm_readout_query(4, 8, 16, 4, 6, None) == -1
    ro = lambda fl=0, B=4, R=8, s=P, ld_s=16, n=16, trg=P, ld_trg=4, nt=4, att=P, ld_att=6, E=6, W=P, b=None, out=P, ld_out=8, ws=P, wsb=1 << 30: \
        Bn.lib.lstm_readout(fl, B, R, s, ld_s, n, trg, ld_trg, nt, att, ld_att, E, W, b, out, ld_out, ws, wsb, None)
    assert ro(s=None) == -1 and ro(trg=None) == -1 and ro(att=None) == -1 and ro(W=None) == -1 and ro(out=None) == -1 and ro(ws=None) == -1
    assert ro(ld_s=15) == -2 and ro(ld_trg=3) == -2 and ro(ld_att=5) == -2 and ro(ld_out=7) == -2 and ro(B=-1) == -2
    assert ro(s=P + 1) == -5 and ro(b=P + 2) == -5
    assert ro(wsb=8) == -6 and ro(fl=3) == -4
    assert ro(B=0) == 0 and ro(fl=8, B=0) == 0


def test_beam_argument_errors():
    import ctypes
    q = ctypes.c_uint64(0)
    L = Bn.lib
    assert L.lstm_beam_query(4, 12, 20000, ctypes.byref(q)) == 0 and q.value > 0
    assert L.lstm_beam_query(4, 12, 20000, None) == -1 and L.lstm_beam_query(-1, 12, 10, ctypes.byref(q)) == -2
    assert L.lstm_beam_query(4, 0, 10, ctypes.byref(q)) == -2 and L.lstm_beam_query(4, 2, 0, ctypes.byref(q)) == -2
    assert L.lstm_beam_query(4, 17, 10, ctypes.byref(q)) == -4 and L.lstm_beam_query(4, 2, (1 << 26) + 1, ctypes.byref(q)) == -4
    st = lambda Q=4, beam=3, V=10, lg=P, ld=10, si=P, so=P, src=P, lab=P, ws=P, wsb=1 << 20: L.lstm_beam_step(Q, beam, V, lg, ld, si, so, src, lab, ws, wsb, None)
    for k in ("lg", "si", "so", "src", "lab", "ws"):
        assert st(**{k: None}) == -1, k
    assert st(ld=9) == -2 and st(Q=-1) == -2 and st(beam=17) == -4 and st(lg=P + 2) == -5 and st(wsb=8) == -6 and st(Q=0) == 0
    # the variant with the library's own scratch array: same argument checks, and a size limit instead of a workspace
    ss = lambda Q=4, beam=3, V=10, lg=P, ld=10, si=P, so=P, src=P, lab=P: L.lstm_beam_step_static(Q, beam, V, lg, ld, si, so, src, lab, None)
    for k in ("lg", "si", "so", "src", "lab"):
        assert ss(**{k: None}) == -1, k
    assert ss(ld=9) == -2 and ss(Q=-1) == -2 and ss(beam=17) == -4 and ss(lg=P + 2) == -5 and ss(Q=0) == 0
    assert ss(Q=257, beam=16) == -6 and ss(Q=65537, beam=1) == -6
    ga = lambda eb=4, Q=4, beam=3, w=8, i=P, ldi=8, src=P, o=P + 4096, ldo=8: L.lstm_beam_gather(eb, Q, beam, w, i, ldi, src, o, ldo, None)
    assert ga(i=None) == -1 and ga(src=None) == -1 and ga(o=None) == -1
    assert ga(w=0) == -2 and ga(ldi=7) == -2 and ga(ldo=7) == -2 and ga(eb=3) == -4 and ga(o=P) == -4 and ga(i=P + 2) == -5 and ga(Q=0) == 0
    def gm(count=2, Q=4, beam=3, src=P, **over):
        arr = (Bn.GatherItem * 8)()
        for it in arr:
            it.elem_bytes, it.width, it.inp, it.ld_in, it.out, it.ld_out = 4, 8, P, 8, P + 4096, 8
        for k, v in over.items():
            setattr(arr[1], k, v)
        return L.lstm_beam_gather_many(Q, beam, count, arr, src, None)
    assert gm(count=0) == -2 and gm(count=9) == -2 and gm(src=None) == -1 and gm(Q=-1) == -2 and gm(Q=0) == 0
    assert L.lstm_beam_gather_many(4, 3, 1, None, P, None) == -1
    assert gm(inp=None) == -1 and gm(width=0) == -2 and gm(ld_out=7) == -2 and gm(elem_bytes=8) == -4 and gm(out=P) == -4 and gm(inp=P + 2) == -5
    em = lambda B=4, n=8, V=10, lab=P, W=P, b=None, o=P, ldo=8: L.lstm_embed(B, n, V, lab, W, b, o, ldo, None)
    assert em(lab=None) == -1 and em(W=None) == -1 and em(o=None) == -1
    assert em(n=0) == -2 and em(V=0) == -2 and em(ldo=7) == -2 and em(o=P + 1) == -5 and em(b=P + 2) == -5 and em(B=0) == 0


def test_strerror():
    for s in range(0, -8, -1):
        assert Bn.strerror(s) and "unknown" not in Bn.strerror(s)
    assert "unknown" in Bn.strerror(-99)
