"""GPU parity of the chained search step in the arrangement the benchmark times (bench.py --config 9): cell -> attention ->
readout -> output layer -> beam step -> state gather -> target embedding, two dependent steps, the context written straight
into the next step's cell input rows.  Every stage is compared with the oracle evaluated on the inputs that stage actually
received on the GPU (so that bfloat16 roundings of earlier stages do not blur later comparisons); integer results of the
beam step are validated as in tests/test_gpu_beam.py."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import decoder_oracle as D
from oracle import lstm_oracle as O
from paper_1805_05225_amd import synth
from tests.gpu_util import TOL, check, dev, host

TOL_BF16, TOL_F32 = 5e-3, 1e-4


def test_two_chained_search_steps():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1805_05225_amd import binding as Bn
    dec = synth.make_decoder(Q=3, beam=4, len_lo=5, len_hi=11, A=48, E=64, n=40, n_trg=24, R=32)
    cfg, S, B = dec["cfg"], dec["S"], dec["B"]
    Q, beam, A, E, n, nt, R, V = cfg["Q"], cfg["beam"], cfg["A"], cfg["E"], cfg["n"], cfg["n_trg"], cfg["R"], 200
    rng = np.random.default_rng(77)
    bfr = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()
    Wx, Wh = bfr(rng.uniform(-.2, .2, (nt + E, 4 * n))), bfr(rng.uniform(-.2, .2, (n, 4 * n)))
    b = rng.uniform(-.1, .1, 4 * n).astype(np.float32)
    W_o, b_o = bfr(rng.uniform(-.5, .5, (V, R))), rng.uniform(-.5, .5, V).astype(np.float32)
    W_trg, b_trg = bfr(rng.uniform(-.5, .5, (V, nt))), rng.uniform(-.1, .1, nt).astype(np.float32)
    g = lambda k, dt=None: dev(dec[k], dt)
    enc, ctx, lens = g("H", "bf16"), g("ctx", "bf16"), dev(dec["src_lens"])
    W_s, W_r = g("W_s", "bf16"), g("W_r", "bf16")
    vecs = [g(k) for k in ("b_s", "w_fb", "b_fb", "v")]
    dWx, dWh, db = dev(Wx, "bf16"), dev(Wh, "bf16"), dev(b)
    dW_o, db_o, dW_trg, db_trg = dev(W_o, "bf16"), dev(b_o), dev(W_trg, "bf16"), dev(b_trg)
    xin = [torch.zeros(B, nt + E, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    xin[0][:, :nt] = g("trg", "bf16")
    h = torch.zeros(B, n, device="cuda"); c = torch.zeros(B, n, device="cuda")
    accum = torch.zeros(B, S, device="cuda")
    score = torch.zeros(Q, beam, device="cuda"); score[:, 1:] = float("-inf")
    f64 = lambda t: host(t)
    for step in range(2):
        p = step % 2
        x_in, h_in, c_in, acc_in, sc_in = f64(xin[p]), f64(h), f64(c), f64(accum), f64(score)
        print("  search step", step, flush=True)
        # cell: one time step of the layer
        f = Bn.forward(xin[p].view(1, B, nt + E), dWx, dWh, db, h, c, None, bidirectional=False, flags=Bn.FLAG_INFERENCE, want_c=False)
        y, h_new, c_new = f["y"][0], f["hT"], f["cT"]
        yo, _, hTo, cTo = O.lstm_fwd(x_in[None], Wx.astype(np.float64), Wh.astype(np.float64), b.astype(np.float64), h_in, c_in, None, 1)
        check("s", y, yo[0], TOL["bf16"]); check("h", h_new, hTo, TOL["bf16"]); check("c", c_new, cTo, TOL["bf16"])      # the layer's own tolerance
        # attention on the cell output the GPU produced, context written into the next step's cell input rows
        att_view = xin[1 - p][:, nt:]
        r = Bn.attention_step(enc, ctx, lens, beam, y, W_s, *vecs, dec["b_e"], accum, att=att_view)
        a_o, acc_o, att_o, _ = D.attention_step(f64(enc), f64(ctx), dec["src_lens"], beam, f64(y), acc_in, f64(W_s).T, *[f64(t) for t in vecs],
                                                dec["b_e"])
        check("a", r["a"], a_o, TOL_F32); check("accum", r["accum"], acc_o, TOL_F32); check("att", att_view, att_o, TOL_BF16)
        # readout from s, the previous target embedding (first columns of this step's cell input) and att where it lies
        ro = Bn.readout(y, xin[p][:, :nt], att_view, W_r, g("b_r"))
        check("readout", ro, D.readout(f64(y), x_in[:, :nt], f64(att_view), f64(W_r).T, f64(g("b_r"))), TOL_BF16)
        # output layer and beam step
        logits = Bn.gemm(ro, dW_o, a_kcontig=True, b_kcontig=True, M=B, N=V, K=R, bias=db_o)
        lo = f64(ro) @ W_o.astype(np.float64).T + b_o
        check("logits", logits, lo, TOL_F32)
        bs = Bn.beam_step(logits, score)
        torch.cuda.synchronize()
        sc_o, src_o, lab_o = D.beam_step(f64(logits), sc_in, beam)
        got_sc, got_src, got_lab = f64(bs["score"]), bs["src"].cpu().numpy().astype(np.int64), bs["label"].cpu().numpy().astype(np.int64)
        assert np.abs(got_sc - sc_o).max() < 2e-5
        cand = sc_in[:, :, None] + D.log_softmax_rows(f64(logits)).reshape(Q, beam, V)
        assert np.abs(cand[np.arange(Q)[:, None], got_src, got_lab] - got_sc).max() < 2e-5
        assert (np.array_equal(got_src, src_o) and np.array_equal(got_lab, lab_o)) or np.abs(np.diff(sc_o, axis=1)).min() < 4e-5
        # state follows the chosen hypotheses; the chosen labels are embedded into the next step's cell input
        h2, c2, acc2 = Bn.beam_gather(h_new, bs["src"]), Bn.beam_gather(c_new, bs["src"]), Bn.beam_gather(r["accum"], bs["src"])
        att_g = Bn.beam_gather(att_view.contiguous(), bs["src"])
        assert np.array_equal(f64(h2), D.gather_rows(f64(h_new), got_src, beam)) and np.array_equal(f64(c2), D.gather_rows(f64(c_new), got_src, beam))
        assert np.array_equal(f64(acc2), D.gather_rows(f64(r["accum"]), got_src, beam))
        assert np.array_equal(f64(att_g), D.gather_rows(f64(att_view), got_src, beam))
        xin[1 - p][:, nt:] = att_g
        Bn.embed(bs["label"], dW_trg, db_trg, out=xin[1 - p][:, :nt])
        torch.cuda.synchronize()
        want = torch.from_numpy(D.embed(got_lab, W_trg.astype(np.float64), b_trg.astype(np.float64)).astype(np.float32)).to(torch.bfloat16)
        assert torch.equal(xin[1 - p][:, :nt].cpu(), want)
        h, c, accum, score = h2, c2, acc2, bs["score"]
    assert bool(torch.isfinite(score).all())                     # after the first step every hypothesis is alive
