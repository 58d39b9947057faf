"""Pins of the attention-step oracle (oracle/decoder_oracle.py) to things other than itself: a hand-worked example,
closed forms, invariants, brute force with scalar loops and an independent evaluation with torch routines."""
import math
import os

import numpy as np
import torch

from oracle import decoder_oracle as D

HERE = os.path.dirname(os.path.abspath(__file__))


def case(S=7, Q=3, beam=2, A=5, E=4, n=6, lens=(7, 3, 5), seed=0):
    rng = np.random.default_rng(seed)
    B = Q * beam
    return dict(H=rng.standard_normal((S, Q, E)), ctx=rng.standard_normal((S, Q, A)), src_lens=np.array(lens), beam=beam,
                s=rng.standard_normal((B, n)), accum=rng.uniform(0, 2, (B, S)), W_s=rng.uniform(-.5, .5, (n, A)),
                b_s=rng.uniform(-.5, .5, A), w_fb=rng.uniform(-.5, .5, A), b_fb=rng.uniform(-.5, .5, A),
                v=rng.uniform(-1, 1, A), b_e=0.3)


def run(c, **over):
    d = dict(c); d.update(over)
    return D.attention_step(d["H"], d["ctx"], d["src_lens"], d["beam"], d["s"], d["accum"], d["W_s"], d["b_s"], d["w_fb"], d["b_fb"],
                            d["v"], d["b_e"])


def test_hand_worked_example():
    want = np.loadtxt(os.path.join(HERE, "golden", "attention_case.txt"))
    t = math.atanh(0.5)
    a, acc, att, e = D.attention_step(H=np.array([[[4.0, 0.0]], [[0.0, 8.0]]]), ctx=np.zeros((2, 1, 1)), src_lens=[2], beam=1,
                                      s=[[2.0]], accum=[[1.0, 0.0]], W_s=[[0.25]], b_s=[-0.5], w_fb=[t], b_fb=[0.0],
                                      v=[2 * math.log(3.0)], b_e=0.0)
    got = np.concatenate([a[0], acc[0], att[0], e[0]])
    np.testing.assert_allclose(got, want, rtol=1e-14, atol=1e-15)


def test_zero_v_gives_uniform_weights_and_mean_state():
    c = case()
    a, acc, att, e = run(c, v=np.zeros(5))
    for r in range(6):
        L = c["src_lens"][r // 2]
        np.testing.assert_allclose(a[r, :L], 1.0 / L, rtol=1e-14)
        assert np.all(a[r, L:] == 0)
        np.testing.assert_allclose(att[r], c["H"][:L, r // 2].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_one_dominant_position_selects_its_state():
    c = case()
    # tanh saturates: the energy of position 2 of every sentence is about 40 above the others
    ctx = np.zeros_like(c["ctx"]); ctx[2] = 50.0
    a, acc, att, e = run(c, ctx=ctx, v=np.full(5, 8.0), w_fb=np.zeros(5), b_fb=np.zeros(5), W_s=np.zeros((6, 5)), b_s=np.zeros(5))
    for r in range(6):
        assert a[r, 2] > 1 - 1e-15
        np.testing.assert_allclose(att[r], c["H"][2, r // 2], rtol=1e-12, atol=1e-12)


def test_invariants_shift_sum_and_accumulation():
    c = case(seed=1)
    a, acc, att, e = run(c)
    a2, acc2, att2, e2 = run(c, b_e=c["b_e"] + 7.5)
    np.testing.assert_allclose(a2, a, rtol=1e-12, atol=1e-15)          # softmax ignores a common shift of the energies
    np.testing.assert_allclose(e2 - e, 7.5 * (e != 0), rtol=1e-12)
    np.testing.assert_allclose(a.sum(axis=1), 1.0, rtol=1e-14)
    for r in range(6):
        L = c["src_lens"][r // 2]
        np.testing.assert_allclose(acc[r, :L] - c["accum"][r, :L], a[r, :L], rtol=1e-13, atol=1e-15)
        assert np.all(acc[r, L:] == 0) and np.all(a[r, L:] == 0)
    assert np.all(a >= 0)


def test_padding_is_never_read_and_empty_sentence():
    c = case(lens=(7, 0, 5), seed=2)
    ref = run(c)
    d = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in c.items()}
    for q, L in enumerate(c["src_lens"]):
        d["H"][L:, q] = np.nan; d["ctx"][L:, q] = np.nan
        d["accum"][q * 2:(q + 1) * 2, L:] = np.nan
    got = run(d)
    for x, y in zip(ref, got):
        np.testing.assert_array_equal(x, y)
    assert np.all(got[0][2:4] == 0) and np.all(got[2][2:4] == 0) and np.all(got[1][2:4] == 0)


def test_permutation_of_source_positions():
    c = case(lens=(7, 7, 7), seed=3)
    perm = np.array([3, 0, 6, 1, 5, 2, 4])
    a, acc, att, e = run(c)
    ap, accp, attp, ep = run(c, H=c["H"][perm], ctx=c["ctx"][perm], accum=c["accum"][:, perm])
    np.testing.assert_allclose(ap, a[:, perm], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(accp, acc[:, perm], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(attp, att, rtol=1e-12, atol=1e-14)


def test_rows_are_independent_and_a_beam_shares_its_sentence():
    c = case(seed=4)
    ref = run(c)
    s2 = c["s"].copy(); s2[3] += 1.0                            # only row 3 may change
    got = run(c, s=s2)
    for x, y in zip(ref, got):
        keep = np.arange(6) != 3
        np.testing.assert_array_equal(x[keep], y[keep])
        assert np.abs(x[3] - y[3]).max() > 1e-6
    s3 = c["s"].copy(); s3[1] = s3[0]                           # two hypotheses of sentence 0 in the same state
    acc3 = c["accum"].copy(); acc3[1] = acc3[0]
    got = run(c, s=s3, accum=acc3)
    for y in got:
        np.testing.assert_array_equal(y[0], y[1])
    # row r reads sentence r // beam: swapping the encoder states of sentences 0 and 1 (same length needed) swaps nothing else
    c5 = case(lens=(5, 5, 4), seed=5)
    a, acc, att, e = run(c5)
    sw = [1, 0, 2]
    rows = [2, 3, 0, 1, 4, 5]
    a2, acc2, att2, e2 = run(c5, H=c5["H"][:, sw], ctx=c5["ctx"][:, sw], s=c5["s"][rows], accum=c5["accum"][rows])
    np.testing.assert_allclose(a2, a[rows], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(att2, att[rows], rtol=1e-13, atol=1e-15)


def test_brute_force_scalar_loops():
    c = case(S=4, Q=2, beam=2, A=3, E=2, n=2, lens=(4, 2), seed=6)
    a, acc, att, e = run(c)
    for r in range(4):
        q = r // 2
        L = c["src_lens"][q]
        en = []
        for j in range(L):
            tot = c["b_e"]
            for k in range(3):
                s_tr = c["b_s"][k]
                for i in range(2):
                    s_tr += c["s"][r, i] * c["W_s"][i, k]
                tot += c["v"][k] * math.tanh(c["ctx"][j, q, k] + c["accum"][r, j] * c["w_fb"][k] + c["b_fb"][k] + s_tr)
            en.append(tot)
        z = sum(math.exp(x) for x in en)
        for j in range(L):
            assert abs(a[r, j] - math.exp(en[j]) / z) < 1e-14
            assert abs(e[r, j] - en[j]) < 1e-14
            assert abs(acc[r, j] - c["accum"][r, j] - math.exp(en[j]) / z) < 1e-14
        for f in range(2):
            assert abs(att[r, f] - sum(math.exp(en[j]) / z * c["H"][j, q, f] for j in range(L))) < 1e-13


def test_against_torch_routines():
    c = case(S=9, Q=4, beam=3, A=6, E=5, n=4, lens=(9, 1, 6, 4), seed=7)
    a, acc, att, e = run(c)
    t = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in c.items() if k not in ("beam", "b_e", "src_lens")}
    qr = torch.arange(12) // 3
    s_tr = torch.nn.functional.linear(t["s"], t["W_s"].T, t["b_s"])                              # [B, A]
    e_in = t["ctx"][:, qr] + t["accum"].T[:, :, None] * t["w_fb"] + t["b_fb"] + s_tr[None]       # [S, B, A]
    en = torch.tanh(e_in) @ t["v"] + c["b_e"]                                                    # [S, B]
    mask = torch.arange(9)[:, None] < torch.from_numpy(c["src_lens"])[qr][None, :]
    at = torch.softmax(en.masked_fill(~mask, float("-inf")), dim=0)                              # [S, B]
    ctxv = torch.bmm(at.T[:, None, :], t["H"][:, qr].permute(1, 0, 2))[:, 0]                     # [B, E]
    np.testing.assert_allclose(a, at.T.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(att, ctxv.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(acc, ((t["accum"] + at.T) * mask.T).numpy(), rtol=1e-12, atol=1e-15)


def test_enc_ctx_and_readout():
    rng = np.random.default_rng(8)
    H = rng.standard_normal((3, 2, 4)); W = rng.standard_normal((4, 5)); b = rng.standard_normal(5)
    got = D.enc_ctx(H, W, b)
    for j in range(3):
        for q in range(2):
            for k in range(5):
                assert abs(got[j, q, k] - (b[k] + sum(H[j, q, i] * W[i, k] for i in range(4)))) < 1e-13
    s, trg, att = rng.standard_normal((2, 3)), rng.standard_normal((2, 2)), rng.standard_normal((2, 4))
    W_r = rng.standard_normal((9, 6)); b_r = rng.standard_normal(6)
    ro = D.readout(s, trg, att, W_r, b_r)
    want = torch.relu(torch.nn.functional.linear(torch.from_numpy(np.concatenate([s, trg, att], 1)), torch.from_numpy(W_r.T.copy()),
                                                 torch.from_numpy(b_r))).numpy()
    np.testing.assert_allclose(ro, want, rtol=1e-13, atol=1e-14)
    assert (ro == 0).any() and (ro > 0).any()
    # rows of W_r are ordered s | trg | att: zeroing the att rows removes att's influence
    W0 = W_r.copy(); W0[5:] = 0
    np.testing.assert_array_equal(D.readout(s, trg, att, W0, b_r), D.readout(s, trg, att * 3 + 1, W0, b_r))


# ---- beam-search step ----------------------------------------------------------------------------------------------
def test_beam_hand_worked_example():
    want = np.loadtxt(os.path.join(HERE, "golden", "beam_case.txt"))
    sc, src, lab = D.beam_step(np.log([[1.0, 2.0, 5.0], [1.0, 1.0, 1.0]]), np.log([[0.5, 0.25]]), 2)
    np.testing.assert_allclose(np.exp(sc[0]), want[:2], rtol=1e-14)
    assert src[0].tolist() == want[2:4].tolist() and lab[0].tolist() == want[4:6].tolist()


def test_beam_brute_force_and_invariants():
    rng = np.random.default_rng(12)
    Q, beam, V = 3, 4, 9
    logits = rng.standard_normal((Q * beam, V)) * 2
    score = -rng.uniform(0, 5, (Q, beam))
    sc, src, lab = D.beam_step(logits, score, beam)
    for q in range(Q):
        cands = []
        for b in range(beam):
            row = logits[q * beam + b]
            lse = math.log(sum(math.exp(x) for x in row))
            cands += [(-(score[q, b] + x - lse), b * V + v) for v, x in enumerate(row)]
        cands.sort()
        for k in range(beam):
            assert abs(-cands[k][0] - sc[q, k]) < 1e-12 and cands[k][1] == src[q, k] * V + lab[q, k]
    assert np.all(np.diff(sc, axis=1) <= 0)                                           # best first
    sc2, src2, lab2 = D.beam_step(logits + rng.standard_normal((Q * beam, 1)) * 10, score, beam)   # softmax ignores a row shift
    np.testing.assert_allclose(sc2, sc, rtol=1e-12, atol=1e-12)
    assert np.array_equal(src2, src) and np.array_equal(lab2, lab)
    np.testing.assert_allclose(np.exp(D.log_softmax_rows(logits)).sum(axis=1), 1.0, rtol=1e-13)


def test_beam_ties_first_step_and_torch_topk():
    # uniform logits: every label has log-probability -log V; the best hypotheses win, labels ascending on ties
    sc, src, lab = D.beam_step(np.zeros((3, 5)), np.array([[-1.0, -0.5, -2.0]]), 3)
    np.testing.assert_allclose(sc[0], -0.5 - math.log(5), rtol=1e-14)
    assert src[0].tolist() == [1, 1, 1] and lab[0].tolist() == [0, 1, 2]
    # first step of a search: only hypothesis 0 is alive
    rng = np.random.default_rng(13)
    logits = rng.standard_normal((4, 7))
    sc, src, lab = D.beam_step(logits, np.array([[0.0, -np.inf, -np.inf, -np.inf]]), 4)
    assert src[0].tolist() == [0, 0, 0, 0] and lab[0].tolist() == np.argsort(-logits[0], kind="stable")[:4].tolist()
    # torch.log_softmax + torch.topk on tie-free data
    Q, beam, V = 5, 6, 50
    logits = rng.standard_normal((Q * beam, V)) * 3
    score = -rng.uniform(0, 3, (Q, beam))
    sc, src, lab = D.beam_step(logits, score, beam)
    cand = torch.from_numpy(score)[:, :, None] + torch.log_softmax(torch.from_numpy(logits), dim=1).view(Q, beam, V)
    top = torch.topk(cand.view(Q, -1), beam, dim=1)
    np.testing.assert_allclose(sc, top.values.numpy(), rtol=1e-12)
    assert np.array_equal(src * V + lab, top.indices.numpy())


def test_gather_rows_and_embed():
    st = np.arange(6 * 2).reshape(6, 2)
    src = np.array([[2, 0, 0], [1, 1, 2]])
    assert D.gather_rows(st, src, 3)[:, 0].tolist() == [4, 0, 0, 8, 8, 10]
    W, b = np.arange(12.0).reshape(4, 3), np.array([0.5, 0.5, 0.5])
    np.testing.assert_array_equal(D.embed(np.array([[3, 0]]), W, b), np.array([[9.5, 10.5, 11.5], [0.5, 1.5, 2.5]]))
