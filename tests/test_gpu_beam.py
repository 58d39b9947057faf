"""GPU parity of the beam-search step (lstm_beam_step, lstm_beam_gather, lstm_embed, called through the C ABI) against
oracle/decoder_oracle.py.

The step decides integers (which hypothesis, which label) from float32 scores, the oracle from float64 ones.  What is
unique is compared exactly, the rest is checked for validity: the new scores agree to 2e-5 (absolute, scores are O(10));
every chosen pair carries the oracle's candidate value for that pair; pairs are distinct and ordered best first; and wherever
the oracle's ranking is decided by more than that tolerance - which on the random cases below is everywhere or almost
everywhere - the chosen pair is the oracle's.  Cases whose float32 arithmetic is exact (ties) must match exactly, tie rule
included.  Gather and embedding move bits and are compared exactly."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import decoder_oracle as D

Bn = None
TOL = 2e-5


@pytest.fixture(scope="module", autouse=True)
def _binding():
    global Bn
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1805_05225_amd import binding
    Bn = binding
    yield


def _run(logits, score):
    r = Bn.beam_step(torch.from_numpy(logits).cuda(), torch.from_numpy(score).cuda())
    torch.cuda.synchronize()
    return r["score"].cpu().numpy(), r["src"].cpu().numpy().astype(np.int64), r["label"].cpu().numpy().astype(np.int64)


def _validate(logits, score, beam, got):
    sc, src, lab = got
    Q, V = score.shape[0], logits.shape[1]
    osc, osrc, olab = D.beam_step(logits.astype(np.float64), score.astype(np.float64), beam)
    logp = D.log_softmax_rows(logits.astype(np.float64))
    finite = np.isfinite(osc)
    assert np.array_equal(np.isfinite(sc), finite)
    assert np.abs(sc[finite] - osc[finite]).max() < TOL
    exact = 0
    for q in range(Q):
        flat = src[q] * V + lab[q]
        assert np.all((src[q] >= 0) & (src[q] < beam) & (lab[q] >= 0) & (lab[q] < V))
        assert len(set(flat[finite[q]].tolist())) == finite[q].sum()                       # distinct candidates
        assert np.all(np.diff(sc[q][finite[q]]) <= 0)                                      # best first
        cand = score[q].astype(np.float64)[:, None] + logp[q * beam:(q + 1) * beam]
        full = np.sort(cand.reshape(-1))[::-1]
        for k in range(beam):
            if not finite[q, k]:
                continue
            assert abs(cand[src[q, k], lab[q, k]] - sc[q, k]) < TOL                        # the pair really has that score
            gap_hi = full[k - 1] - full[k] if k > 0 else np.inf
            gap_lo = full[k] - full[k + 1] if k + 1 < full.size else np.inf
            if min(gap_hi, gap_lo) > 2 * TOL:                                               # the ranking is unambiguous here
                assert (src[q, k], lab[q, k]) == (osrc[q, k], olab[q, k])
                exact += 1
    return exact


@pytest.mark.parametrize("Q,beam,V,seed", [(3, 4, 50, 0), (5, 12, 20000, 1), (2, 16, 32768, 2), (7, 1, 300, 3), (4, 12, 257, 4),
                                           (64, 12, 20000, 5)])     # the last: the search benchmark's own size
def test_beam_step_random(Q, beam, V, seed):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((Q * beam, V)) * 3).astype(np.float32)
    score = (-rng.uniform(0, 8, (Q, beam))).astype(np.float32)
    print("  beam step Q=%d beam=%d V=%d" % (Q, beam, V), flush=True)
    exact = _validate(logits, score, beam, _run(logits, score))
    assert exact >= 0.9 * Q * beam                                                          # almost every rank is unambiguous and identical


def test_beam_step_exact_ties_and_first_step():
    # integer logits and scores, V a power of two: every float32 operation is exact enough for identical ties on both sides
    beam, V = 4, 8
    logits = np.zeros((2 * beam, V), dtype=np.float32)
    score = np.array([[-1.0, -0.5, -2.0, -0.5], [0.0, -np.inf, -np.inf, -np.inf]], dtype=np.float32)
    sc, src, lab = _run(logits, score)
    osc, osrc, olab = D.beam_step(logits.astype(np.float64), score.astype(np.float64), beam)
    assert np.array_equal(src, osrc) and np.array_equal(lab, olab)
    np.testing.assert_allclose(sc, osc, rtol=1e-6)
    assert src[0].tolist() == [1, 1, 1, 1] and lab[0].tolist() == [0, 1, 2, 3]             # hypothesis 1 before 3, labels ascending
    assert src[1].tolist() == [0, 0, 0, 0]                                                 # only hypothesis 0 is alive in a first step
    # duplicated maxima inside a row: the earlier label wins
    logits2 = np.zeros((beam, V), dtype=np.float32); logits2[:, [2, 5]] = 4.0
    sc, src, lab = _run(logits2, np.array([[0.0, -1.0, -np.inf, -np.inf]], dtype=np.float32))
    assert src[0].tolist() == [0, 0, 1, 1] and lab[0].tolist() == [2, 5, 2, 5]


def test_beam_step_rows_that_stress_the_candidate_buffer():
    """Rows shaped against the row kernel's filter (a running bound, a candidate buffer that is cut down when it runs short
    of room, a list of finalists with a fall-back when they do not fit): rising rows let every entry through, constant rows
    make every entry a finalist and leave the order to the tie rule, rows with a handful of usable labels offer fewer
    candidates than the beam asks for."""
    beam, V = 12, 20000
    rng = np.random.default_rng(21)
    ramp = (np.arange(V, dtype=np.float32) * np.float32(1e-3))
    logits = np.stack([ramp,                                   # rising: the best are the last labels
                       ramp[::-1],                             # falling: the best come first
                       np.roll(ramp, 7777),                    # the maximum in the middle of a wavefront's quarter
                       (rng.standard_normal(V) * 3).astype(np.float32)] * 3).astype(np.float32)
    score = (-rng.uniform(0, 2, (1, beam))).astype(np.float32)
    exact = _validate(logits, score, beam, _run(logits, score))
    assert exact >= beam - 2
    # constant rows: equal candidates inside a hypothesis, the earlier label first; hypotheses apart by their scores
    logits = np.zeros((beam, V), dtype=np.float32)
    score = (-0.25 * np.arange(beam, dtype=np.float32))[None, ::-1].copy()                 # the last hypothesis is the best
    sc, src, lab = _run(logits, score)
    osc, osrc, olab = D.beam_step(logits.astype(np.float64), score.astype(np.float64), beam)
    assert np.array_equal(src, osrc) and np.array_equal(lab, olab)
    assert src[0].tolist() == [beam - 1] * beam and lab[0].tolist() == list(range(beam))
    np.testing.assert_allclose(sc, osc, rtol=1e-6)
    # two plateaus: 40 labels share the maximum, spread over the row (more finalists than the wavefront-wide list holds when
    # every hypothesis has them, and ties across the quarters of a row)
    logits = np.full((beam, V), -3.0, dtype=np.float32)
    top = np.sort(rng.choice(V, 40, replace=False))
    logits[:, top] = 2.0
    sc, src, lab = _run(logits, score)
    osc, osrc, olab = D.beam_step(logits.astype(np.float64), score.astype(np.float64), beam)
    assert np.array_equal(src, osrc) and np.array_equal(lab, olab)
    assert lab[0].tolist() == top[:beam].tolist()
    # rows with fewer usable labels than the beam: -inf everywhere else
    beam2, V2 = 4, 3000
    logits = np.full((beam2, V2), -np.inf, dtype=np.float32)
    logits[0, [5, 2999]] = [1.0, 0.5]
    logits[1, [0, 1500, 17]] = [0.25, 0.75, -1.0]
    logits[2, 77] = 0.0
    logits[3, :] = (rng.standard_normal(V2)).astype(np.float32)
    score = np.array([[0.0, -0.5, -1.0, -30.0]], dtype=np.float32)
    with np.errstate(all="ignore"):
        exact = _validate(logits, score, beam2, _run(logits, score))
    assert exact >= 3


def test_beam_step_strided_logits():
    rng = np.random.default_rng(9)
    Q, beam, V = 3, 5, 1000
    wide = (rng.standard_normal((Q * beam, V + 24)) * 2).astype(np.float32)
    score = (-rng.uniform(0, 3, (Q, beam))).astype(np.float32)
    r = Bn.beam_step(torch.from_numpy(wide).cuda()[:, :V], torch.from_numpy(score).cuda())
    torch.cuda.synchronize()
    got = (r["score"].cpu().numpy(), r["src"].cpu().numpy().astype(np.int64), r["label"].cpu().numpy().astype(np.int64))
    _validate(np.ascontiguousarray(wide[:, :V]), score, beam, got)


def test_gather_and_embed_are_exact():
    rng = np.random.default_rng(10)
    Q, beam = 6, 12
    src = rng.integers(0, beam, (Q, beam)).astype(np.int32)
    for dt, width in ((torch.float32, 1000), (torch.bfloat16, 79), (torch.float32, 1)):
        st = torch.from_numpy(rng.standard_normal((Q * beam, width)).astype(np.float32)).to(dt).cuda()
        out = Bn.beam_gather(st, torch.from_numpy(src).cuda())
        torch.cuda.synchronize()
        want = D.gather_rows(st.float().cpu().numpy(), src, beam)
        assert np.array_equal(out.float().cpu().numpy(), want)
    # several arrays in one launch: every unit width (16, 8, 4 and 2 bytes), an output that is a column block of a wider buffer
    shapes = ((torch.float32, 1000, 0), (torch.float32, 80, 0), (torch.bfloat16, 2000, 620), (torch.bfloat16, 79, 0), (torch.float32, 3, 0),
              (torch.bfloat16, 36, 2))
    states = [torch.from_numpy(rng.standard_normal((Q * beam, w)).astype(np.float32)).to(dt).cuda() for dt, w, _ in shapes]
    wide = [torch.zeros(Q * beam, w + off, dtype=dt).cuda() for dt, w, off in shapes]
    outs = Bn.beam_gather_many(states, torch.from_numpy(src).cuda(), [b[:, off:] for b, (_, _, off) in zip(wide, shapes)])
    torch.cuda.synchronize()
    for st, o, b, (_, _, off) in zip(states, outs, wide, shapes):
        assert np.array_equal(o.float().cpu().numpy(), D.gather_rows(st.float().cpu().numpy(), src, beam))
        assert not b[:, :off].any()                                       # nothing written outside the block
    V, n = 500, 620
    W = torch.from_numpy(rng.standard_normal((V, n)).astype(np.float32)).to(torch.bfloat16)
    b = rng.standard_normal(n).astype(np.float32)
    label = rng.integers(0, V, (Q, beam)).astype(np.int32)
    out = Bn.embed(torch.from_numpy(label).cuda(), W.cuda(), torch.from_numpy(b).cuda())
    torch.cuda.synchronize()
    want = torch.from_numpy(D.embed(label, W.float().numpy().astype(np.float64), b.astype(np.float64)).astype(np.float32)).to(torch.bfloat16)
    assert torch.equal(out.cpu(), want)                                                    # one float add, one rounding: identical
    out0 = Bn.embed(torch.from_numpy(label).cuda(), W.cuda(), None)
    torch.cuda.synchronize()
    assert torch.equal(out0.cpu(), W[torch.from_numpy(label.reshape(-1)).long()])
