"""GPU parity of the attention step and the readout (lstm_attention_step, lstm_readout, called through the C ABI)
against oracle/decoder_oracle.py on identical seeded inputs.

Tolerances, relative to the largest oracle magnitude of each tensor: 1e-4 for the float outputs a and accum' (float
accumulation over A = 1000 terms, hardware exp / reciprocal inside tanh and softmax), 5e-3 for the bfloat16 outputs
att and readout (one rounding to 8 significant bits: at most 2^-8 = 3.9e-3 of the element, plus the above)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import decoder_oracle as D
from paper_1805_05225_amd import synth
from tests.gpu_util import check, dev

Bn = None
TOL_F32, TOL_BF16 = 1e-4, 5e-3


@pytest.fixture(scope="module", autouse=True)
def _binding():
    global Bn
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1805_05225_amd import binding
    Bn = binding
    yield


def _gpu_step(inp, src_lens=True, att=None):
    g = lambda k, dt="f32": dev(inp[k], dt)
    return Bn.attention_step(g("H", "bf16"), g("ctx", "bf16"), dev(inp["src_lens"]) if src_lens else None, inp["cfg"]["beam"], g("s", "bf16"),
                             g("W_s", "bf16"), g("b_s"), g("w_fb"), g("b_fb"), g("v"), inp["b_e"], g("accum"), att=att)


def _oracle_step(inp, src_lens=True):
    f = lambda k: inp[k].astype(np.float64)
    lens = inp["src_lens"] if src_lens else np.full(inp["cfg"]["Q"], inp["S"])
    return D.attention_step(f("H"), f("ctx"), lens, inp["cfg"]["beam"], f("s"), f("accum"), f("W_s").T, f("b_s"), f("w_fb"), f("b_fb"),
                            f("v"), inp["b_e"])


CASES = [dict(Q=3, beam=2, len_lo=1, len_hi=9, A=40, E=6, n=24),                 # tiny
         dict(Q=5, beam=12, len_lo=0, len_hi=37, A=1000, E=2000, n=1000),         # the paper's widths, ragged lengths, an empty sentence possible
         dict(Q=4, beam=1, len_lo=60, len_hi=70, A=300, E=514, n=136),            # no beam, S > 64, E not a multiple of 512
         dict(Q=2, beam=16, len_lo=5, len_hi=5, A=257, E=1026, n=72),             # widest beam, odd A
         dict(Q=7, beam=5, len_lo=1, len_hi=130, A=64, E=64, n=8),                # S > 128
         dict(Q=64, beam=12, len_lo=20, len_hi=80, A=1000, E=2000, n=1000),       # the benchmark's decoder step at its full size
         dict(Q=2, beam=16, len_lo=1024, len_hi=1024, A=64, E=128, n=16)]         # the largest S and beam the entry point takes


@pytest.mark.parametrize("over", CASES)
def test_attention_step_matches_oracle(over):
    inp = synth.make_decoder(**over)
    print("  attention step: S=%d Q=%d beam=%d A=%d E=%d n=%d lens=%s" % (inp["S"], over["Q"], over["beam"], over["A"], over["E"], over["n"],
                                                                          inp["src_lens"].tolist()), flush=True)
    got = _gpu_step(inp)
    torch.cuda.synchronize()
    a, acc, att, e = _oracle_step(inp)
    check("a", got["a"], a, TOL_F32)
    check("accum", got["accum"], acc, TOL_F32)
    check("att", got["att"], att, TOL_BF16)
    ga = got["a"].cpu().numpy()
    for r in range(inp["B"]):                                   # exact zeros at padded positions
        L = inp["src_lens"][r // over["beam"]]
        assert np.all(ga[r, L:] == 0) and np.all(got["accum"][r, L:].cpu().numpy() == 0)
        if L == 0:
            assert np.all(got["att"][r].float().cpu().numpy() == 0)


def test_attention_step_without_lengths_and_into_a_wider_row():
    inp = synth.make_decoder(Q=3, beam=4, len_lo=11, len_hi=11, A=128, E=256, n=64)
    wide = torch.full((inp["B"], 64 + 20 + 256), 7.0, dtype=torch.bfloat16, device="cuda")
    got = _gpu_step(inp, src_lens=False, att=wide[:, 84:])
    torch.cuda.synchronize()
    a, acc, att, e = _oracle_step(inp, src_lens=False)
    check("a", got["a"], a, TOL_F32)
    check("att", wide[:, 84:], att, TOL_BF16)
    assert torch.all(wide[:, :84] == 7.0)                       # nothing outside the att columns was touched


def test_padding_values_are_never_read():
    inp = synth.make_decoder(Q=4, beam=3, len_lo=2, len_hi=20, A=96, E=128, n=32)
    ref = _gpu_step(inp)
    bad = dict(inp)
    for k in ("H", "ctx"):
        t = inp[k].copy()
        for q, L in enumerate(inp["src_lens"]):
            t[L:, q] = np.nan
        bad[k] = t
    acc = inp["accum"].copy()
    for r in range(inp["B"]):
        acc[r, inp["src_lens"][r // 3]:] = np.nan
    bad["accum"] = acc
    got = _gpu_step(bad)
    torch.cuda.synchronize()
    for k in ("a", "accum", "att"):
        assert torch.equal(ref[k], got[k]), k


def test_readout_matches_oracle():
    inp = synth.make_decoder(Q=5, beam=12, len_lo=3, len_hi=9, A=8, E=2000, n=1000)
    f = lambda k: inp[k].astype(np.float64)
    att = np.asarray(torch.from_numpy(np.random.default_rng(1).uniform(-1, 1, (inp["B"], 2000))).to(torch.bfloat16).float())
    # trg and att as the two halves of the cell's input rows (row stride 2620), s by itself
    xin = dev(np.concatenate([inp["trg"], att], axis=1), "bf16")
    out = Bn.readout(dev(inp["s"], "bf16"), xin[:, :620], xin[:, 620:], dev(inp["W_r"], "bf16"), dev(inp["b_r"]))
    torch.cuda.synchronize()
    ref = D.readout(f("s"), f("trg"), att.astype(np.float64), f("W_r").T, f("b_r"))
    check("readout", out, ref, TOL_BF16)
    assert (out == 0).any() and (out > 0).any()
    # a small, ragged shape through the same entry point (K = 5 + 3 + 7: not a multiple of 8)
    rng = np.random.default_rng(2)
    bfr = lambda a: torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    s2, t2, a2 = bfr(rng.standard_normal((7, 5))), bfr(rng.standard_normal((7, 3))), bfr(rng.standard_normal((7, 7)))
    W2, b2 = bfr(rng.standard_normal((9, 15))), rng.standard_normal(9).astype(np.float32)
    out2 = Bn.readout(dev(s2, "bf16"), dev(t2, "bf16"), dev(a2, "bf16"), dev(W2, "bf16"), dev(b2))
    check("readout small", out2, D.readout(s2, t2, a2, W2.astype(np.float64).T, b2.astype(np.float64)), TOL_BF16)


def test_hoisted_enc_ctx_through_lstm_gemm():
    """"enc_ctx" is computed once per sentence by the caller; with lstm_gemm that is one product over all S*Q positions."""
    rng = np.random.default_rng(3)
    bfr = lambda a: torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    S, Q, E, A = 13, 5, 64, 40
    H, W, b = bfr(rng.uniform(-1, 1, (S, Q, E))), bfr(rng.uniform(-.2, .2, (E, A))), rng.uniform(-.1, .1, A).astype(np.float32)
    C = Bn.gemm(dev(H.reshape(S * Q, E), "bf16"), dev(W, "bf16"), a_kcontig=True, b_kcontig=False, M=S * Q, N=A, K=E, bias=dev(b),
                out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    check("enc_ctx", C, D.enc_ctx(H, W, b).reshape(S * Q, A), TOL_BF16)
