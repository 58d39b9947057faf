"""CPU oracle for one step of the attention decoder (everything between the stepped LSTM cell and the readout) and for
one step of the batched beam search that follows it.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
may import it.  It shares nothing with the HIP path and never imports it.  All arithmetic is numpy float64; the
library primitives used as steps are `@`, `np.exp`, `np.log`, `np.tanh`, `np.maximum` and a stable `np.argsort`.

What it computes.  The paper gives the decoder as a network definition (Listing 1, the sub-network of layer "output"),
not as equations.  Written out, with j a source position, r a row of the decoder batch and q(r) the sentence the row
belongs to, one step is

    s_tr[r]      = s[r] W_s + b_s                                   ("s_tr": linear from the cell output s)
    fb[j, r]     = accum[r, j] w_fb + b_fb                          ("weight_feedback": linear from the accumulated weights)
    e[r, j]      = v . tanh(ctx[j, q(r)] + fb[j, r] + s_tr[r]) + b_e   ("e_in" add, "e_tanh", "e": linear to one output)
    a[r, :]      = softmax of e[r, :] over the positions j < src_lens[q(r)]    ("a": softmax over the source axis)
    accum'[r, j] = accum[r, j] + a[r, j]                            ("accum_a")
    att[r]       = sum_j a[r, j] H[j, q(r)]                         ("att": attention-weighted sum of the encoder states)
    readout[r]   = max(0, [s[r], trg[r], att[r]] W_r + b_r)         ("readout": linear with relu)

with ctx = H W_ctx + b_ctx ("enc_ctx") computed once per sentence, outside the loop (Sec. 7: work that does not depend
on the loop is moved out of it).  The cell that produces s from the previous step's trg and att is the stepped LSTM of
lstm_oracle.lstm_fwd with T = 1.

Readings (conventions of this repository; the listing fixes none of them):
  * the decoder batch holds `beam` hypotheses per sentence, those of one sentence next to each other: q(r) = r // beam
    (Sec. 3, Table 2: beam 12);
  * accum has one number per source position (the listing's "accum_a" adds the weights, which have one), so
    "weight_feedback" is a linear map from 1 to A values: a weight vector w_fb[A] and a bias b_fb[A];
  * positions j >= src_lens[q] take no part: a, accum' and the sum for att are 0 there, values stored there in ctx, H or
    accum are never read; a sentence of length 0 gives a = 0, att = 0;
  * Sec. 4 mentions an inverse form of the fertility feedback; the listing, which is what is built here, feeds the
    plain accumulated weights back.

Pins (tests/test_decoder_oracle_pins.py): closed forms (v = 0 gives uniform weights and att = mean of the valid encoder
states; one dominant energy gives att = that state), invariance under a shift of b_e, sum of a = 1 and accum' - accum = a,
NaN at padded positions, equivariance under a permutation of the valid source positions, independence of rows and
sharing inside a beam, a hand-worked example (tests/golden/attention_case.txt), brute force with scalar loops, and
torch.nn.functional softmax / bmm as an independent evaluation of the same step.

The beam-search step (beam_step, gather_rows, embed; described in the comment above them) is pinned by a hand-worked
example (tests/golden/beam_case.txt), brute force over all candidates, shift invariance of the softmax, the tie rule
on uniform logits, the first step of a search, and torch.log_softmax + torch.topk on tie-free data.
"""
import numpy as np

F64 = np.float64


def enc_ctx(H, W_ctx, b_ctx=None):
    """ctx[j, q, :] = H[j, q, :] W_ctx + b_ctx for every source position: loop-invariant, computed once per sentence
    (Listing 1, "enc_ctx")."""
    H = np.asarray(H, dtype=F64)
    out = H @ np.asarray(W_ctx, dtype=F64)
    if b_ctx is not None:
        out = out + np.asarray(b_ctx, dtype=F64)
    return out


def attention_step(H, ctx, src_lens, beam, s, accum, W_s, b_s, w_fb, b_fb, v, b_e):
    """One attention step (Listing 1: "s_tr", "weight_feedback", "e_in", "e_tanh", "e", "a", "accum_a", "att").

    H[S,Q,E], ctx[S,Q,A], src_lens[Q], s[B,n] with B = Q*beam, accum[B,S], W_s[n,A], b_s[A], w_fb[A], b_fb[A], v[A],
    b_e scalar  ->  a[B,S], accum'[B,S], att[B,E], e[B,S] (e is 0 at padded positions)."""
    H = np.asarray(H, dtype=F64)
    ctx = np.asarray(ctx, dtype=F64)
    s = np.asarray(s, dtype=F64)
    accum = np.asarray(accum, dtype=F64)
    W_s, b_s, w_fb, b_fb, v = (np.asarray(t, dtype=F64) for t in (W_s, b_s, w_fb, b_fb, v))
    S, Q, E = H.shape
    B = s.shape[0]
    assert B == Q * beam and accum.shape == (B, S) and ctx.shape[:2] == (S, Q)
    s_tr = s @ W_s + b_s
    a = np.zeros((B, S), dtype=F64)
    e = np.zeros((B, S), dtype=F64)
    att = np.zeros((B, E), dtype=F64)
    new_accum = np.zeros((B, S), dtype=F64)
    for r in range(B):
        q = r // beam
        L = int(min(max(int(src_lens[q]), 0), S))
        if L == 0:
            continue
        for j in range(L):
            fb = accum[r, j] * w_fb + b_fb
            e[r, j] = v @ np.tanh(ctx[j, q] + fb + s_tr[r]) + b_e
        w = np.exp(e[r, :L] - e[r, :L].max())
        a[r, :L] = w / w.sum()
        new_accum[r, :L] = accum[r, :L] + a[r, :L]
        att[r] = a[r, :L] @ H[:L, q]
    return a, new_accum, att, e


def readout(s, trg, att, W_r, b_r):
    """readout = relu([s, trg, att] W_r + b_r) (Listing 1, "readout"); W_r rows ordered s | trg | att."""
    x = np.concatenate([np.asarray(s, dtype=F64), np.asarray(trg, dtype=F64), np.asarray(att, dtype=F64)], axis=1)
    return np.maximum(x @ np.asarray(W_r, dtype=F64) + np.asarray(b_r, dtype=F64), 0.0)


# ---- one step of batched beam search -------------------------------------------------------------------------------
# The paper decodes with a batched beam search that runs on the GPU, beam size 12 (Sec. 3, Table 2, the decoding-speed table
# and the paragraph before it); it gives no further detail.  Listing 1 supplies the pieces around it: "output_prob" is a
# softmax over the labels computed from "readout", "output" chooses labels from it, and "trg" embeds the chosen label
# for the next step.  Reading of this repository for one step, with q a sentence, b one of its `beam` hypotheses
# (row r = q * beam + b) and v a label:
#     logp[r, v]   = logits[r, v] - log sum_v' exp(logits[r, v'])                  (log of the softmax)
#     cand[q, b, v] = score[q, b] + logp[r, v]
#     the `beam` largest cand[q, :, :] become the new hypotheses of sentence q, best first; each remembers the
#     hypothesis b it extends (src) and its label v.  Equal candidates are ordered by the smaller flat index b * V + v.
# A hypothesis with score -inf (used for the unused slots of the very first step) never wins against a finite one.
# Handling of finished hypotheses and length normalisation are not described by the paper and not part of this step.
# Afterwards every per-hypothesis state row (cell h and c, accumulated attention weights) of the new hypothesis k of
# sentence q is the row of the hypothesis it extends: new[q * beam + k] = old[q * beam + src[q, k]]  (gather_rows), and
# the next target embedding is the row `label` of the embedding table plus its bias (Listing 1, "trg").
def log_softmax_rows(logits):
    x = np.asarray(logits, dtype=F64)
    m = x.max(axis=1, keepdims=True)
    return x - (m + np.log(np.exp(x - m).sum(axis=1, keepdims=True)))


def beam_step(logits, score, beam):
    """logits[Q*beam, V], score[Q, beam] -> new_score[Q, beam], src[Q, beam] (int), label[Q, beam] (int), best first."""
    score = np.asarray(score, dtype=F64)
    Q = score.shape[0]
    logp = log_softmax_rows(logits)
    V = logp.shape[1]
    assert logp.shape[0] == Q * beam and score.shape == (Q, beam) and beam <= beam * V
    new_score = np.zeros((Q, beam), dtype=F64)
    src = np.zeros((Q, beam), dtype=np.int64)
    label = np.zeros((Q, beam), dtype=np.int64)
    for q in range(Q):
        cand = (score[q][:, None] + logp[q * beam:(q + 1) * beam]).reshape(-1)
        order = np.argsort(-cand, kind="stable")[:beam]         # stable: equal candidates keep ascending flat index
        new_score[q] = cand[order]
        src[q] = order // V
        label[q] = order % V
    return new_score, src, label


def gather_rows(state, src, beam):
    """state[Q*beam, ...] -> the rows of the hypotheses that the new ones extend."""
    state = np.asarray(state)
    Q = src.shape[0]
    rows = (np.arange(Q)[:, None] * beam + np.asarray(src)).reshape(-1)
    return state[rows]


def embed(label, W_trg, b_trg=None):
    """trg[r] = W_trg[label[r]] + b_trg (Listing 1, "trg": a linear layer on the chosen label = a row of its weights)."""
    out = np.asarray(W_trg, dtype=F64)[np.asarray(label).reshape(-1)]
    return out if b_trg is None else out + np.asarray(b_trg, dtype=F64)
