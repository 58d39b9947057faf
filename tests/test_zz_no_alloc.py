"""lstm_beam_step_static (the beam-search step for callers that cannot allocate: its scratch is a device array inside the
library) against lstm_beam_step (the same step with a caller-supplied workspace), through the C ABI.

Both run the same kernels, so every output must agree bit for bit.  Two calls in a row, the second with a smaller
problem, so that whatever the first call left in the shared array cannot leak into the second; then the size limit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(Bn, Q, beam, V, seed, first_step=False):
    rng = np.random.default_rng(seed)
    logits = torch.from_numpy((rng.standard_normal((Q * beam, V)) * 3).astype(np.float32)).cuda()
    score = (rng.standard_normal((Q, beam)) * 2).astype(np.float32)
    if first_step:
        score[:, 1:] = -np.inf                      # only hypothesis 0 is alive before the first choice
    score = torch.from_numpy(score).cuda()
    print("  static beam step Q=%d beam=%d V=%d seed=%d" % (Q, beam, V, seed), flush=True)
    ref = Bn.beam_step(logits, score)
    got = Bn.beam_step_static(logits, score)
    torch.cuda.synchronize()
    for name in ("score", "src", "label"):
        a, b = ref[name].cpu().numpy(), got[name].cpu().numpy()
        assert np.array_equal(a, b, equal_nan=True), (name, Q, beam, V)
    return got


def test_static_scratch_matches_workspace_two_calls():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1805_05225_amd import binding as Bn
    _case(Bn, 64, 12, 20000, 1)                     # the search benchmark's size
    _case(Bn, 3, 5, 777, 2)                         # smaller, right behind it: stale entries of the first call stay unread
    _case(Bn, 7, 16, 1031, 3, first_step=True)
    _case(Bn, 256, 16, 40, 4)                       # exactly at the limit Q * beam * beam = 65536


def test_static_scratch_rejects_sizes_beyond_the_array():
    from paper_1805_05225_amd import binding as Bn
    Q, beam, V = 257, 16, 8
    logits = torch.zeros(Q * beam, V, device="cuda")
    score = torch.zeros(Q, beam, device="cuda")
    with pytest.raises(Bn.LstmError) as e:
        Bn.beam_step_static(logits, score)
    assert e.value.status == -6
