"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on identical inputs.

Tolerances (relative to the largest oracle magnitude of each tensor): 1e-4 for float storage,
2e-2 for bfloat16 storage with float state.  The oracle always gets the storage-rounded inputs.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import lstm_oracle as O
from paper_1805_05225_amd import synth
from tests.gpu_util import TOL, check, dev, host, tdtype

Bn = None


@pytest.fixture(scope="module", autouse=True)
def _binding():
    global Bn
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1805_05225_amd import binding
    Bn = binding
    yield


def rnd_case(rng, T, B, n_in, n, D, lens, dt, scale=0.3, with_state=True, with_bias=True):
    """Random layer problem with every optional input present; values pre-rounded to the storage type."""
    def r(a):
        t = torch.from_numpy(a).to(torch.float32)
        return (t.to(torch.bfloat16).to(torch.float32) if dt == "bf16" else t).numpy().astype(np.float64)
    c = dict(x=r(rng.standard_normal((T, B, n_in))), W_x=r(rng.uniform(-scale, scale, (D, n_in, 4 * n))),
             W_h=r(rng.uniform(-scale, scale, (D, n, 4 * n))), lens=None if lens is None else np.asarray(lens, dtype=np.int32),
             dy=r(rng.standard_normal((T, B, D * n))))
    f32 = lambda a: a.astype(np.float32).astype(np.float64)
    c["b"] = f32(rng.uniform(-scale, scale, (D, 4 * n))) if with_bias else None
    for k in ("h0", "c0", "dhT", "dcT"):
        c[k] = f32(rng.standard_normal((D, B, n)) * 0.5) if with_state else None
    return c


def run_gpu(c, dt, bidir, direction=1, x_override=None, dy_override=None, flags=0, poison=False):
    sq = (lambda a: a) if bidir else (lambda a: None if a is None else a[0])
    x = dev(c["x"] if x_override is None else x_override, dt)
    dy = dev(c["dy"] if dy_override is None else dy_override, dt)
    Wx, Wh = dev(sq(c["W_x"]), dt), dev(sq(c["W_h"]), dt)
    b, h0, c0 = dev(sq(c["b"])), dev(sq(c["h0"])), dev(sq(c["c0"]))
    dhT, dcT = dev(sq(c["dhT"])), dev(sq(c["dcT"]))
    lens = dev(c["lens"]) if c["lens"] is not None else None
    f = Bn.forward(x, Wx, Wh, b, h0, c0, lens, bidirectional=bidir, direction=direction, flags=flags, poison=poison)
    assert not Bn.sync_status(f["workspace"]), "a bounded wait expired in the forward kernel"
    g = Bn.backward(f, x, Wx, Wh, h0, c0, lens, dy, dhT, dcT)
    assert not Bn.sync_status(f["workspace"]), "a bounded wait expired in the backward kernel"
    torch.cuda.synchronize()
    return f, g


def run_oracle(c, bidir, direction=1):
    if bidir:
        f = O.blstm_fwd(c["x"], c["W_x"], c["W_h"], c["b"], c["h0"], c["c0"], c["lens"])
        g = O.blstm_bwd(c["x"], c["W_x"], c["W_h"], c["b"], c["h0"], c["c0"], c["lens"], c["dy"], c["dhT"], c["dcT"])
    else:
        z = lambda a: None if a is None else a[0]
        f = O.lstm_fwd(c["x"], c["W_x"][0], c["W_h"][0], z(c["b"]), z(c["h0"]), z(c["c0"]), c["lens"], direction)
        g = O.lstm_bwd(c["x"], c["W_x"][0], c["W_h"][0], z(c["b"]), z(c["h0"]), z(c["c0"]), c["lens"], direction, c["dy"],
                       z(c["dhT"]), z(c["dcT"]))
    return f, g


def compare(f, g, fo, go, tol):
    for name, got, ref in (("y", f["y"], fo[0]), ("c", f["c"], fo[1]), ("hT", f["hT"], fo[2]), ("cT", f["cT"], fo[3]),
                           ("dx", g["dx"], go[0]), ("dW_x", g["dW_x"], go[1]), ("dW_h", g["dW_h"], go[2]),
                           ("db", g["db"], go[3]), ("dh0", g["dh0"], go[4]), ("dc0", g["dc0"], go[5])):
        check(name, got, ref, tol)


# ---- the hoisted GEMM by itself -----------------------------------------------------------------------
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("M,N,K", [(130, 140, 70), (257, 129, 620), (5, 7, 3), (256, 256, 256), (300, 520, 136), (1000, 260, 2048),
                                   (300, 520, 160), (513, 300, 4096), (40, 1030, 32), (264, 520, 200), (40, 4096, 333), (1024, 256, 64),
                                   (300, 520, 1000), (520, 300, 4000), (260, 260, 8), (260, 260, 72)])
def test_gemm_layouts(dt, M, N, K):
    rng = np.random.default_rng(M * 1000 + N + K)
    td = tdtype(dt)
    A = torch.from_numpy(rng.standard_normal((M, K))).to(td)
    B = torch.from_numpy(rng.standard_normal((K, N))).to(td)
    bias = torch.from_numpy(rng.standard_normal(N)).float()
    ref = A.double() @ B.double()
    tol = 1e-5 if dt == "f32" else 1e-5          # inputs are exact in both cases; only accumulation order differs
    Ad, Bd = A.cuda(), B.cuda()
    print("  gemm", dt, M, N, K, flush=True)
    C = Bn.gemm(Ad, Bd, a_kcontig=True, b_kcontig=False, M=M, N=N, K=K, bias=bias.cuda())
    check("NN", C, (ref + bias.double()).numpy(), tol)
    C = Bn.gemm(Ad, Bd.t().contiguous(), a_kcontig=True, b_kcontig=True, M=M, N=N, K=K)
    check("NT", C, ref.numpy(), tol)
    C0 = torch.from_numpy(rng.standard_normal((M, N))).float().cuda()
    C = Bn.gemm(Ad.t().contiguous(), Bd, a_kcontig=False, b_kcontig=False, M=M, N=N, K=K, C=C0.clone(), accumulate=True)
    check("TN+acc", C, (ref + C0.cpu().double()).numpy(), tol)
    C = Bn.gemm(Ad.t().contiguous(), Bd, a_kcontig=False, b_kcontig=False, M=M, N=N, K=K)
    check("TN", C, ref.numpy(), tol)
    if dt == "bf16":
        C = Bn.gemm(Ad, Bd.t().contiguous(), a_kcontig=True, b_kcontig=True, M=M, N=N, K=K, out_dtype=torch.bfloat16)
        check("NT->bf16", C, ref.numpy(), 1e-2)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_gemm_frame_mask_ignores_nan_rows(dt):
    rng = np.random.default_rng(3)
    T, Bt, M, N = 9, 5, 37, 45
    lens = np.array([9, 0, 4, 7, 1], dtype=np.int32)
    td = tdtype(dt)
    X = torch.from_numpy(rng.standard_normal((T * Bt, M))).to(td)
    DZ = torch.from_numpy(rng.standard_normal((T * Bt, N))).to(td)
    valid = (np.arange(T)[:, None] < lens[None, :]).reshape(-1)
    Xn = X.clone()
    Xn[torch.from_numpy(~valid)] = float("nan")
    ref = (X.double() * torch.from_numpy(valid)[:, None]).t() @ DZ.double()
    C = Bn.gemm(Xn.cuda(), DZ.cuda(), a_kcontig=False, b_kcontig=False, M=M, N=N, K=T * Bt, lens=torch.from_numpy(lens).cuda(),
                Bt=Bt, T=T)
    check("masked TN", C, ref.numpy(), 1e-5)


# ---- small odd shapes, every optional input, both dtypes ------------------------------------------------
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("direction", [1, -1])
def test_lstm_small_odd_shapes(dt, direction):
    rng = np.random.default_rng(42 + direction)
    c = rnd_case(rng, T=7, B=5, n_in=7, n=20, D=1, lens=[7, 0, 3, 5, 1], dt=dt)
    print("  lstm small", dt, direction, flush=True)
    f, g = run_gpu(c, dt, False, direction)
    fo, go = run_oracle(c, False, direction)
    compare(f, g, fo, go, TOL[dt])
    assert (host(f["y"])[3:, 2] == 0).all() and (host(g["dx"])[:, 1] == 0).all()


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_blstm_small_odd_shapes(dt):
    rng = np.random.default_rng(43)
    c = rnd_case(rng, T=9, B=35, n_in=12, n=36, D=2, lens=list(rng.integers(0, 10, 35)), dt=dt)
    c["lens"][0] = 9
    print("  blstm small", dt, flush=True)
    f, g = run_gpu(c, dt, True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL[dt])


def test_optional_inputs_null_and_T1_B1():
    rng = np.random.default_rng(44)
    c = rnd_case(rng, T=1, B=1, n_in=3, n=5, D=1, lens=None, dt="f32", with_state=False, with_bias=False)
    c["lens"] = None
    f, g = run_gpu(c, "f32", False, 1)
    fo, go = run_oracle(c, False, 1)
    compare(f, g, fo, go, TOL["f32"])


# ---- padding invariance on the GPU: NaN in every padded frame of x and dy ---------------------------------
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_padding_nan_never_reaches_results(dt):
    rng = np.random.default_rng(45)
    lens = [6, 2, 0, 4]
    c = rnd_case(rng, T=8, B=4, n_in=10, n=24, D=2, lens=lens, dt=dt)
    xn, dyn = c["x"].copy(), c["dy"].copy()
    for b, L in enumerate(lens):
        xn[L:, b] = np.nan
        dyn[L:, b] = np.nan
    # reserve and workspace start as all-ones bytes (NaN as float and as bfloat16): the forward pass leaves the gate
    # pre-activations of padded frames unwritten, and nothing may ever read them
    f, g = run_gpu(c, dt, True, x_override=xn, dy_override=dyn, poison=True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL[dt])


# ---- composition properties on the GPU ----------------------------------------------------------------------
def test_blstm_equals_two_lstm_and_stepping_equals_sequence():
    rng = np.random.default_rng(46)
    dt = "f32"
    c = rnd_case(rng, T=6, B=3, n_in=9, n=16, D=2, lens=[6, 4, 5], dt=dt)
    f, g = run_gpu(c, dt, True)
    for d, direction in enumerate((1, -1)):
        c1 = {k: (v[d:d + 1] if k in ("W_x", "W_h", "b", "h0", "c0", "dhT", "dcT") else v) for k, v in c.items()}
        c1["dy"] = c["dy"][:, :, d * 16:(d + 1) * 16]
        f1, g1 = run_gpu(c1, dt, False, direction)
        assert torch.equal(f["y"][:, :, d * 16:(d + 1) * 16], f1["y"]) and torch.equal(f["hT"][d], f1["hT"])
        assert torch.equal(g["dW_h"][d], g1["dW_h"]) and torch.equal(g["dh0"][d], g1["dh0"])
    # stepping: T calls with T = 1 in inference mode, state fed back
    x = dev(c["x"], dt)
    Wx, Wh, b = dev(c["W_x"][0], dt), dev(c["W_h"][0], dt), dev(c["b"][0])
    h, cc = dev(c["h0"][0]), dev(c["c0"][0])
    # T = 1 calls run the per-step kernel: bit for bit the sequence call on the same kernels (one launch per time step),
    # and to rounding the sequence call on its default path (one launch for the whole loop, another summation order)
    full = Bn.forward(x, Wx, Wh, b, h, cc, None, bidirectional=False, direction=1, flags=Bn.FLAG_PER_STEP)
    full_default = Bn.forward(x, Wx, Wh, b, h, cc, None, bidirectional=False, direction=1)
    for k in ("y", "hT", "cT"):
        check(k + " (paths)", full_default[k], host(full[k]), 1e-5)
    ys = []
    for t in range(6):
        s = Bn.forward(x[t:t + 1].clone(), Wx, Wh, b, h, cc, None, bidirectional=False, direction=1,
                       flags=Bn.FLAG_INFERENCE, want_c=False)
        h, cc = s["hT"], s["cT"]
        ys.append(s["y"][0])
    torch.cuda.synchronize()
    assert torch.equal(torch.stack(ys), full["y"]) and torch.equal(h, full["hT"]) and torch.equal(cc, full["cT"])


def test_accumulate_flag_adds_into_gradients():
    rng = np.random.default_rng(47)
    c = rnd_case(rng, T=5, B=4, n_in=6, n=8, D=1, lens=[5, 3, 4, 1], dt="f32")
    x, dy = dev(c["x"], "f32"), dev(c["dy"], "f32")
    Wx, Wh, b = dev(c["W_x"][0], "f32"), dev(c["W_h"][0], "f32"), dev(c["b"][0])
    lens = dev(c["lens"])
    f = Bn.forward(x, Wx, Wh, b, None, None, lens, bidirectional=False)
    g = Bn.backward(f, x, Wx, Wh, None, None, lens, dy)
    acc = (torch.ones_like(g["dW_x"]), torch.full_like(g["dW_h"], 2.0), torch.full_like(g["db"], 3.0))
    g2 = Bn.backward(f, x, Wx, Wh, None, None, lens, dy, accumulate_into=acc)
    torch.cuda.synchronize()
    assert torch.allclose(g2["dW_x"], g["dW_x"] + 1, atol=1e-5) and torch.allclose(g2["dW_h"], g["dW_h"] + 2, atol=1e-5)
    assert torch.allclose(g2["db"], g["db"] + 3, atol=1e-5)


def test_accumulate_with_split_k_bf16():
    """bf16 storage with enough frames that the weight-gradient products cut K into ranges (partial results summed by a
    second kernel): the accumulate flag must add the sum of the ranges to what the caller's buffers hold."""
    rng = np.random.default_rng(48)
    T, B, n_in, n = 300, 32, 24, 64
    lens = rng.integers(T // 2, T + 1, B)
    c = rnd_case(rng, T=T, B=B, n_in=n_in, n=n, D=2, lens=lens, dt="bf16", scale=0.1, with_state=False)
    x, dy = dev(c["x"], "bf16"), dev(c["dy"], "bf16")
    Wx, Wh, b = dev(c["W_x"], "bf16"), dev(c["W_h"], "bf16"), dev(c["b"])
    ln = dev(c["lens"])
    f = Bn.forward(x, Wx, Wh, b, None, None, ln, bidirectional=True)
    g = Bn.backward(f, x, Wx, Wh, None, None, ln, dy)
    acc = (torch.ones_like(g["dW_x"]), torch.full_like(g["dW_h"], 2.0), torch.full_like(g["db"], 3.0))
    g2 = Bn.backward(f, x, Wx, Wh, None, None, ln, dy, accumulate_into=acc)
    torch.cuda.synchronize()
    fo, go = run_oracle(c, True)
    check("dW_x", g["dW_x"], go[1], TOL["bf16"])
    check("dW_h", g["dW_h"], go[2], TOL["bf16"])
    scale = float(g["dW_h"].abs().max())
    assert torch.allclose(g2["dW_x"], g["dW_x"] + 1, atol=1e-3 * scale) and torch.allclose(g2["dW_h"], g["dW_h"] + 2, atol=1e-3 * scale)
    assert torch.allclose(g2["db"], g["db"] + 3, atol=1e-3 * float(g["db"].abs().max()))


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_all_rows_empty_and_single_frame_training(dt):
    """Degenerate batches: every length 0 (outputs zero, state and its gradient passed through, weight gradients zero), and
    T = 1 in training mode (forward + backward of a single frame)."""
    rng = np.random.default_rng(49)
    c = rnd_case(rng, T=6, B=5, n_in=16, n=24, D=2, lens=[0, 0, 0, 0, 0], dt=dt)
    f, g = run_gpu(c, dt, True)
    assert float(f["y"].float().abs().max()) == 0.0 and float(g["dx"].float().abs().max()) == 0.0
    assert float(g["dW_x"].abs().max()) == 0.0 and float(g["dW_h"].abs().max()) == 0.0 and float(g["db"].abs().max()) == 0.0
    check("hT", f["hT"], c["h0"], 1e-6)
    check("cT", f["cT"], c["c0"], 1e-6)
    check("dh0", g["dh0"], c["dhT"], 1e-6)
    check("dc0", g["dc0"], c["dcT"], 1e-6)
    c = rnd_case(rng, T=1, B=9, n_in=16, n=24, D=2, lens=[1, 1, 0, 1, 1, 1, 0, 1, 1], dt=dt)
    f, g = run_gpu(c, dt, True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL[dt])


# ---- the single-launch recurrent kernels against one launch per time step ------------------------------------
@pytest.mark.parametrize("dt,B,n,T", [("bf16", 32, 64, 40), ("f32", 5, 20, 9), ("bf16", 70, 136, 25), ("bf16", 32, 1024, 12), ("bf16", 19, 1000, 7),
                                      ("bf16", 64, 1000, 9), ("bf16", 41, 1024, 6), ("bf16", 150, 264, 8)])
def test_single_launch_equals_per_step(dt, B, n, T):
    rng = np.random.default_rng(B * n + T)
    lens = rng.integers(0, T + 1, B)
    lens[0] = T
    c = rnd_case(rng, T=T, B=B, n_in=24, n=n, D=2, lens=lens, dt=dt, scale=0.1)
    print("  single launch vs per step", dt, B, n, T, flush=True)
    f1, g1 = run_gpu(c, dt, True)
    f2, g2 = run_gpu(c, dt, True, flags=Bn.FLAG_PER_STEP)
    # the two paths sum over K in different orders, so they agree to rounding, not bit for bit
    for k in ("y", "c", "hT", "cT"):
        check(k + " (paths)", f1[k], host(f2[k]), 1e-5 if dt == "f32" else 1e-2)
    for k in ("dx", "dW_x", "dW_h", "db", "dh0", "dc0"):
        check(k + " (paths)", g1[k], host(g2[k]), 1e-5 if dt == "f32" else 1e-2)
    fo, go = run_oracle(c, True)
    compare(f1, g1, fo, go, TOL[dt])
    compare(f2, g2, fo, go, TOL[dt])


@pytest.mark.parametrize("B,n,T,bidir,direction", [(64, 1000, 12, True, 1), (70, 136, 9, True, 1), (3, 8, 33, True, 1),
                                                    (150, 264, 5, False, -1), (17, 1024, 6, False, 1), (33, 40, 2, True, 1),
                                                    (100, 1000, 4, True, 1), (64, 1000, 150, True, 1)])
def test_float_single_launch_loops(B, n, T, bidir, direction):
    """Float storage runs its time loops in one launch each (n a multiple of 8): rows of
    length 0, 1 and T, one to five slabs of 32 rows with ragged last slabs and, in the last case, more slabs than one launch
    holds, both directions and each alone, an initial cell state, and one long case (150 steps at the full width: the kernels
    consume ring loads while stores are in flight, and a wait that is one load short shows as a wrong row now and then);
    compared with one launch per time step, with the ordinary launch mode, and with the oracle."""
    rng = np.random.default_rng(7 * B + n + T)
    lens = rng.integers(0, T + 1, B)
    lens[0] = T
    if B > 2:
        lens[1], lens[2] = 0, 1
    c = rnd_case(rng, T=T, B=B, n_in=24, n=n, D=2 if bidir else 1, lens=lens, dt="f32", scale=0.1)
    if (B + T) % 2:                                    # without an initial hidden state in about half of the cases; with one, its
        c["h0"] = None                                 # values (N(0, 1/4), many beyond 1 - and times 8 below) never enter the ring
    else:
        c["h0"] = c["h0"] * 8.0
    # (the paths sum in different orders; with initial states of magnitude 10 their pre-activations differ by a few 1e-5)
    print("  float single launch", B, n, T, bidir, direction, flush=True)
    f1, g1 = run_gpu(c, "f32", bidir, direction)
    f2, g2 = run_gpu(c, "f32", bidir, direction, flags=Bn.FLAG_PER_STEP)
    f3, g3 = run_gpu(c, "f32", bidir, direction, flags=Bn.FLAG_PLAIN_LAUNCH)
    for k in ("y", "c", "hT", "cT"):
        check(k + " (paths)", f1[k], host(f2[k]), 5e-5)
        check(k + " (launch modes)", f3[k], host(f1[k]), 1e-5)
    for k in ("dx", "dW_x", "dW_h", "db", "dh0", "dc0"):
        check(k + " (paths)", g1[k], host(g2[k]), 5e-5)
        check(k + " (launch modes)", g3[k], host(g1[k]), 1e-5)
    fo, go = run_oracle(c, bidir, direction)
    compare(f1, g1, fo, go, TOL["f32"])


@pytest.mark.parametrize("B,n,T", [(32, 1024, 12), (64, 1000, 9), (41, 1024, 6), (70, 136, 25)])
def test_plain_launch_equals_cooperative(B, n, T):
    """LSTM_FLAG_PLAIN_LAUNCH starts the same kernels with an ordinary launch: same results (to the rounding of a
    different summation order where a stale ring load was repeated), no bounded wait expired, oracle parity."""
    rng = np.random.default_rng(3 * B + n + T)
    lens = rng.integers(0, T + 1, B)
    lens[0] = T
    c = rnd_case(rng, T=T, B=B, n_in=24, n=n, D=2, lens=lens, dt="bf16", scale=0.1)
    print("  plain launch vs cooperative", B, n, T, flush=True)
    f1, g1 = run_gpu(c, "bf16", True)
    f2, g2 = run_gpu(c, "bf16", True, flags=Bn.FLAG_PLAIN_LAUNCH)
    for k in ("y", "c", "hT", "cT"):
        check(k + " (launch modes)", f2[k], host(f1[k]), 1e-2)
    for k in ("dx", "dW_x", "dW_h", "db", "dh0", "dc0"):
        check(k + " (launch modes)", g2[k], host(g1[k]), 1e-2)
    fo, go = run_oracle(c, True)
    compare(f2, g2, fo, go, TOL["bf16"])


@pytest.mark.parametrize("B,n,T", [(19, 1000, 7), (40, 1024, 6), (32, 264, 12)])
def test_large_initial_state_single_launch(B, n, T):
    """Initial hidden states far outside (-1, 1), rows of length 0, 1 and T, both directions.  The single-launch forward
    kernels exchange h through units whose tag is a bit that |h| <= 1 leaves free; the initial state therefore never
    travels that way (its product with W_h is added to each row's first frame), and rows that have not started publish
    zeros.  Every output and gradient against the oracle."""
    rng = np.random.default_rng(11 * B + n + T)
    lens = rng.integers(0, T + 1, B)
    lens[0], lens[1], lens[2] = T, 0, 1
    c = rnd_case(rng, T=T, B=B, n_in=24, n=n, D=2, lens=lens, dt="bf16", scale=0.1)
    # |h0| up to about 25, on bf16 values: the path rounds the initial state to bf16 where it enters a product, and at this
    # magnitude that rounding alone would exceed the tolerance against an oracle that keeps the float values
    c["h0"] = torch.from_numpy(c["h0"] * 12.0).to(torch.bfloat16).to(torch.float64).numpy()
    print("  large initial state", B, n, T, "max |h0| %.1f" % np.abs(c["h0"]).max(), flush=True)
    f, g = run_gpu(c, "bf16", True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL["bf16"])
    c1 = rnd_case(rng, T=T, B=B, n_in=24, n=n, D=1, lens=lens, dt="bf16", scale=0.1)
    c1["h0"] = torch.from_numpy(c1["h0"] * 12.0).to(torch.bfloat16).to(torch.float64).numpy()
    for direction in (1, -1):
        f, g = run_gpu(c1, "bf16", False, direction)
        fo, go = run_oracle(c1, False, direction)
        compare(f, g, fo, go, TOL["bf16"])


def test_single_launch_random_shapes_bf16():
    """Seeded sweep over batch sizes, hidden sizes (multiples of 4 and not, below and above a 32-unit tile, padded
    and exact), lengths and directions: the single-launch kernels (or their fallbacks) against the oracle."""
    rng0 = np.random.default_rng(7)
    for it in range(12):
        B = int(rng0.choice([1, 3, 9, 16, 17, 32, 33, 64, 100]))
        n = int(rng0.choice([4, 20, 33, 36, 100, 132, 260, 500, 1000, 1024, 7]))
        T = int(rng0.integers(1, 30))
        uni = bool(rng0.integers(0, 2))
        rng = np.random.default_rng(500 + it)
        lens = rng.integers(0, T + 1, B)
        lens[rng.integers(0, B)] = T
        c = rnd_case(rng, T=T, B=B, n_in=int(rng0.choice([8, 24, 40])), n=n, D=1 if uni else 2, lens=lens, dt="bf16", scale=0.1)
        direction = int(rng0.choice([1, -1]))
        print("  random shape", it, "B", B, "n", n, "T", T, "uni %d" % direction if uni else "bi", flush=True)
        if uni:
            f, g = run_gpu(c, "bf16", False, direction)
            fo, go = run_oracle(c, False, direction)
        else:
            f, g = run_gpu(c, "bf16", True)
            fo, go = run_oracle(c, True)
        compare(f, g, fo, go, TOL["bf16"])


# ---- max-pooling in time between encoder layers: exact operation, bit-exact bar ---------------------------------
@pytest.mark.parametrize("dt", ["bf16", "f32"])
@pytest.mark.parametrize("T,B,F,pool", [(9, 4, 16, 2), (7, 3, 5, 3), (1, 2, 8, 2), (40, 33, 2048, 2), (13, 5, 264, 4), (6, 2, 24, 1)])
def test_time_pool_matches_oracle_exactly(dt, T, B, F, pool):
    rng = np.random.default_rng(T * 1000 + F + pool)
    lens = rng.integers(0, T + 1, B)
    lens[0] = T
    if B > 1:
        lens[1] = 0                                           # an empty row
    y = dev(rng.integers(-6, 7, (T, B, F)) * 0.25 if F == 16 else rng.standard_normal((T, B, F)), dt)      # F == 16: many ties
    yo = host(y)                                              # the oracle gets the storage-rounded values
    yo_nan = yo.copy()
    for b in range(B):
        yo_nan[lens[b]:, b, :] = np.nan                       # and must not look at padded frames
    out_o, lens_o, arg_o = O.time_maxpool_fwd(yo_nan, lens, pool)
    r = Bn.time_pool_fwd(y, dev(lens), pool)
    assert np.array_equal(host(r["out"]), out_o)
    assert np.array_equal(r["lens"].cpu().numpy(), lens_o)
    valid = (np.arange(out_o.shape[0])[:, None] < lens_o[None, :])[:, :, None]
    assert np.array_equal(np.where(valid, r["arg"].cpu().numpy(), 0), arg_o)
    dout = dev(rng.standard_normal(out_o.shape), dt)
    dy = Bn.time_pool_bwd(dout, r["arg"], dev(lens), pool, T)
    assert np.array_equal(host(dy), O.time_maxpool_bwd(host(dout), arg_o, lens, pool, T))
    # without lengths every row is full
    r2 = Bn.time_pool_fwd(y, None, pool, want_arg=False)
    assert np.array_equal(host(r2["out"]), O.time_maxpool_fwd(yo, None, pool)[0]) and r2["arg"] is None


def test_time_pool_full_size_of_the_pooled_encoder():
    """The first pooling of the pooled-encoder benchmark at its full size and in its launch configuration: T = 1491, B = 32,
    F = 2048 bfloat16, windows of 2, config 4's sequence lengths; every element of out, arg (at valid frames), lens and dy."""
    inp = synth.make(4, layers=1)
    T, B, F, pool = inp["T"], inp["cfg"]["B"], 2 * inp["cfg"]["n"], 2
    lens = inp["seq_lens"].astype(np.int64)
    g = torch.Generator(device="cpu").manual_seed(46)
    y = torch.randn(T, B, F, generator=g).to(torch.bfloat16).cuda()
    print("  pooling at full size: T=%d B=%d F=%d" % (T, B, F), flush=True)
    out_o, lens_o, arg_o = O.time_maxpool_fwd(host(y), lens, pool)
    r = Bn.time_pool_fwd(y, dev(inp["seq_lens"]), pool)
    assert np.array_equal(host(r["out"]), out_o) and np.array_equal(r["lens"].cpu().numpy(), lens_o)
    valid = (np.arange(out_o.shape[0])[:, None] < lens_o[None, :])[:, :, None]
    assert np.array_equal(np.where(valid, r["arg"].cpu().numpy(), 0), arg_o)
    dout = torch.randn(out_o.shape, generator=g).to(torch.bfloat16).cuda()
    dy = Bn.time_pool_bwd(dout, r["arg"], dev(inp["seq_lens"]), pool, T)
    assert np.array_equal(host(dy), O.time_maxpool_bwd(host(dout), arg_o, lens, pool, T))


def test_time_pool_unaligned_rows_and_strided_input():
    """Rows that are not 16-byte multiples (scalar path) and a pooled view of one direction's half of a wider tensor."""
    rng = np.random.default_rng(77)
    T, B, F, pool = 10, 3, 24, 2
    lens = np.array([10, 7, 3])
    wide = dev(rng.standard_normal((T, B, 2 * F + 3)), "bf16")
    y = wide[:, :, 3:3 + F]                                   # element-aligned only, leading dimension 2F + 3
    r = Bn.time_pool_fwd(y, dev(lens), pool)
    out_o, _, arg_o = O.time_maxpool_fwd(host(y), lens, pool)
    assert np.array_equal(host(r["out"]), out_o)
    dout = dev(rng.standard_normal(out_o.shape), "bf16")
    assert np.array_equal(host(Bn.time_pool_bwd(dout, r["arg"], dev(lens), pool, T)), O.time_maxpool_bwd(host(dout), arg_o, lens, pool, T))


# ---- the benchmark configurations ------------------------------------------------------------------------------
def _config_case(inp, layer=0):
    L = inp["layers"][layer]
    D = inp["D"]
    return dict(x=inp["x"].astype(np.float64), W_x=L["W_x"].astype(np.float64), W_h=L["W_h"].astype(np.float64),
                b=L["b"].astype(np.float64), h0=None, c0=None, dhT=None, dcT=None, lens=inp["seq_lens"],
                dy=inp["dy"].astype(np.float64))


def test_config1_unidirectional_f32():
    inp = synth.make(1)
    c = _config_case(inp)
    f, g = run_gpu(c, "f32", False, 1)
    fo, go = run_oracle(c, False, 1)
    compare(f, g, fo, go, TOL["f32"])


def test_config2_blstm_f32_full_size():
    inp = synth.make(2)
    c = _config_case(inp)
    print("  config 2: T=%d frames=%d" % (inp["T"], synth.real_frames(inp)), flush=True)
    f, g = run_gpu(c, "f32", True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL["f32"])


def _stack_gpu(inp, dt):
    lens = dev(inp["seq_lens"])
    cur = dev(inp["x"], dt)
    saved = []
    ws = None
    for L in inp["layers"]:
        Wx, Wh, b = dev(L["W_x"], dt), dev(L["W_h"], dt), dev(L["b"])
        f = Bn.forward(cur, Wx, Wh, b, None, None, lens, bidirectional=L["W_x"].shape[0] == 2, workspace=ws, want_state=False)
        ws = f["workspace"]
        saved.append((cur, Wx, Wh, f))
        cur = f["y"]
    y = cur
    d = dev(inp["dy"], dt)
    grads = [None] * len(saved)
    for k in range(len(saved) - 1, -1, -1):
        xin, Wx, Wh, f = saved[k]
        g = Bn.backward(f, xin, Wx, Wh, None, None, lens, d, want_dstate=False)
        grads[k] = g
        d = g["dx"]
    torch.cuda.synchronize()
    return y, d, grads


@pytest.mark.parametrize("k,over", [(3, dict(layers=2, len_lo=5, len_hi=24)), (4, dict(layers=2, len_lo=10, len_hi=40, B=32))])
def test_bf16_stack_reduced(k, over):
    inp = synth.make(k, **over)
    print("  config %d reduced: T=%d layers=%d" % (k, inp["T"], len(inp["layers"])), flush=True)
    y, dx, grads = _stack_gpu(inp, "bf16")
    layers = [{kk: v.astype(np.float64) for kk, v in L.items()} for L in inp["layers"]]
    acts, yo = O.blstm_stack_fwd(inp["x"].astype(np.float64), layers, inp["seq_lens"])
    dxo, go = O.blstm_stack_bwd(acts, layers, inp["seq_lens"], inp["dy"].astype(np.float64))
    tol = TOL["bf16"]
    check("y", y, yo, tol)
    check("dx", dx, dxo, tol)
    for l, (g, r) in enumerate(zip(grads, go)):
        check("dW_x%d" % l, g["dW_x"], r[0], tol)
        check("dW_h%d" % l, g["dW_h"], r[1], tol)
        check("db%d" % l, g["db"], r[2], tol)


@pytest.mark.parametrize("over", [dict(layers=4, len_lo=5, len_hi=24), dict(layers=3, len_lo=3, len_hi=40, B=32, n=1024),
                                  dict(layers=3, len_lo=0, len_hi=21, B=19, n=200, n_in=70)])
def test_mixed_encoder_stack_reduced(over):
    """One bidirectional layer below unidirectional ones (the translation encoder of the speed comparison), reduced in
    depth and length so that the oracle finishes in seconds: y of the top layer, dx of the bottom layer and every
    weight gradient against the oracle's mixed stack."""
    inp = synth.make(7, **over)
    print("  config 7 reduced: T=%d B=%d n=%d layers=%d" % (inp["T"], inp["cfg"]["B"], inp["cfg"]["n"], len(inp["layers"])), flush=True)
    y, dx, grads = _stack_gpu(inp, "bf16")
    layers = [{kk: v.astype(np.float64) for kk, v in L.items()} for L in inp["layers"]]
    acts, yo = O.encoder_stack_fwd(inp["x"].astype(np.float64), layers, inp["seq_lens"])
    dxo, go = O.encoder_stack_bwd(acts, layers, inp["seq_lens"], inp["dy"].astype(np.float64))
    tol = TOL["bf16"]
    check("y", y, yo, tol)
    check("dx", dx, dxo, tol)
    for l, (g, r) in enumerate(zip(grads, go)):
        check("dW_x%d" % l, g["dW_x"], r[0], tol)
        check("dW_h%d" % l, g["dW_h"], r[1], tol)
        check("db%d" % l, g["db"], r[2], tol)


@pytest.mark.timeout(900)
def test_config4_first_layer_full_size():
    """Config 4 at its full size (T = 1491, B = 32, n = 1024, bf16): the launch configuration the benchmark times
    (single-launch recurrent kernels on 256 work-groups, products over real frames only).  One layer, because the
    oracle's inputs must be synthetic: every output of the first layer is compared element by element.  The oracle
    needs about a minute for it."""
    inp = synth.make(4, layers=1)
    c = _config_case(inp)
    print("  config 4, first layer, full size: T=%d frames=%d" % (inp["T"], synth.real_frames(inp)), flush=True)
    f, g = run_gpu(c, "bf16", True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL["bf16"])



@pytest.mark.timeout(900)
def test_config4_deeper_layer_full_size():
    """A layer k > 1 of config 4 at its full size (n_in = 2n = 2048, T = 1491, B = 32, n = 1024, bf16): the shape five of
    the benchmark's six layers run, in the benchmark's launch configuration (products over the 31 597 real frames only,
    weight gradients with K cut into ranges).  Every output, dW_x, dW_h and db included, element by element against the
    oracle on all frames (about a minute and a half of oracle time)."""
    inp = synth.make(4, layers=1, n_in=2048)
    c = _config_case(inp)
    print("  config 4, deeper layer, full size: T=%d frames=%d" % (inp["T"], synth.real_frames(inp)), flush=True)
    f, g = run_gpu(c, "bf16", True, flags=Bn.FLAG_PLAIN_LAUNCH)          # the launch mode bench.py times
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL["bf16"])
    lens = inp["seq_lens"]
    b = int(np.argmin(lens))
    assert float(f["y"][lens[b]:, b].float().abs().max()) == 0.0 and float(g["dx"][lens[b]:, b].float().abs().max()) == 0.0


def test_config3_one_layer_full_size():
    """Config 3's first layer at its full size (620 -> 1000 per direction, B = 64, lengths U{20..80}, bf16): 64 rows x 2
    directions need more work-groups than the device holds at once, so this is the batch-slab launch path at the real T."""
    inp = synth.make(3, layers=1)
    c = _config_case(inp)
    print("  config 3, first layer, full size: T=%d frames=%d" % (inp["T"], synth.real_frames(inp)), flush=True)
    f, g = run_gpu(c, "bf16", True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL["bf16"])


def test_config3_upper_layer_full_size():
    """A layer k > 1 of config 3 at its full size (n_in = 2n = 2000, n = 1000, B = 64, T = 80, bf16)."""
    inp = synth.make(3, layers=1, n_in=2000)
    c = _config_case(inp)
    print("  config 3, upper layer, full size: T=%d frames=%d" % (inp["T"], synth.real_frames(inp)), flush=True)
    f, g = run_gpu(c, "bf16", True)
    fo, go = run_oracle(c, True)
    compare(f, g, fo, go, TOL["bf16"])
    f, g = run_gpu(c, "bf16", True, flags=Bn.FLAG_PLAIN_LAUNCH)          # the launch mode bench.py times
    compare(f, g, fo, go, TOL["bf16"])


@pytest.mark.timeout(600)
@pytest.mark.parametrize("k,over", [(3, dict(len_lo=8, len_hi=36)), (4, dict(len_lo=10, len_hi=40)), (7, dict(len_lo=8, len_hi=36))])
def test_six_layer_stack_full_width(k, over):
    """The whole depth of the three encoder stacks (six layers, the configurations' own n, n_in and B) with the lengths
    cut to at most 40 frames so that the oracle finishes in seconds: what grows through six bfloat16 layers - the error of
    y at the top, of dx at the bottom and of every layer's weight gradients - against the float64 oracle stack."""
    inp = synth.make(k, **over)
    print("  config %d, six layers: T=%d B=%d n=%d frames=%d" % (k, inp["T"], inp["cfg"]["B"], inp["cfg"]["n"], synth.real_frames(inp)), flush=True)
    assert len(inp["layers"]) == 6
    y, dx, grads = _stack_gpu(inp, "bf16")
    layers = [{kk: v.astype(np.float64) for kk, v in L.items()} for L in inp["layers"]]
    acts, yo = O.encoder_stack_fwd(inp["x"].astype(np.float64), layers, inp["seq_lens"])
    dxo, go = O.encoder_stack_bwd(acts, layers, inp["seq_lens"], inp["dy"].astype(np.float64))
    tol = TOL["bf16"]
    check("y", y, yo, tol)
    check("dx", dx, dxo, tol)
    for l, (g, r) in enumerate(zip(grads, go)):
        check("dW_x%d" % l, g["dW_x"], r[0], tol)
        check("dW_h%d" % l, g["dW_h"], r[1], tol)
        check("db%d" % l, g["db"], r[2], tol)


@pytest.mark.parametrize("over,pool_after", [(dict(layers=3, len_lo=9, len_hi=41, B=32), (0, 1)),
                                             (dict(layers=3, len_lo=0, len_hi=23, B=9, n=72, n_in=24), (0, 1)),
                                             (dict(layers=2, len_lo=1, len_hi=30, B=5, n=40), (0,))])
def test_pooled_encoder_chain(over, pool_after):
    """The pooled encoder as a chain: bidirectional layer -> max-pooling in time (windows of 2, inside each sequence) ->
    next layer on the pooled frames and the pooled LENGTHS the pooling call wrote on the device, and the backward chain
    through the pooling's gradient.  Against the same chain composed of the oracle's layer and pooling functions.

    The pooling decides an integer (which frame of a window holds the maximum) from floating-point values that differ
    between the two sides by the bfloat16 rounding of y, so where two frames of a window are closer than that, either choice
    is right.  The forward chain is compared directly (the maximum itself is continuous).  For the backward chain the HIP
    path's choices are first checked for validity against the oracle's y (the chosen frame holds the oracle's maximum up to
    the tolerance, and the very same frame wherever the oracle's window is decided by more than that), and the oracle's
    backward chain then routes the gradient through those same choices."""
    inp = synth.make(4, **over)
    pool = 2
    lens0 = inp["seq_lens"]
    nl = len(inp["layers"])
    tol = TOL["bf16"]
    print("  pooled chain: T=%d B=%d n=%d layers=%d" % (inp["T"], inp["cfg"]["B"], inp["cfg"]["n"], nl), flush=True)
    # HIP forward chain: the lengths of every layer come from the device array the pooling call before it wrote
    cur_g, lens_g = dev(inp["x"], "bf16"), dev(lens0)
    g_saved = []
    for l, L in enumerate(inp["layers"]):
        Wx, Wh, b = dev(L["W_x"], "bf16"), dev(L["W_h"], "bf16"), dev(L["b"])
        f = Bn.forward(cur_g, Wx, Wh, b, None, None, lens_g, bidirectional=True, want_state=False)
        assert not Bn.sync_status(f["workspace"])
        rec = dict(x=cur_g, lens=lens_g, f=f, Wx=Wx, Wh=Wh, T=cur_g.shape[0])
        if l in pool_after:
            r = Bn.time_pool_fwd(f["y"], lens_g, pool)
            rec.update(arg=r["arg"])
            cur_g, lens_g = r["out"], r["lens"]
        else:
            cur_g = f["y"]
        g_saved.append(rec)
    torch.cuda.synchronize()
    # oracle forward chain, with its own maxima; the HIP path's choices are validated against it layer by layer
    layers = [{kk: v.astype(np.float64) for kk, v in L.items()} for L in inp["layers"]]
    cur, lens = inp["x"].astype(np.float64), lens0.copy()
    o_saved = []
    for l, L in enumerate(layers):
        y = O.blstm_fwd(cur, L["W_x"], L["W_h"], L["b"], None, None, lens)[0]
        rec = dict(x=cur, lens=lens, T=cur.shape[0])
        if l in pool_after:
            out, lens_p, arg = O.time_maxpool_fwd(y, lens, pool)
            arg_g = g_saved[l]["arg"].cpu().numpy().astype(np.int64)
            Tp, B_, F_ = out.shape
            valid = (np.arange(Tp)[:, None] < lens_p[None, :])[:, :, None] & np.ones((1, 1, F_), dtype=bool)
            assert np.all(arg_g[valid] < pool)
            tt = np.minimum(np.arange(Tp)[:, None, None] * pool + np.where(valid, arg_g, 0), y.shape[0] - 1)
            inside = tt < np.asarray(lens)[None, :, None]                      # the chosen frame is a real frame of its row
            assert np.all(inside[valid])
            chosen = np.take_along_axis(y, tt, axis=0)
            slack = 2 * tol * np.abs(y).max()
            assert np.all(np.abs(chosen - out)[valid] <= slack), "a chosen frame does not hold the window's maximum"
            # where the oracle's window is decided by more than the slack, the choice must be the oracle's
            other = np.take_along_axis(y, np.minimum(np.arange(Tp)[:, None, None] * pool + (1 - np.where(valid, arg, 0)), y.shape[0] - 1), axis=0)
            two = valid & ((np.arange(Tp)[:, None, None] * pool + 1) < np.asarray(lens)[None, :, None])
            decided = two & (np.abs(out - other) > slack)
            assert np.array_equal(arg_g[decided], arg[decided])
            print("    layer %d pooling: %d of %d windows decided beyond the slack, %d choices differ from the oracle's" % (
                l, int(decided.sum()), int(valid.sum()), int((arg_g != arg)[valid].sum())), flush=True)
            rec.update(arg=np.where(valid, arg_g, 0), lens_p=lens_p)
            cur, lens = out, lens_p
        else:
            cur = y
        o_saved.append(rec)
    yo_top = cur
    assert np.array_equal(lens_g.cpu().numpy(), lens)
    check("y top", cur_g, yo_top, tol)
    rng = np.random.default_rng(66)
    dy_top = torch.from_numpy(rng.standard_normal(yo_top.shape)).to(torch.bfloat16).float().numpy().astype(np.float64)
    d = dy_top
    o_grads = [None] * nl
    for l in range(nl - 1, -1, -1):
        rec, L = o_saved[l], layers[l]
        if l in pool_after:
            d = O.time_maxpool_bwd(d, rec["arg"], rec["lens"], pool, rec["T"])
        g = O.blstm_bwd(rec["x"], L["W_x"], L["W_h"], L["b"], None, None, rec["lens"], d)
        o_grads[l] = g
        d = g[0]
    dxo = d
    dg = dev(dy_top, "bf16")
    for l in range(nl - 1, -1, -1):
        rec = g_saved[l]
        if l in pool_after:
            dg = Bn.time_pool_bwd(dg, rec["arg"], rec["lens"], pool, rec["T"])
        g = Bn.backward(rec["f"], rec["x"], rec["Wx"], rec["Wh"], None, None, rec["lens"], dg, want_dstate=False)
        assert not Bn.sync_status(rec["f"]["workspace"])
        check("dW_x%d" % l, g["dW_x"], o_grads[l][1], tol)
        check("dW_h%d" % l, g["dW_h"], o_grads[l][2], tol)
        check("db%d" % l, g["db"], o_grads[l][3], tol)
        dg = g["dx"]
    torch.cuda.synchronize()
    check("dx bottom", dg, dxo, tol)


@pytest.mark.parametrize("bidir,B,n_in,n", [(False, 70, 37, 50), (True, 33, 24, 18), (False, 300, 136, 100), (False, 1, 5, 6)])
def test_single_step_cell_bf16(bidir, B, n_in, n):
    """T = 1 in inference mode (the stepped decoder cell runs as one product over [x | h]): three chained steps with
    bias, initial state, rows of length 0 and the packed weights kept from the second step on, against the oracle."""
    rng = np.random.default_rng(1000 + B)
    D = 2 if bidir else 1
    lens = np.ones(B, dtype=np.int32)
    lens[::5] = 0                                           # these rows keep their state and output zero
    c = rnd_case(rng, 1, B, n_in, n, D, lens, "bf16")
    sq = (lambda a: a) if bidir else (lambda a: a[0])
    Wx, Wh, b = dev(sq(c["W_x"]), "bf16"), dev(sq(c["W_h"]), "bf16"), dev(sq(c["b"]))
    h, cc = dev(sq(c["h0"])), dev(sq(c["c0"]))
    ho, co = sq(c["h0"]), sq(c["c0"])
    ws = None
    for step in range(3):
        xt = torch.from_numpy(rng.standard_normal((1, B, n_in))).to(torch.bfloat16)
        flags = Bn.FLAG_INFERENCE | (Bn.FLAG_WEIGHTS_PACKED if step else 0)
        s = Bn.forward(xt.cuda(), Wx, Wh, b, h, cc, dev(lens), bidirectional=bidir, flags=flags, workspace=ws, want_c=True)
        ws = s["workspace"]
        x64 = xt.float().numpy().astype(np.float64)
        if bidir:
            yo, cso, ho, co = O.blstm_fwd(x64, c["W_x"], c["W_h"], c["b"], ho, co, lens)
        else:
            yo, cso, ho, co = O.lstm_fwd(x64, c["W_x"][0], c["W_h"][0], c["b"][0], ho, co, lens, 1)
        torch.cuda.synchronize()
        check("y", s["y"], yo, TOL["bf16"])
        check("c", s["c"], cso, TOL["bf16"])
        check("hT", s["hT"], ho, TOL["bf16"])
        check("cT", s["cT"], co, TOL["bf16"])
        assert float(s["y"].float()[0, ::5].abs().max()) == 0.0
        h, cc = s["hT"], s["cT"]


def test_config5_decoder_stepping_bf16():
    inp = synth.make(5)
    L = inp["layers"][0]
    rng = np.random.default_rng(5)
    Wx, Wh = dev(L["W_x"][0], "bf16"), dev(L["W_h"][0], "bf16")
    h = torch.zeros(768, 1000, device="cuda")
    c = torch.zeros(768, 1000, device="cuda")
    ho, co = np.zeros((768, 1000)), np.zeros((768, 1000))
    ws = None
    for step in range(4):
        xt = torch.from_numpy(rng.standard_normal((1, 768, 2620))).to(torch.bfloat16)
        s = Bn.forward(xt.cuda(), Wx, Wh, None, h, c, None, bidirectional=False,
                       flags=Bn.FLAG_INFERENCE | (Bn.FLAG_WEIGHTS_PACKED if step else 0), workspace=ws, want_c=False)
        ws = s["workspace"]
        h, c = s["hT"], s["cT"]
        _, _, ho, co = O.lstm_fwd(xt.float().numpy().astype(np.float64), L["W_x"][0].astype(np.float64),
                                  L["W_h"][0].astype(np.float64), None, ho, co, None, 1)
        torch.cuda.synchronize()
        print("  step", step, flush=True)
        check("h", h, ho, TOL["bf16"])
        check("c", c, co, TOL["bf16"])
