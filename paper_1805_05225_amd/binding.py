"""ctypes binding of the C ABI in include/lstm_abi.h.

Argument marshalling only: every step of the computation runs inside the HIP library.  PyTorch
is used to own device memory and to name the stream.  If the library is not built the import
fails loudly - there is no fallback path.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MI355X_LSTM_LIB", os.path.join(_HERE, "libmi355x_lstm.so"))   # override: diagnostic builds

LSTM_F32, LSTM_BF16_F32STATE = 0, 1
FLAG_ACCUMULATE, FLAG_PER_STEP, FLAG_INFERENCE, FLAG_WEIGHTS_PACKED, FLAG_PLAIN_LAUNCH = 1, 2, 4, 8, 16
EXPORTS = ("lstm_query", "lstm_fwd", "lstm_bwd", "blstm_fwd", "blstm_bwd", "lstm_gemm", "lstm_time_pool_fwd", "lstm_time_pool_bwd", "lstm_attention_query", "lstm_attention_step",
           "lstm_readout_query", "lstm_readout", "lstm_beam_query", "lstm_beam_step", "lstm_beam_step_static", "lstm_beam_gather", "lstm_beam_gather_many", "lstm_embed",
           "lstm_sync_status", "lstm_profile_enable", "lstm_profile_read",
           "lstm_strerror")


class GatherItem(ctypes.Structure):
    _fields_ = [("elem_bytes", ctypes.c_int32), ("width", ctypes.c_int32), ("inp", ctypes.c_void_p), ("ld_in", ctypes.c_int64),
                ("out", ctypes.c_void_p), ("ld_out", ctypes.c_int64)]


class AttDesc(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int32), ("Q", ctypes.c_int32), ("beam", ctypes.c_int32), ("A", ctypes.c_int32), ("E", ctypes.c_int32),
                ("n", ctypes.c_int32), ("workspace_bytes", ctypes.c_uint64)]


class LstmDesc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("B", ctypes.c_int32), ("n_in", ctypes.c_int32), ("n", ctypes.c_int32),
                ("direction", ctypes.c_int32), ("dtype", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("reserve_bytes", ctypes.c_uint64), ("workspace_bytes", ctypes.c_uint64)]


class LstmError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__("lstm library status %d: %s" % (status, strerror(status)))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("HIP library %s is not built; run `python -m paper_1805_05225_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, ip = ctypes.c_void_p, ctypes.c_int
    dp = ctypes.POINTER(LstmDesc)
    lib.lstm_query.restype = ip
    lib.lstm_query.argtypes = [dp, ip, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
    for name in ("lstm_fwd", "blstm_fwd"):
        f = getattr(lib, name)
        f.restype = ip
        f.argtypes = [dp] + [vp] * 14
    for name in ("lstm_bwd", "blstm_bwd"):
        f = getattr(lib, name)
        f.restype = ip
        f.argtypes = [dp] + [vp] * 20
    lib.lstm_gemm.restype = ip
    lib.lstm_gemm.argtypes = [ip] * 7 + [vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ip, vp, ip, ip, vp]
    i64 = ctypes.c_int64
    lib.lstm_time_pool_fwd.restype = ip
    lib.lstm_time_pool_fwd.argtypes = [ip] * 5 + [vp, i64, vp, vp, i64, vp, vp, vp]
    lib.lstm_time_pool_bwd.restype = ip
    lib.lstm_time_pool_bwd.argtypes = [ip] * 5 + [vp, i64, vp, vp, vp, i64, vp]
    fp, u64p = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint64)
    lib.lstm_attention_query.restype = ip
    lib.lstm_attention_query.argtypes = [ctypes.POINTER(AttDesc), u64p]
    lib.lstm_attention_step.restype = ip
    lib.lstm_attention_step.argtypes = [ctypes.POINTER(AttDesc), vp, vp, vp, vp, i64, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, vp, i64, vp, vp]
    lib.lstm_readout_query.restype = ip
    lib.lstm_readout_query.argtypes = [ip, ip, ip, ip, ip, u64p]
    lib.lstm_readout.restype = ip
    lib.lstm_readout.argtypes = [ip, ip, ip, vp, i64, ip, vp, i64, ip, vp, i64, ip, vp, vp, vp, i64, vp, ctypes.c_uint64, vp]
    lib.lstm_beam_query.restype = ip
    lib.lstm_beam_query.argtypes = [ip, ip, ip, u64p]
    lib.lstm_beam_step.restype = ip
    lib.lstm_beam_step.argtypes = [ip, ip, ip, vp, i64, vp, vp, vp, vp, vp, ctypes.c_uint64, vp]
    lib.lstm_beam_step_static.restype = ip
    lib.lstm_beam_step_static.argtypes = [ip, ip, ip, vp, i64, vp, vp, vp, vp, vp]
    lib.lstm_beam_gather.restype = ip
    lib.lstm_beam_gather.argtypes = [ip, ip, ip, ip, vp, i64, vp, vp, i64, vp]
    lib.lstm_beam_gather_many.restype = ip
    lib.lstm_beam_gather_many.argtypes = [ip, ip, ip, ctypes.POINTER(GatherItem), vp, vp]
    lib.lstm_embed.restype = ip
    lib.lstm_embed.argtypes = [ip, ip, ip, vp, vp, vp, vp, i64, vp]
    lib.lstm_sync_status.restype = ip
    lib.lstm_sync_status.argtypes = [vp, ctypes.POINTER(ctypes.c_int32)]
    lib.lstm_profile_enable.restype = ip
    lib.lstm_profile_enable.argtypes = [ip]
    lib.lstm_profile_read.restype = ip
    lib.lstm_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.lstm_strerror.restype = ctypes.c_char_p
    lib.lstm_strerror.argtypes = [ip]
    return lib


lib = _load()


def strerror(status):
    return lib.lstm_strerror(int(status)).decode()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors crossing the ABI must be contiguous"
    return t.data_ptr()


def _check(status):
    if status != 0:
        raise LstmError(status)


def make_desc(T, B, n_in, n, dtype, direction=1, flags=0):
    return LstmDesc(T, B, n_in, n, direction, dtype, flags, 0, 0, 0)


def query(desc, bidirectional):
    r, w = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib.lstm_query(ctypes.byref(desc), int(bool(bidirectional)), ctypes.byref(r), ctypes.byref(w)))
    return r.value, w.value


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dtype_of(x):
    return LSTM_BF16_F32STATE if x.dtype == torch.bfloat16 else LSTM_F32


def forward(x, W_x, W_h, b=None, h0=None, c0=None, seq_lens=None, *, bidirectional, direction=1, flags=0,
            workspace=None, want_c=True, want_state=True, poison=False):
    """Allocates the outputs and calls lstm_fwd / blstm_fwd.  Returns a dict with y, c, hT, cT,
    reserve, workspace and the descriptor (everything the backward call needs).  poison: fill reserve and workspace
    with 0xFF bytes first."""
    T, B, n_in = x.shape
    n = W_h.shape[-2]
    D = 2 if bidirectional else 1
    dev = x.device
    desc = make_desc(T, B, n_in, n, _dtype_of(x), direction, flags)
    rb, wb = query(desc, bidirectional)
    infer = bool(flags & FLAG_INFERENCE)
    reserve = None if infer else torch.empty(rb, dtype=torch.uint8, device=dev)
    if workspace is None or workspace.numel() < wb:
        workspace = torch.empty(wb, dtype=torch.uint8, device=dev)
    if poison:          # tests: every byte the library has not written reads as NaN
        workspace.fill_(0xFF)
        if reserve is not None:
            reserve.fill_(0xFF)
    desc.reserve_bytes = 0 if infer else rb
    desc.workspace_bytes = workspace.numel()
    y = torch.empty(T, B, D * n, dtype=x.dtype, device=dev)
    shp = (D, B, n) if bidirectional else (B, n)
    c = torch.empty((D, T, B, n) if bidirectional else (T, B, n), dtype=torch.float32, device=dev) if (want_c or not infer) else None
    hT = torch.empty(shp, dtype=torch.float32, device=dev) if want_state else None
    cT = torch.empty(shp, dtype=torch.float32, device=dev) if want_state else None
    fn = lib.blstm_fwd if bidirectional else lib.lstm_fwd
    _check(fn(ctypes.byref(desc), _ptr(x), _ptr(W_x), _ptr(W_h), _ptr(b), _ptr(h0), _ptr(c0), _ptr(seq_lens),
              _ptr(y), _ptr(c), _ptr(hT), _ptr(cT), _ptr(reserve), _ptr(workspace), _stream()))
    return dict(y=y, c=c, hT=hT, cT=cT, reserve=reserve, workspace=workspace, desc=desc, bidirectional=bidirectional)


def backward(fwd, x, W_x, W_h, h0, c0, seq_lens, dy, dhT=None, dcT=None, *, want_dx=True, want_dstate=True,
             accumulate_into=None):
    """Allocates the gradients and calls lstm_bwd / blstm_bwd with the buffers of `forward`'s result."""
    desc = fwd["desc"]
    bidirectional = fwd["bidirectional"]
    T, B, n_in = x.shape
    n = W_h.shape[-2]
    dev = x.device
    if accumulate_into is not None:
        dW_x, dW_h, db = accumulate_into
        desc = LstmDesc(desc.T, desc.B, desc.n_in, desc.n, desc.direction, desc.dtype, desc.flags | FLAG_ACCUMULATE, 0,
                        desc.reserve_bytes, desc.workspace_bytes)
    else:
        dW_x = torch.empty(W_x.shape, dtype=torch.float32, device=dev)
        dW_h = torch.empty(W_h.shape, dtype=torch.float32, device=dev)
        db = torch.empty(W_x.shape[:-2] + (4 * n,), dtype=torch.float32, device=dev)
    dx = torch.empty_like(x) if want_dx else None
    shp = (2, B, n) if bidirectional else (B, n)
    dh0 = torch.empty(shp, dtype=torch.float32, device=dev) if want_dstate else None
    dc0 = torch.empty(shp, dtype=torch.float32, device=dev) if want_dstate else None
    fn = lib.blstm_bwd if bidirectional else lib.lstm_bwd
    _check(fn(ctypes.byref(desc), _ptr(x), _ptr(W_x), _ptr(W_h), _ptr(h0), _ptr(c0), _ptr(seq_lens),
              _ptr(fwd["y"]), _ptr(fwd["c"]), _ptr(fwd["reserve"]), _ptr(dy), _ptr(dhT), _ptr(dcT),
              _ptr(dx), _ptr(dW_x), _ptr(dW_h), _ptr(db), _ptr(dh0), _ptr(dc0), _ptr(fwd["workspace"]), _stream()))
    return dict(dx=dx, dW_x=dW_x, dW_h=dW_h, db=db, dh0=dh0, dc0=dc0)


def gemm(A, B, *, a_kcontig, b_kcontig, M, N, K, out_dtype=torch.float32, bias=None, C=None, accumulate=False,
         lens=None, Bt=1, T=0):
    """C[M,N] (+)= A B + bias through lstm_gemm; A and B are 2-D tensors in the stated storage order."""
    in_bf16 = A.dtype == torch.bfloat16
    if C is None:
        C = torch.empty(M, N, dtype=out_dtype, device=A.device)
    _check(lib.lstm_gemm(int(in_bf16), int(C.dtype == torch.bfloat16), int(a_kcontig), int(b_kcontig), M, N, K,
                         _ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(C), C.stride(0), _ptr(bias), int(accumulate),
                         _ptr(lens), Bt, T, _stream()))
    return C


def time_pool_fwd(y, seq_lens, pool, *, want_arg=True):
    """Max-pooling in time of y [T, B, F] (float or bfloat16) with windows of `pool` frames inside every sequence.
    -> dict(out [T', B, F], lens [B] int32, arg [T', B, F] uint8 or None)."""
    T, B, F = y.shape
    assert y.stride(2) == 1 and y.stride(0) == B * y.stride(1)
    Tp = -(-T // pool)
    out = torch.empty(Tp, B, F, dtype=y.dtype, device=y.device)
    arg = torch.empty(Tp, B, F, dtype=torch.uint8, device=y.device) if want_arg else None
    lens_out = torch.empty(B, dtype=torch.int32, device=y.device)
    _check(lib.lstm_time_pool_fwd(_dtype_of(y), T, B, F, pool, y.data_ptr(), y.stride(1), _ptr(seq_lens), _ptr(out), F, _ptr(arg),
                                  _ptr(lens_out), _stream()))
    return dict(out=out, lens=lens_out, arg=arg)


def time_pool_bwd(dout, arg, seq_lens, pool, T):
    """Gradient of time_pool_fwd: dy [T, B, F] from dout [T', B, F]."""
    Tp, B, F = dout.shape
    assert dout.is_contiguous()
    dy = torch.empty(T, B, F, dtype=dout.dtype, device=dout.device)
    _check(lib.lstm_time_pool_bwd(_dtype_of(dout), T, B, F, pool, _ptr(dout), F, _ptr(arg), _ptr(seq_lens), _ptr(dy), F, _stream()))
    return dy


def attention_query(S, Q, beam, A, E, n):
    d = AttDesc(S, Q, beam, A, E, n, 0)
    need = ctypes.c_uint64(0)
    _check(lib.lstm_attention_query(ctypes.byref(d), ctypes.byref(need)))
    d.workspace_bytes = need.value
    return d


def attention_step(enc, enc_ctx, src_lens, beam, s, W_s, b_s, w_fb, b_fb, v, b_e, accum, *, att=None, workspace=None, want_a=True):
    """One attention step through lstm_attention_step.  enc [S,Q,E], enc_ctx [S,Q,A], s [B,n] (a view with a row stride is
    fine), W_s [A,n] bfloat16; b_s, w_fb, b_fb, v float [A]; accum float [B,S]; att: optional bfloat16 [B,>=E] view to write into.
    -> dict(a, accum, att, workspace)."""
    S, Q, E = enc.shape
    A = enc_ctx.shape[2]
    B, n = s.shape
    d = attention_query(S, Q, beam, A, E, n)
    if workspace is None or workspace.numel() < d.workspace_bytes:
        workspace = torch.empty(d.workspace_bytes, dtype=torch.uint8, device=enc.device)
    d.workspace_bytes = workspace.numel()
    if att is None:
        att = torch.empty(B, E, dtype=torch.bfloat16, device=enc.device)
    a = torch.empty(B, S, dtype=torch.float32, device=enc.device) if want_a else None
    accum_out = torch.empty(B, S, dtype=torch.float32, device=enc.device)
    assert enc.is_contiguous() and enc_ctx.is_contiguous() and accum.is_contiguous() and s.stride(1) == 1 and att.stride(1) == 1
    _check(lib.lstm_attention_step(ctypes.byref(d), _ptr(enc), _ptr(enc_ctx), _ptr(src_lens), s.data_ptr(), s.stride(0), _ptr(W_s), _ptr(b_s),
                                   _ptr(w_fb), _ptr(b_fb), _ptr(v), float(b_e), _ptr(accum), _ptr(accum_out), _ptr(a), att.data_ptr(),
                                   att.stride(0), _ptr(workspace), _stream()))
    return dict(a=a, accum=accum_out, att=att, workspace=workspace)


def readout(s, trg, att, W_r, b_r, *, out=None, workspace=None, flags=0):
    """out = relu([s | trg | att] W_r^T + b_r) through lstm_readout; s [B,n], trg [B,n_trg], att [B,E] bfloat16 (views with a
    row stride are fine), W_r [R, n+n_trg+E] bfloat16, b_r float [R]."""
    B, n = s.shape
    nt, E, R = trg.shape[1], att.shape[1], W_r.shape[0]
    need = ctypes.c_uint64(0)
    _check(lib.lstm_readout_query(B, R, n, nt, E, ctypes.byref(need)))
    if workspace is None or workspace.numel() < need.value:
        workspace = torch.empty(need.value, dtype=torch.uint8, device=s.device)
    if out is None:
        out = torch.empty(B, R, dtype=torch.bfloat16, device=s.device)
    assert s.stride(1) == 1 and trg.stride(1) == 1 and att.stride(1) == 1 and W_r.is_contiguous() and out.stride(1) == 1
    _check(lib.lstm_readout(flags, B, R, s.data_ptr(), s.stride(0), n, trg.data_ptr(), trg.stride(0), nt, att.data_ptr(), att.stride(0), E,
                            _ptr(W_r), _ptr(b_r), out.data_ptr(), out.stride(0), _ptr(workspace), workspace.numel(), _stream()))
    return out


def beam_step(logits, score, *, workspace=None):
    """One beam-search step through lstm_beam_step.  logits float [Q*beam, V] (row stride allowed), score float [Q, beam]
    -> dict(score [Q,beam] float, src [Q,beam] int32, label [Q,beam] int32, workspace)."""
    Q, beam = score.shape
    V = logits.shape[1]
    need = ctypes.c_uint64(0)
    _check(lib.lstm_beam_query(Q, beam, V, ctypes.byref(need)))
    if workspace is None or workspace.numel() < need.value:
        workspace = torch.empty(need.value, dtype=torch.uint8, device=logits.device)
    out = torch.empty(Q, beam, dtype=torch.float32, device=logits.device)
    src = torch.empty(Q, beam, dtype=torch.int32, device=logits.device)
    label = torch.empty(Q, beam, dtype=torch.int32, device=logits.device)
    assert logits.stride(1) == 1 and logits.dtype == torch.float32 and score.dtype == torch.float32
    _check(lib.lstm_beam_step(Q, beam, V, logits.data_ptr(), logits.stride(0), _ptr(score), _ptr(out), _ptr(src), _ptr(label),
                              _ptr(workspace), workspace.numel(), _stream()))
    return dict(score=out, src=src, label=label, workspace=workspace)


def beam_step_static(logits, score):
    """lstm_beam_step_static: the same step with the library's own scratch array (no workspace, nothing allocated by the
    call itself; the outputs are the caller's, allocated here)."""
    Q, beam = score.shape
    V = logits.shape[1]
    out = torch.empty(Q, beam, dtype=torch.float32, device=logits.device)
    src = torch.empty(Q, beam, dtype=torch.int32, device=logits.device)
    label = torch.empty(Q, beam, dtype=torch.int32, device=logits.device)
    assert logits.stride(1) == 1 and logits.dtype == torch.float32 and score.dtype == torch.float32
    _check(lib.lstm_beam_step_static(Q, beam, V, logits.data_ptr(), logits.stride(0), _ptr(score), _ptr(out), _ptr(src), _ptr(label),
                                     _stream()))
    return dict(score=out, src=src, label=label)


def beam_gather(state, src):
    """Rows of per-hypothesis state [Q*beam, width] (float or bfloat16) moved behind the choice `src` [Q, beam]."""
    Q, beam = src.shape
    out = torch.empty_like(state)
    assert state.stride(1) == 1
    _check(lib.lstm_beam_gather(state.element_size(), Q, beam, state.shape[1], state.data_ptr(), state.stride(0), _ptr(src), _ptr(out),
                                out.stride(0), _stream()))
    return out


def gather_items(pairs):
    """ctypes array of lstm_gather_item for (in, out) pairs of 2-D tensors (float or bfloat16, rows contiguous)."""
    arr = (GatherItem * len(pairs))()
    for it, (a, o) in zip(arr, pairs):
        assert a.stride(1) == 1 and o.stride(1) == 1 and a.dtype == o.dtype and a.shape == o.shape
        it.elem_bytes, it.width, it.inp, it.ld_in, it.out, it.ld_out = a.element_size(), a.shape[1], a.data_ptr(), a.stride(0), o.data_ptr(), o.stride(0)
    return arr


def beam_gather_many(states, src, outs=None):
    """beam_gather for up to 8 state arrays in one launch (lstm_beam_gather_many); `outs` may be views with a larger row stride."""
    Q, beam = src.shape
    if outs is None:
        outs = [torch.empty_like(a) for a in states]
    arr = gather_items(list(zip(states, outs)))
    _check(lib.lstm_beam_gather_many(Q, beam, len(arr), arr, _ptr(src), _stream()))
    return outs


def embed(label, W_trg, b_trg=None, *, out=None):
    """trg = W_trg[label] + b_trg through lstm_embed; label int32 (any shape), W_trg [V, n] bfloat16 -> [label.numel(), n] bfloat16."""
    V, n = W_trg.shape
    B = label.numel()
    if out is None:
        out = torch.empty(B, n, dtype=torch.bfloat16, device=W_trg.device)
    _check(lib.lstm_embed(B, n, V, _ptr(label), _ptr(W_trg), _ptr(b_trg), out.data_ptr(), out.stride(0), _stream()))
    return out


PHASES = ("prep", "gemm_zx", "loop_fwd", "loop_bwd", "gemm_dx", "gemm_dwx", "gemm_dwh", "db")


def profile_enable(on):
    _check(lib.lstm_profile_enable(int(on)))


def profile_read():
    """-> {phase: (milliseconds, launches)} accumulated since the last read."""
    ms = (ctypes.c_double * len(PHASES))()
    ln = (ctypes.c_int64 * len(PHASES))()
    _check(lib.lstm_profile_read(ms, ln))
    return {p: (ms[i], ln[i]) for i, p in enumerate(PHASES)}


def sync_status(workspace):
    """True if a bounded wait of a single-launch recurrent kernel expired in the last call that used
    this workspace (synchronises the device)."""
    flag = ctypes.c_int32(0)
    _check(lib.lstm_sync_status(_ptr(workspace), ctypes.byref(flag)))
    return bool(flag.value)
