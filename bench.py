#!/usr/bin/env python3
"""Benchmark: BLSTM forward + backward frames/sec at n = 1024 on one MI355X.

One "step" is one forward pass through the six bidirectional layers of the speech-shaped
configuration (input 40, n = 1024 per direction, B = 32, lengths ~ U{200..1500}, bf16 storage
with float state) followed by one backward pass through all six layers, on synthetic seeded
inputs that are resident in HBM before the timed region starts.  frames = sum(seq_lens), each
real frame counted once for the whole stack.

Prints ONE JSON line.  `roofline` describes the dominant kernel (the backward recurrent loop, one
launch per layer); `cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
BF16_PEAK_TFLOPS = 2500.0
# The benchmark owns the device and uses one stream: the single-launch recurrent kernels are started with ordinary
# launches (LSTM_FLAG_PLAIN_LAUNCH, 16); every timed run ends with a check that no bounded wait expired.
LAUNCH_FLAGS = 16


def build_stack(inp, Bn):
    dt = torch.bfloat16 if inp["cfg"]["dtype"] == "bf16" else torch.float32
    x = torch.from_numpy(inp["x"]).to(dt).cuda()
    lens = torch.from_numpy(inp["seq_lens"]).to(torch.int32).cuda()
    dy = torch.from_numpy(inp["dy"]).to(dt).cuda()
    layers = []
    for L in inp["layers"]:
        layers.append((torch.from_numpy(L["W_x"]).to(dt).cuda(), torch.from_numpy(L["W_h"]).to(dt).cuda(),
                       torch.from_numpy(L["b"]).float().cuda()))
    return x, lens, dy, layers


class Stack:
    """Pre-allocates every buffer once so the timed region holds ABI calls only."""

    def __init__(self, Bn, x, lens, dy, layers):
        import ctypes
        self.Bn, self.ct = Bn, ctypes
        self.x, self.lens, self.dy, self.layers = x, lens, dy, layers
        T, B, _ = x.shape
        n = layers[0][1].shape[-2]
        dev = x.device
        self.bufs = []
        wmax = 0
        cur_in = x.shape[2]
        for (Wx, Wh, b) in layers:
            desc = Bn.make_desc(T, B, cur_in, n, Bn.LSTM_BF16_F32STATE if x.dtype == torch.bfloat16 else Bn.LSTM_F32, 1, LAUNCH_FLAGS)
            rb, wb = Bn.query(desc, True)
            wmax = max(wmax, wb)
            desc.reserve_bytes = rb
            self.bufs.append(dict(
                desc=desc, reserve=torch.empty(rb, dtype=torch.uint8, device=dev),
                y=torch.empty(T, B, 2 * n, dtype=x.dtype, device=dev), c=torch.empty(2, T, B, n, dtype=torch.float32, device=dev),
                dx=torch.empty(T, B, cur_in, dtype=x.dtype, device=dev),
                dW_x=torch.empty_like(Wx, dtype=torch.float32), dW_h=torch.empty_like(Wh, dtype=torch.float32),
                db=torch.empty(2, 4 * n, dtype=torch.float32, device=dev)))
            cur_in = 2 * n
        self.ws = torch.empty(wmax, dtype=torch.uint8, device=dev)
        for bf in self.bufs:
            bf["desc"].workspace_bytes = wmax

    def verify(self):
        """A bounded wait that expires inside a single-launch recurrent kernel leaves invalid results behind a call that
        returned LSTM_OK (and a drained step is FASTER): the word that says so is checked here (synchronises)."""
        if self.Bn.sync_status(self.ws):
            raise RuntimeError("a bounded wait expired inside a recurrent kernel: the timed results are invalid")

    def step(self, check=False):
        Bn, ct = self.Bn, self.ct
        s = torch.cuda.current_stream().cuda_stream
        cur = self.x
        for (Wx, Wh, b), bf in zip(self.layers, self.bufs):
            rc = Bn.lib.blstm_fwd(ct.byref(bf["desc"]), cur.data_ptr(), Wx.data_ptr(), Wh.data_ptr(), b.data_ptr(), None, None,
                                  self.lens.data_ptr(), bf["y"].data_ptr(), bf["c"].data_ptr(), None, None,
                                  bf["reserve"].data_ptr(), self.ws.data_ptr(), s)
            assert rc == 0, Bn.strerror(rc)
            if check:
                self.verify()
            cur = bf["y"]
        d = self.dy
        for k in range(len(self.layers) - 1, -1, -1):
            Wx, Wh, b = self.layers[k]
            bf = self.bufs[k]
            xin = self.x if k == 0 else self.bufs[k - 1]["y"]
            rc = Bn.lib.blstm_bwd(ct.byref(bf["desc"]), xin.data_ptr(), Wx.data_ptr(), Wh.data_ptr(), None, None,
                                  self.lens.data_ptr(), bf["y"].data_ptr(), bf["c"].data_ptr(), bf["reserve"].data_ptr(),
                                  d.data_ptr(), None, None, bf["dx"].data_ptr(), bf["dW_x"].data_ptr(), bf["dW_h"].data_ptr(),
                                  bf["db"].data_ptr(), None, None, self.ws.data_ptr(), s)
            assert rc == 0, Bn.strerror(rc)
            if check:
                self.verify()
            d = bf["dx"]


class MixedStack:
    """One bidirectional layer below unidirectional ones; every buffer allocated once."""

    def __init__(self, Bn, x, lens, dy, layers):
        import ctypes
        self.Bn, self.ct = Bn, ctypes
        self.x, self.lens, self.dy, self.layers = x, lens, dy, layers
        T, B, _ = x.shape
        n = layers[0][1].shape[-2]
        dev = x.device
        self.bufs = []
        wmax = 0
        cur = x
        for (Wx, Wh, b) in layers:
            D = Wx.shape[0]
            desc = Bn.make_desc(T, B, cur.shape[2], n, Bn.LSTM_BF16_F32STATE if x.dtype == torch.bfloat16 else Bn.LSTM_F32, 1, LAUNCH_FLAGS)
            rb, wb = Bn.query(desc, D == 2)
            wmax = max(wmax, wb)
            desc.reserve_bytes = rb
            bf = dict(desc=desc, D=D, xin=cur, reserve=torch.empty(rb, dtype=torch.uint8, device=dev),
                      y=torch.empty(T, B, D * n, dtype=x.dtype, device=dev), c=torch.empty(D, T, B, n, dtype=torch.float32, device=dev),
                      dx=torch.empty_like(cur), dW_x=torch.empty_like(Wx, dtype=torch.float32),
                      dW_h=torch.empty_like(Wh, dtype=torch.float32), db=torch.empty(D, 4 * n, dtype=torch.float32, device=dev))
            self.bufs.append(bf)
            cur = bf["y"]
        self.ws = torch.empty(wmax, dtype=torch.uint8, device=dev)
        for bf in self.bufs:
            bf["desc"].workspace_bytes = wmax

    verify = Stack.verify

    def step(self, check=False):
        lib, ct = self.Bn.lib, self.ct
        s = torch.cuda.current_stream().cuda_stream
        for (Wx, Wh, b), bf in zip(self.layers, self.bufs):
            fn = lib.blstm_fwd if bf["D"] == 2 else lib.lstm_fwd
            rc = fn(ct.byref(bf["desc"]), bf["xin"].data_ptr(), Wx.data_ptr(), Wh.data_ptr(), b.data_ptr(), None, None,
                    self.lens.data_ptr(), bf["y"].data_ptr(), bf["c"].data_ptr(), None, None, bf["reserve"].data_ptr(),
                    self.ws.data_ptr(), s)
            assert rc == 0, self.Bn.strerror(rc)
            if check:
                self.verify()
        d = self.dy
        for k in range(len(self.layers) - 1, -1, -1):
            Wx, Wh, b = self.layers[k]
            bf = self.bufs[k]
            fn = lib.blstm_bwd if bf["D"] == 2 else lib.lstm_bwd
            rc = fn(ct.byref(bf["desc"]), bf["xin"].data_ptr(), Wx.data_ptr(), Wh.data_ptr(), None, None, self.lens.data_ptr(),
                    bf["y"].data_ptr(), bf["c"].data_ptr(), bf["reserve"].data_ptr(), d.data_ptr(), None, None, bf["dx"].data_ptr(),
                    bf["dW_x"].data_ptr(), bf["dW_h"].data_ptr(), bf["db"].data_ptr(), None, None, self.ws.data_ptr(), s)
            assert rc == 0, self.Bn.strerror(rc)
            if check:
                self.verify()
            d = bf["dx"]


def bench_mixed(args, Bn, synth):
    """--config 7: the translation encoder of the speed comparison, one bidirectional layer below five unidirectional ones."""
    inp = synth.make(7)
    cfg = inp["cfg"]
    frames = synth.real_frames(inp)
    flops = synth.flops_fwd_bwd(inp)
    x, lens, dy, layers = build_stack(inp, Bn)
    st = MixedStack(Bn, x, lens, dy, layers)
    for _ in range(args.warmup):
        st.step()
    torch.cuda.synchronize()
    Bn.profile_enable(1)              # loops and products only: an event between kernels idles the device for microseconds
    t0 = time.perf_counter()
    for _ in range(args.steps):
        st.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    Bn.profile_enable(False)
    prof = Bn.profile_read()
    st.verify()                       # the last call of the timed region
    st.step(check=True)               # and one untimed step with the word checked behind every call
    T, B, n, nl = inp["T"], cfg["B"], cfg["n"], cfg["layers"]
    # recurrent loops: algorithmic HBM bytes per REAL frame of one row and ONE direction (as for the bidirectional stacks;
    # padded frames are skipped by the kernels and not counted); the stack runs (nl + 1) directions over `frames` frames
    fwd_row_bytes = 2 * 4 * n * 4 + n * 4 + n * 2
    bwd_row_bytes = 4 * n * 4 + 2 * n * 4 + n * 2 + 4 * n * 2
    def loop(phase, by, name):
        ms, launches = prof[phase]
        total = by * frames * (nl + 1) * args.steps
        gbs = total / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        return {"bound": "hbm", "kernel": name, "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                "traffic": None, "launches": int(launches), "avg_launch_ms": ms / max(launches, 1),
                "us_per_layer_time_step": ms * 1e3 / (args.steps * nl * T), "algorithmic_bytes_per_row_frame_direction": by}
    out = {
        "metric": "encoder fwd+bwd frames/sec (n=%d), 1 bidirectional + %d unidirectional layers" % (n, nl - 1),
        "value": frames * args.steps / dt, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"],
        "data": "synthetic",
        "config": {"workload": "config 7: 1 BLSTM layer + %d LSTM layers, n_in=%d, n=%d, B=%d, seq_lens~U{%d..%d} (T=%d, %d real frames), "
                               "bf16 storage / f32 state, forward + backward" % (nl - 1, cfg["n_in"], n, B, cfg["len_lo"], cfg["len_hi"], T, frames)},
        "useful_tflops": flops * args.steps / dt / 1e12,
        "roofline": loop("loop_bwd", bwd_row_bytes, "backward recurrent loops"),
        "roofline_forward_loop": loop("loop_fwd", fwd_row_bytes, "forward recurrent loops"),
        "phases_ms_per_step": {k: v[0] / args.steps for k, v in prof.items()},
    }
    print(json.dumps(out))


def cpu_baseline(inp):
    """The CPU oracle, as it stands (float64 numpy), on a bounded sample: layer 2 of the stack
    (n_in = 2n) over the first `cap` frames of every sequence, forward + backward; the per-layer
    rate is divided by the number of layers to stand beside the whole-stack GPU figure."""
    from oracle import lstm_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    cap = 320                          # about 11 s of CPU work on the 16 host threads of the GPU machine
    nl = len(inp["layers"])
    L = inp["layers"][min(1, nl - 1)]
    lens = np.minimum(inp["seq_lens"], cap)
    T = int(lens.max())
    n_in = L["W_x"].shape[1]
    rng = np.random.default_rng(0)
    x = rng.standard_normal((T, len(lens), n_in))
    dy = rng.standard_normal((T, len(lens), 2 * L["W_h"].shape[1]))
    Wx, Wh = L["W_x"].astype(np.float64), L["W_h"].astype(np.float64)
    t0 = time.perf_counter()
    O.blstm_fwd(x, Wx, Wh, None, None, None, lens)
    O.blstm_bwd(x, Wx, Wh, None, None, None, lens, dy)
    dt = time.perf_counter() - t0
    frames = int(lens.sum())
    return {"value": frames / dt / nl, "unit": "frames/s", "cores": int(cores), "kind": "oracle",
            "sample": "float64 numpy oracle, layer 2 of %d (n_in=%d, n=%d), B=%d, first %d frames of every sequence "
                      "(%d frames, %.1f s fwd+bwd); per-layer rate divided by %d layers" % (
                          nl, n_in, L["W_h"].shape[1], len(lens), cap, frames, dt, nl)}


def bench_decoder(args, Bn, synth):
    """--config 5: the stepped decoder cell (one LSTM of n = 1000 fed by 620 + 2000 inputs, 768 rows = 64 sentences x
    beam 12), forward only, one time step per call with the state fed back.  One "step" here is one block of 100
    dependent decoder steps; the figure of merit is the latency of one decoder step."""
    import ctypes as ct
    inp = synth.make(5)
    cfg = inp["cfg"]
    L = inp["layers"][0]
    n, n_in, B, nsteps = cfg["n"], cfg["n_in"], cfg["B"], cfg["steps"]
    Wx = torch.from_numpy(L["W_x"][0]).to(torch.bfloat16).cuda()
    Wh = torch.from_numpy(L["W_h"][0]).to(torch.bfloat16).cuda()
    b = torch.from_numpy(L["b"][0]).float().cuda()
    g = torch.Generator(device="cpu").manual_seed(5)
    xs = torch.randn(nsteps, B, n_in, generator=g).to(torch.bfloat16).cuda()     # embedding | context, fresh every step
    desc = Bn.make_desc(1, B, n_in, n, Bn.LSTM_BF16_F32STATE, 1, Bn.FLAG_INFERENCE)
    _, wb = Bn.query(desc, False)
    desc.workspace_bytes = wb
    desc_packed = Bn.make_desc(1, B, n_in, n, Bn.LSTM_BF16_F32STATE, 1, Bn.FLAG_INFERENCE | Bn.FLAG_WEIGHTS_PACKED)
    desc_packed.workspace_bytes = wb
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    y = torch.empty(1, B, n, dtype=torch.bfloat16, device="cuda")
    state = [torch.zeros(B, n, device="cuda") for _ in range(4)]                  # h, c ping-pong
    s = torch.cuda.current_stream().cuda_stream

    def block(first_call):
        for i in range(nsteps):
            h0, c0, h1, c1 = state if i % 2 == 0 else (state[2], state[3], state[0], state[1])
            d = desc if (first_call and i == 0) else desc_packed
            rc = Bn.lib.lstm_fwd(ct.byref(d), xs[i].data_ptr(), Wx.data_ptr(), Wh.data_ptr(), b.data_ptr(), h0.data_ptr(),
                                 c0.data_ptr(), None, y.data_ptr(), None, h1.data_ptr(), c1.data_ptr(), None, ws.data_ptr(), s)
            assert rc == 0, Bn.strerror(rc)

    block(True)                                   # packs the weights once
    for _ in range(args.warmup):
        block(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        block(False)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us = dt / (args.steps * nsteps) * 1e6
    flops = 8.0 * n * (n_in + n) * B
    tflops = flops / (us * 1e-6) / 1e12
    out = {
        "metric": "LSTM decoder step latency (n=%d, %d rows)" % (n, B), "value": us, "unit": "us/step", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 5: one LSTM stepped one time step per call, n_in=%d (620 + 2000), n=%d, rows=%d, "
                               "%d dependent steps per block, bf16 storage / f32 state, forward only" % (n_in, n, B, nsteps)},
        "useful_tflops": tflops,
        "roofline": {"bound": "mfma", "kernel": "step product [x | h] [W_x ; W_h] (+ concatenation and cell update)",
                     "achieved": tflops, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / BF16_PEAK_TFLOPS,
                     "traffic": None},
    }
    print(json.dumps(out))


def bench_decoder_attention(args, Bn, synth):
    """--config 8: the whole recurrent part of one decoder step (Listing 1): stepped LSTM cell on [trg | att of the previous
    step], attention (energies with weight feedback, softmax over the source positions, accumulated weights, context) and
    readout, for 64 sentences x beam 12.  The context of step i is written straight into the cell input of step i+1, so the
    steps of a block depend on each other exactly as in a search; the target embedding is a fixed random one (choosing the
    output label is not part of this path).  One "step" is a block of 100 dependent decoder steps; the figure of merit is the
    latency of one decoder step."""
    import ctypes as ct
    inp5 = synth.make(5)
    L = inp5["layers"][0]
    dec = synth.make_decoder()
    cfg = dec["cfg"]
    Q, beam, A, E, n, nt, R, S, B = cfg["Q"], cfg["beam"], cfg["A"], cfg["E"], cfg["n"], cfg["n_trg"], cfg["R"], dec["S"], dec["B"]
    nsteps = inp5["cfg"]["steps"]
    assert inp5["cfg"]["n"] == n and inp5["cfg"]["n_in"] == nt + E and inp5["cfg"]["B"] == B
    bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    f32 = lambda a: torch.from_numpy(a).float().cuda()
    Wx, Wh, b = bf(L["W_x"][0]), bf(L["W_h"][0]), f32(L["b"][0])
    enc, W_s, W_r = bf(dec["H"]), bf(dec["W_s"]), bf(dec["W_r"])
    b_s, w_fb, b_fb, v, b_r = (f32(dec[k]) for k in ("b_s", "w_fb", "b_fb", "v", "b_r"))
    lens = torch.from_numpy(dec["src_lens"]).cuda()
    # the loop-invariant projection of the encoder states, once per sentence batch: one product over all S*Q positions
    g = torch.Generator(device="cpu").manual_seed(8)
    W_ctx = ((torch.rand(E, A, generator=g) * 2 - 1) * 0.05).to(torch.bfloat16).cuda()
    ctx = Bn.gemm(enc.view(S * Q, E), W_ctx, a_kcontig=True, b_kcontig=False, M=S * Q, N=A, K=E, out_dtype=torch.bfloat16).view(S, Q, A)
    xin = [torch.zeros(B, nt + E, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    for t in xin:
        t[:, :nt] = bf(dec["trg"])
    state = [torch.zeros(B, n, device="cuda") for _ in range(4)]                  # h, c ping-pong
    accum = [torch.zeros(B, S, device="cuda") for _ in range(2)]
    y = torch.empty(1, B, n, dtype=torch.bfloat16, device="cuda")
    ro = torch.empty(B, R, dtype=torch.bfloat16, device="cuda")
    desc = Bn.make_desc(1, B, nt + E, n, Bn.LSTM_BF16_F32STATE, 1, Bn.FLAG_INFERENCE)
    _, wb = Bn.query(desc, False)
    desc.workspace_bytes = wb
    desc_packed = Bn.make_desc(1, B, nt + E, n, Bn.LSTM_BF16_F32STATE, 1, Bn.FLAG_INFERENCE | Bn.FLAG_WEIGHTS_PACKED)
    desc_packed.workspace_bytes = wb
    ws_cell = torch.empty(wb, dtype=torch.uint8, device="cuda")
    ad = Bn.attention_query(S, Q, beam, A, E, n)
    ws_att = torch.empty(ad.workspace_bytes, dtype=torch.uint8, device="cuda")
    need = ct.c_uint64(0)
    assert Bn.lib.lstm_readout_query(B, R, n, nt, E, ct.byref(need)) == 0
    ws_ro = torch.empty(need.value, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    lib = Bn.lib

    def one(i, first, ev=None):
        p = i % 2
        h0, c0, h1, c1 = (state[0], state[1], state[2], state[3]) if p == 0 else (state[2], state[3], state[0], state[1])
        if ev: ev[0].record()
        rc = lib.lstm_fwd(ct.byref(desc if first else desc_packed), xin[p].data_ptr(), Wx.data_ptr(), Wh.data_ptr(), b.data_ptr(),
                          h0.data_ptr(), c0.data_ptr(), None, y.data_ptr(), None, h1.data_ptr(), c1.data_ptr(), None, ws_cell.data_ptr(), st)
        assert rc == 0, Bn.strerror(rc)
        if ev: ev[1].record()
        rc = lib.lstm_attention_step(ct.byref(ad), enc.data_ptr(), ctx.data_ptr(), lens.data_ptr(), y.data_ptr(), n, W_s.data_ptr(),
                                     b_s.data_ptr(), w_fb.data_ptr(), b_fb.data_ptr(), v.data_ptr(), float(dec["b_e"]), accum[p].data_ptr(),
                                     accum[1 - p].data_ptr(), None, xin[1 - p].data_ptr() + 2 * nt, nt + E, ws_att.data_ptr(), st)
        assert rc == 0, Bn.strerror(rc)
        if ev: ev[2].record()
        rc = lib.lstm_readout(0 if first else Bn.FLAG_WEIGHTS_PACKED, B, R, y.data_ptr(), n, n, xin[p].data_ptr(), nt + E, nt,
                              xin[1 - p].data_ptr() + 2 * nt, nt + E, E, W_r.data_ptr(), b_r.data_ptr(), ro.data_ptr(), R, ws_ro.data_ptr(),
                              ws_ro.numel(), st)
        assert rc == 0, Bn.strerror(rc)
        if ev: ev[3].record()

    def block(first=False):
        for i in range(nsteps):
            one(i, first and i == 0)

    block(True)                                   # packs the weights once
    for _ in range(args.warmup):
        block()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        block()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us = dt / (args.steps * nsteps) * 1e6
    # break-down from one more block with events between the three calls (not part of `value`)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(nsteps)]
    for i in range(nsteps):
        one(i, False, evs[i])
    torch.cuda.synchronize()
    part = [sum(e[k].elapsed_time(e[k + 1]) for e in evs) / nsteps * 1e3 for k in range(3)]
    # attention energies: per (row, valid source position, attention feature) 11 float operations (multiply-add of the weight
    # feedback, add of s_tr, tanh as 2x, exp, +1, reciprocal, multiply-add, multiply-add into the sum), on the vector ALU
    valid = int(dec["src_lens"].astype("int64").sum()) * beam
    alu_flops = 11.0 * valid * A
    mfma_flops = 2.0 * B * (n * (nt + E + n) * 4 + n * A + (n + nt + E) * R)
    out = {
        "metric": "attention decoder step latency (n=%d, %d rows)" % (n, B), "value": us, "unit": "us/step", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 8: LSTM cell (620 + 2000 -> %d) + attention over S<=%d source positions (A=%d, E=%d, weight "
                               "feedback) + readout (-> %d), %d sentences x beam %d = %d rows, %d dependent steps per block, bf16 storage, "
                               "forward only" % (n, S, A, E, R, Q, beam, B, nsteps)},
        "us_per_step_cell_attention_readout": part,
        "useful_tflops_products": mfma_flops / (us * 1e-6) / 1e12,
        "roofline": {"bound": "alu", "kernel": "att_energy_kernel (inside the attention call, which also runs the s_tr product and "
                                               "att_context_kernel)", "achieved": alu_flops / (part[1] * 1e-6) / 1e12, "peak": 157.3,
                     "unit": "TFLOP/s", "frac": alu_flops / (part[1] * 1e-6) / 1e12 / 157.3, "traffic": None,
                     "note": "achieved = energy flops / time of the whole attention call (s_tr product, energies, softmax, context); "
                             "the kernel alone: profiles/bench_config8_kernel_trace.txt"},
    }
    print(json.dumps(out))


def bench_search_step(args, Bn, synth):
    """--config 9: one complete step of the batched beam search (Sec. 3, Table 2; Listing 1): cell, attention, readout, output
    layer over V = 20000 labels, beam step, state gather and target embedding, for 64 sentences x beam 12, with no host
    round trip between the steps: the labels and hypotheses chosen in step i feed step i+1 on the device.  One "step" is a
    block of 50 dependent search steps; the figure of merit is the latency of one search step."""
    import ctypes as ct
    inp5 = synth.make(5)
    L = inp5["layers"][0]
    dec = synth.make_decoder()
    cfg = dec["cfg"]
    Q, beam, A, E, n, nt, R, S, B = cfg["Q"], cfg["beam"], cfg["A"], cfg["E"], cfg["n"], cfg["n_trg"], cfg["R"], dec["S"], dec["B"]
    V, nsteps = 20000, 50
    bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    f32 = lambda a: torch.from_numpy(a).float().cuda()
    Wx, Wh, b = bf(L["W_x"][0]), bf(L["W_h"][0]), f32(L["b"][0])
    enc, W_s, W_r = bf(dec["H"]), bf(dec["W_s"]), bf(dec["W_r"])
    b_s, w_fb, b_fb, v, b_r = (f32(dec[k]) for k in ("b_s", "w_fb", "b_fb", "v", "b_r"))
    lens = torch.from_numpy(dec["src_lens"]).cuda()
    g = torch.Generator(device="cpu").manual_seed(9)
    u = lambda *shape: torch.rand(*shape, generator=g) * 2 - 1
    W_ctx = (u(E, A) * 0.05).to(torch.bfloat16).cuda()
    W_o = (u(V, R) * 0.1).to(torch.bfloat16).cuda()              # output layer, a row per label
    b_o = (u(V) * 0.5).cuda()
    W_trg = (u(V, nt) * 0.5).to(torch.bfloat16).cuda()            # target embedding table
    ctx = Bn.gemm(enc.view(S * Q, E), W_ctx, a_kcontig=True, b_kcontig=False, M=S * Q, N=A, K=E, out_dtype=torch.bfloat16).view(S, Q, A)
    z = lambda *shape, dt=torch.float32: torch.zeros(*shape, dtype=dt, device="cuda")
    xin = [z(B, nt + E, dt=torch.bfloat16) for _ in range(2)]
    h, c, accum, score = [z(B, n) for _ in range(2)], [z(B, n) for _ in range(2)], [z(B, S) for _ in range(2)], [z(Q, beam) for _ in range(2)]
    score[0][:, 1:] = float("-inf")                               # first step: one live hypothesis per sentence
    h_new, c_new, accum_new = z(B, n), z(B, n), z(B, S)
    att_buf, y, ro = z(B, E, dt=torch.bfloat16), z(1, B, n, dt=torch.bfloat16), z(B, R, dt=torch.bfloat16)
    logits = torch.empty(B, V, dtype=torch.float32, device="cuda")
    src, label = torch.zeros(Q, beam, dtype=torch.int32, device="cuda"), torch.zeros(Q, beam, dtype=torch.int32, device="cuda")
    desc = Bn.make_desc(1, B, nt + E, n, Bn.LSTM_BF16_F32STATE, 1, Bn.FLAG_INFERENCE)
    _, wb = Bn.query(desc, False)
    desc.workspace_bytes = wb
    desc_packed = Bn.make_desc(1, B, nt + E, n, Bn.LSTM_BF16_F32STATE, 1, Bn.FLAG_INFERENCE | Bn.FLAG_WEIGHTS_PACKED)
    desc_packed.workspace_bytes = wb
    ws_cell = torch.empty(wb, dtype=torch.uint8, device="cuda")
    ad = Bn.attention_query(S, Q, beam, A, E, n)
    ws_att = torch.empty(ad.workspace_bytes, dtype=torch.uint8, device="cuda")
    need = ct.c_uint64(0)
    assert Bn.lib.lstm_readout_query(B, R, n, nt, E, ct.byref(need)) == 0
    ws_ro = torch.empty(need.value, dtype=torch.uint8, device="cuda")
    assert Bn.lib.lstm_beam_query(Q, beam, V, ct.byref(need)) == 0
    ws_beam = torch.empty(need.value, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    lib = Bn.lib
    NEV = 6
    # what follows the hypotheses after a step, per parity of the step (the buffers alternate): one launch for all four
    gather = [Bn.gather_items([(h_new, h[1 - p]), (c_new, c[1 - p]), (accum_new, accum[1 - p]), (att_buf, xin[1 - p][:, nt:])]) for p in range(2)]

    def one(i, first, ev=None):
        p = i % 2
        ck = lambda rc: Bn._check(rc)
        if ev: ev[0].record()
        ck(lib.lstm_fwd(ct.byref(desc if first else desc_packed), xin[p].data_ptr(), Wx.data_ptr(), Wh.data_ptr(), b.data_ptr(),
                        h[p].data_ptr(), c[p].data_ptr(), None, y.data_ptr(), None, h_new.data_ptr(), c_new.data_ptr(), None, ws_cell.data_ptr(), st))
        if ev: ev[1].record()
        ck(lib.lstm_attention_step(ct.byref(ad), enc.data_ptr(), ctx.data_ptr(), lens.data_ptr(), y.data_ptr(), n, W_s.data_ptr(),
                                   b_s.data_ptr(), w_fb.data_ptr(), b_fb.data_ptr(), v.data_ptr(), float(dec["b_e"]), accum[p].data_ptr(),
                                   accum_new.data_ptr(), None, att_buf.data_ptr(), E, ws_att.data_ptr(), st))
        if ev: ev[2].record()
        ck(lib.lstm_readout(0 if first else Bn.FLAG_WEIGHTS_PACKED, B, R, y.data_ptr(), n, n, xin[p].data_ptr(), nt + E, nt,
                            att_buf.data_ptr(), E, E, W_r.data_ptr(), b_r.data_ptr(), ro.data_ptr(), R, ws_ro.data_ptr(), ws_ro.numel(), st))
        if ev: ev[3].record()
        ck(lib.lstm_gemm(1, 0, 1, 1, B, V, R, ro.data_ptr(), R, W_o.data_ptr(), R, logits.data_ptr(), V, b_o.data_ptr(), 0, None, 1, 0, st))
        if ev: ev[4].record()
        ck(lib.lstm_beam_step(Q, beam, V, logits.data_ptr(), V, score[p].data_ptr(), score[1 - p].data_ptr(), src.data_ptr(), label.data_ptr(),
                              ws_beam.data_ptr(), ws_beam.numel(), st))
        # the state rows follow their hypotheses: h, c, the attention's accumulated weights and the context (into the next input)
        ck(lib.lstm_beam_gather_many(Q, beam, 4, gather[p], src.data_ptr(), st))
        ck(lib.lstm_embed(B, nt, V, label.data_ptr(), W_trg.data_ptr(), None, xin[1 - p].data_ptr(), nt + E, st))
        if ev: ev[5].record()

    def block(first=False):
        for i in range(nsteps):
            one(i, first and i == 0)

    block(True)
    for _ in range(args.warmup):
        block()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        block()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us = dt / (args.steps * nsteps) * 1e6
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(NEV)] for _ in range(nsteps)]
    for i in range(nsteps):
        one(i, False, evs[i])
    torch.cuda.synchronize()
    part = [sum(e[k].elapsed_time(e[k + 1]) for e in evs) / nsteps * 1e3 for k in range(NEV - 1)]
    assert bool(torch.isfinite(score[0]).all()) and int(label.min()) >= 0 and int(label.max()) < V and int(src.max()) < beam
    # beam step: algorithmic bytes = the logits read once (they were just written by the output layer)
    beam_bytes = float(B) * V * 4
    out = {
        "metric": "beam search step latency (n=%d, %d rows, V=%d)" % (n, B, V), "value": us, "unit": "us/step", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config 9: config 8's decoder step + output layer (%d -> %d labels) + beam step (beam %d) + state gather + "
                               "target embedding; %d sentences, %d rows, %d dependent steps per block, no host round trip" % (R, V, beam, Q, B, nsteps)},
        "us_per_step_cell_attention_readout_output_beam": part,
        "roofline": {"bound": "hbm", "kernel": "beam step + gathers + embedding (beam_row_kernel dominates: one read of the logits)",
                     "achieved": beam_bytes / (part[4] * 1e-6) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": beam_bytes / (part[4] * 1e-6) / 1e9 / HBM_PEAK_GBS, "traffic": None},
    }
    print(json.dumps(out))


class PooledStack:
    """The config-4 stack with max-pooling in time (windows of 2 frames) behind layers 1, 2 and 3: the shape of the
    paper's attention-based speech encoder (6 bidirectional layers, input shortened by a factor of 8 in total)."""

    def __init__(self, Bn, x, lens, dy_top, layers, pool_after=(0, 1, 2), pool=2):
        import ctypes
        self.Bn, self.ct, self.layers, self.pool, self.pool_after = Bn, ctypes, layers, pool, set(pool_after)
        dev = x.device
        B = x.shape[1]
        n = layers[0][1].shape[-2]
        dtype_id = Bn.LSTM_BF16_F32STATE if x.dtype == torch.bfloat16 else Bn.LSTM_F32
        self.dtype_id = dtype_id
        self.bufs, wmax, cur, cur_lens, lens_np = [], 0, x, lens, lens.cpu().numpy()
        self.frames_per_layer = []
        for k, (Wx, Wh, b) in enumerate(layers):
            T, cur_in = cur.shape[0], cur.shape[2]
            desc = Bn.make_desc(T, B, cur_in, n, dtype_id, 1, LAUNCH_FLAGS)
            rb, wb = Bn.query(desc, True)
            wmax = max(wmax, wb)
            desc.reserve_bytes = rb
            self.frames_per_layer.append(int(lens_np.sum()))
            bf = dict(desc=desc, T=T, xin=cur, lens=cur_lens, reserve=torch.empty(rb, dtype=torch.uint8, device=dev),
                      y=torch.empty(T, B, 2 * n, dtype=x.dtype, device=dev), c=torch.empty(2, T, B, n, dtype=torch.float32, device=dev),
                      dx=torch.empty(T, B, cur_in, dtype=x.dtype, device=dev), dW_x=torch.empty_like(Wx, dtype=torch.float32),
                      dW_h=torch.empty_like(Wh, dtype=torch.float32), db=torch.empty(2, 4 * n, dtype=torch.float32, device=dev))
            cur = bf["y"]
            if k in self.pool_after:
                Tp = -(-T // pool)
                bf.update(pooled=torch.empty(Tp, B, 2 * n, dtype=x.dtype, device=dev), arg=torch.empty(Tp, B, 2 * n, dtype=torch.uint8, device=dev),
                          lens_out=torch.empty(B, dtype=torch.int32, device=dev), dy=torch.empty(T, B, 2 * n, dtype=x.dtype, device=dev))
                cur = bf["pooled"]
                cur_lens = bf["lens_out"]
                lens_np = -(-lens_np // pool)
            self.bufs.append(bf)
        self.dy_top = dy_top[:cur.shape[0]].contiguous()
        self.ws = torch.empty(wmax, dtype=torch.uint8, device=dev)
        for bf in self.bufs:
            bf["desc"].workspace_bytes = wmax
        self.pool_events = []

    def step(self, timed=False):
        Bn, ct, lib = self.Bn, self.ct, self.Bn.lib
        s = torch.cuda.current_stream().cuda_stream
        ev = lambda: torch.cuda.Event(enable_timing=True)
        F = self.bufs[0]["y"].shape[2]
        for (Wx, Wh, b), bf in zip(self.layers, self.bufs):
            rc = lib.blstm_fwd(ct.byref(bf["desc"]), bf["xin"].data_ptr(), Wx.data_ptr(), Wh.data_ptr(), b.data_ptr(), None, None,
                               bf["lens"].data_ptr(), bf["y"].data_ptr(), bf["c"].data_ptr(), None, None, bf["reserve"].data_ptr(),
                               self.ws.data_ptr(), s)
            assert rc == 0, Bn.strerror(rc)
            if "pooled" in bf:
                e0, e1 = ev(), ev()
                e0.record()
                rc = lib.lstm_time_pool_fwd(self.dtype_id, bf["T"], bf["y"].shape[1], F, self.pool, bf["y"].data_ptr(), F, bf["lens"].data_ptr(),
                                            bf["pooled"].data_ptr(), F, bf["arg"].data_ptr(), bf["lens_out"].data_ptr(), s)
                e1.record()
                assert rc == 0, Bn.strerror(rc)
                if timed:
                    self.pool_events.append(("fwd", bf["T"], e0, e1))
        d = self.dy_top
        for k in range(len(self.layers) - 1, -1, -1):
            Wx, Wh, b = self.layers[k]
            bf = self.bufs[k]
            if "pooled" in bf:                                   # d is the gradient of the pooled output
                e0, e1 = ev(), ev()
                e0.record()
                rc = lib.lstm_time_pool_bwd(self.dtype_id, bf["T"], bf["y"].shape[1], F, self.pool, d.data_ptr(), F, bf["arg"].data_ptr(),
                                            bf["lens"].data_ptr(), bf["dy"].data_ptr(), F, s)
                e1.record()
                assert rc == 0, Bn.strerror(rc)
                if timed:
                    self.pool_events.append(("bwd", bf["T"], e0, e1))
                d = bf["dy"]
            rc = lib.blstm_bwd(ct.byref(bf["desc"]), bf["xin"].data_ptr(), Wx.data_ptr(), Wh.data_ptr(), None, None, bf["lens"].data_ptr(),
                               bf["y"].data_ptr(), bf["c"].data_ptr(), bf["reserve"].data_ptr(), d.data_ptr(), None, None, bf["dx"].data_ptr(),
                               bf["dW_x"].data_ptr(), bf["dW_h"].data_ptr(), bf["db"].data_ptr(), None, None, self.ws.data_ptr(), s)
            assert rc == 0, Bn.strerror(rc)
            d = bf["dx"]


def bench_pooled(args, Bn, synth):
    """--config 6: config 4's stack with max-pooling in time behind layers 1, 2 and 3 (total factor 8)."""
    inp = synth.make(4)
    cfg = inp["cfg"]
    frames = synth.real_frames(inp)
    x, lens, dy, layers = build_stack(inp, Bn)
    st = PooledStack(Bn, x, lens, dy, layers)
    if args.copy_calibration:                       # a plain copy of known size, for scaling the HBM byte counters
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        st.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        st.step(timed=True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    B, n, esz = cfg["B"], cfg["n"], 2
    F = 2 * n
    # pooling kernels: algorithmic bytes = real input frames read once + every output frame written once (+ one argument byte
    # per element of a real output frame);
    # the backward kernel writes every frame of dy, padded ones included (zeros), so that nothing has to be cleared first
    ms = {"fwd": 0.0, "bwd": 0.0}
    by = {"fwd": 0.0, "bwd": 0.0}
    for kind, T, e0, e1 in st.pool_events:
        ms[kind] += e0.elapsed_time(e1)
    for k, bf in enumerate(st.bufs):
        if "pooled" not in bf:
            continue
        fin, fout = st.frames_per_layer[k], st.frames_per_layer[k + 1]
        Tp = -(-bf["T"] // st.pool)
        by["fwd"] += args.steps * (fin * F * esz + Tp * B * F * esz + fout * F)          # out is defined (zero) at padded frames too
        by["bwd"] += args.steps * (fout * F * (esz + 1) + bf["T"] * B * F * esz)
    tot_ms, tot_by = ms["fwd"] + ms["bwd"], by["fwd"] + by["bwd"]
    traffic = None
    try:   # HBM bytes of the six pooling launches of one step, measured with rocprofv3 --pmc (see profiles/)
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as fh:
            traffic = json.load(fh).get("config6_pool_bytes_per_step")
    except (OSError, ValueError):
        pass
    gbs = tot_by / (tot_ms * 1e-3) / 1e9 if tot_ms > 0 else 0.0
    out = {
        "metric": "BLSTM fwd+bwd frames/sec (n=%d), encoder with time pooling" % n, "value": frames * args.steps / dt, "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "config 6: config 4's 6-layer BLSTM stack (n_in=40, n=%d, B=%d, T=%d, %d real input frames) with max-pooling "
                               "in time, windows of 2 frames, behind layers 1, 2 and 3; frames per layer %s; forward + backward" % (
                                   n, B, inp["T"], frames, st.frames_per_layer)},
        "roofline": {"bound": "hbm", "kernel": "time_pool_fwd_kernel + time_pool_bwd_kernel (three of each per step)", "achieved": gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "ms_per_step": tot_ms / args.steps, "algorithmic_bytes_per_step": tot_by / args.steps},
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4, help="synthetic configuration (4 = headline, n = 1024; 2, 3 = other BLSTM stacks; 5 = stepped decoder cell; 6 = config 4 with max-pooling in time between layers; 7 = one bidirectional layer below five unidirectional ones; 8 = decoder step with attention and readout; 9 = complete beam-search step)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--per-step", action="store_true", help="force one launch per time step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    from paper_1805_05225_amd import binding as Bn
    from paper_1805_05225_amd import synth

    torch.cuda.set_device(0)
    if args.config == 5:
        bench_decoder(args, Bn, synth)
        return
    if args.config == 6:
        bench_pooled(args, Bn, synth)
        return
    if args.config == 7:
        bench_mixed(args, Bn, synth)
        return
    if args.config == 8:
        bench_decoder_attention(args, Bn, synth)
        return
    if args.config == 9:
        bench_search_step(args, Bn, synth)
        return
    inp = synth.make(args.config)
    cfg = inp["cfg"]
    assert cfg["kind"] == "blstm"
    frames = synth.real_frames(inp)
    flops = synth.flops_fwd_bwd(inp)
    x, lens, dy, layers = build_stack(inp, Bn)
    st = Stack(Bn, x, lens, dy, layers)
    if args.per_step:
        for bf in st.bufs:
            bf["desc"].flags |= Bn.FLAG_PER_STEP

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        st.step()
    torch.cuda.synchronize()
    Bn.profile_enable(1)              # loops and products only: an event between kernels idles the device for microseconds
    t0 = time.perf_counter()
    for _ in range(args.steps):
        st.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    Bn.profile_enable(False)
    prof = Bn.profile_read()
    st.verify()                       # the last call of the timed region
    st.step(check=True)               # and one untimed step with the word checked behind every call

    ms_per_step = dt / args.steps * 1e3
    T, B, n = inp["T"], cfg["B"], cfg["n"]
    esz = 2 if cfg["dtype"] == "bf16" else 4
    nl = cfg["layers"]
    # Algorithmic HBM bytes of the recurrent loops, W_h resident on chip, per REAL frame of one row and one direction
    # (the kernels skip padded frames, and so does this count):
    #   forward : read Zx_t (4n*4), write gate activations (4n*4), c_t (n*4), y_t (n*esz); c_{t-1} stays on chip
    #   backward: read gate activations (4n*4), c_t and c_{t-1} (2*n*4), dy_t (n*esz); write dz_t (4n*esz)
    # A launch (one layer, both directions) touches `frames` real frames per direction and walks T time steps.
    fwd_row_bytes = 2 * 4 * n * 4 + n * 4 + n * esz
    bwd_row_bytes = 4 * n * 4 + 2 * n * 4 + n * esz + 4 * n * esz
    steps_total = args.steps * nl * T
    traffic = {}
    try:   # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/)
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as fh:
            tr = json.load(fh)
        if tr.get("workload") == "config %d" % args.config:
            traffic = {"loop_bwd": tr.get("persist_bwd_bytes_per_launch"), "loop_fwd": tr.get("persist_fwd_bytes_per_launch")}
    except (OSError, ValueError):
        pass

    def loop_roofline(phase, row_bytes, name):
        ms, launches = prof[phase]
        layer_runs = args.steps * nl                                # times the loop of one layer ran in the timed region
        per_layer = launches / max(layer_runs, 1)                   # 1; 2 where the batch takes two launches; T on the per-step path
        per_step_path = T > 2 and per_layer >= T                    # one launch per time step: W_h is not resident
        per_launch_ms = ms / max(launches, 1)
        layer_ms = ms / max(layer_runs, 1)
        frame_bytes = row_bytes * frames * 2                        # both directions, real frames only
        # With one launch per time step nothing stays on chip between launches: every launch also reads W_h of both
        # directions (n x 4n values each), which belongs to the algorithmic bytes of THAT kernel.
        weight_bytes = 2 * n * 4 * n * esz * T if per_step_path else 0
        layer_bytes = frame_bytes + weight_bytes
        launch_bytes = layer_bytes / max(per_layer, 1)
        achieved = layer_bytes / (layer_ms * 1e-3) / 1e9 if ms > 0 else 0.0
        padded = (row_bytes * T * B * 2 + weight_bytes) / (layer_ms * 1e-3) / 1e9 if ms > 0 else 0.0
        step_bytes = layer_bytes / T
        tr_bytes = None if per_step_path else traffic.get(phase)
        # the recurrent product itself (h W_h or dz W_h^T: 8 n^2 flops per real frame of a row) against the MFMA peak of
        # the storage type: what bounds the float single-launch kernel (the float MFMA runs at 1/16 of the bf16 rate)
        rec_tflops = 8.0 * n * n * frames * 2 / (layer_ms * 1e-3) / 1e12 if ms > 0 else 0.0
        mfma_peak_loop = BF16_PEAK_TFLOPS if esz == 2 else 157.3
        return {"bound": "hbm", "kernel": name + (" (one launch per time step)" if per_step_path else ""),
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": tr_bytes,
                "recurrent_product_tflops": rec_tflops, "recurrent_product_frac_of_mfma_peak": rec_tflops / mfma_peak_loop,
                "recurrent_product_frac_counting_padded_rows": rec_tflops * (T * B) / max(frames, 1) / mfma_peak_loop,
                "traffic_ratio": (tr_bytes / launch_bytes) if tr_bytes else None, "launches": int(launches),
                "avg_launch_ms": per_launch_ms, "us_per_time_step": ms * 1e3 / max(steps_total, 1),
                "step_roofline_us": step_bytes / (HBM_PEAK_GBS * 1e9) * 1e6,
                "algorithmic_bytes_per_launch": launch_bytes, "algorithmic_bytes_per_time_step": step_bytes,
                "weight_bytes_per_launch": (2 * n * 4 * n * esz) if per_step_path else 0,
                "frac_counting_padded_frames": padded / HBM_PEAK_GBS}

    roof_bwd = loop_roofline("loop_bwd", bwd_row_bytes, "backward recurrent loop (both directions)")
    roof_fwd = loop_roofline("loop_fwd", fwd_row_bytes, "forward recurrent loop (both directions)")
    # hoisted products: algorithmic flops per benchmark step (the products run over the real frames only)
    gemm_flops = {"gemm_zx": 0.0, "gemm_dx": 0.0, "gemm_dwx": 0.0, "gemm_dwh": 0.0}
    for l in range(nl):
        ni = cfg["n_in"] if l == 0 else 2 * n
        gemm_flops["gemm_zx"] += 2.0 * frames * ni * 8 * n
        gemm_flops["gemm_dx"] += 2.0 * frames * ni * 8 * n
        gemm_flops["gemm_dwx"] += 2.0 * frames * ni * 8 * n
        gemm_flops["gemm_dwh"] += 2.0 * frames * n * 8 * n
    per_product = {k: (v * args.steps / (prof[k][0] * 1e-3) / 1e12 if prof[k][0] > 0 else 0.0) for k, v in gemm_flops.items()}
    gemm_ms = sum(prof[k][0] for k in gemm_flops)
    gemm_tflops = sum(gemm_flops.values()) * args.steps / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    mfma_peak = BF16_PEAK_TFLOPS if esz == 2 else 157.3
    dominant = roof_bwd if prof["loop_bwd"][0] >= prof["loop_fwd"][0] else roof_fwd

    out = {
        "metric": "BLSTM fwd+bwd frames/sec (n=%d)" % n, "value": frames * args.steps / dt, "unit": "frames/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "config %d: %d-layer BLSTM stack, n_in=%d, n=%d per direction, B=%d, seq_lens~U{%d..%d} "
                               "(T=%d, %d real frames), %s storage / f32 state, forward + backward" % (
                                   args.config, nl, cfg["n_in"], n, B, cfg["len_lo"], cfg["len_hi"], T, frames,
                                   cfg["dtype"]),
                   "recurrent_path": "per_step" if args.per_step else "default", "launch": "plain (LSTM_FLAG_PLAIN_LAUNCH)"},
        "useful_tflops": flops * args.steps / dt / 1e12,
        "roofline": dominant,
        "roofline_forward_loop": roof_fwd if dominant is roof_bwd else roof_bwd,
        "roofline_hoisted_gemms": {"bound": "mfma", "achieved": gemm_tflops, "peak": mfma_peak, "unit": "TFLOP/s",
                                   "frac": gemm_tflops / mfma_peak, "tflops_per_product": per_product,
                                   "note": "flops of the four hoisted products per layer over the real frames; the operand "
                                           "transposes and the frame map are inside the timed phases"},
        "phases_ms_per_step": {k: v[0] / args.steps for k, v in prof.items()},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
