#!/usr/bin/env python3
"""Benchmark of the conv-GLU + CTC training step on one MI355X.

One "step" = one full forward + criterion + backward pass (w2l_train_step) of the
~105M-parameter bf16 model over one synthetic batch (B=8, T_b ~ U[1000,1500] padded to
1500, 80-dim features; seed 4), inputs resident in HBM before the timed region.
Prints ONE JSON line: training frames/s (valid input frames per second), ms/step, the
roofline of the dominant kernel measured live with events on the launch stream, and the
fp64 CPU oracle timed on the host cores on a bounded sample (a baseline, not the target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15   # dense bf16 MFMA, FLOP/s (MI355X published)
PEAK_HBM = 8.0e12         # B/s
# one step of the criterion recursions on one wavefront with nothing else (no memory traffic, no hand-over):
# CTC 24 instructions (21 vector, the row store, the LDS read, the row-offset add) at the 4-cycle issue cadence,
# ASG's fully connected lattice about 175 cycles, at 2.4 GHz
CTC_BARE_STEP_NS = 40.0
ASG_BARE_STEP_NS = 73.0

# HBM bytes per launch of the dominant kernel, from two `rocprofv3 --pmc` runs
# (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch, scaled by the same counters' reading for a
# device copy of known size).  The runs and the factor are recorded in
# profiles/conv_kernels_config4_body_hbm_traffic.txt.
# (The staging copy each entry point runs first moves another 19 to 57 MB; it is a separate kernel.)
DOMINANT_KERNEL_HBM_BYTES = {"conv1d_bwd_data": 156457160, "conv1d_fwd": 109046066, "conv1d_bwd_weight": 202503374}


def event_time_ms(fn, iters, warmup=None):
    """Average milliseconds per call, HIP events on torch's current stream (the launch stream)."""
    import torch
    if warmup is None:
        warmup = max(2, iters // 10)  # short bursts run at a different clock than sustained work
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


SHORT_TIMING = {"method": "hip graph replay"}


def graph_time_ms(calls, iters, out=None):
    """Average milliseconds per call of launches that run for a few microseconds.  A call through the Python binding
    costs the host about 8 us, more than these kernels run, so a loop of calls measures the caller; here the calls
    (`calls`: a list of them, at least 16 go into one graph) are captured into a HIP graph on a side stream and the
    graph is replayed, which leaves the spacing of the launches to the device.  `out`, if given, is a tensor the
    calls write: what the replays leave in it must equal what the eager calls left.  Should capture fail, the loop
    of calls is timed instead and SHORT_TIMING says so."""
    import torch
    seq = list(calls) * max(1, -(-16 // len(calls)))
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in seq:
                c()
            torch.cuda.synchronize()
            eager = out.clone() if out is not None else None
            if out is not None:
                out.zero_()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for c in seq:
                    c()
            reps = max(2, iters // len(seq))
            for _ in range(max(2, reps // 10)):
                g.replay()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                g.replay()
            b.record()
            torch.cuda.synchronize()
        torch.cuda.current_stream().wait_stream(side)
        if out is not None and not torch.equal(out, eager):
            raise RuntimeError("bench.py: graph replays of a kernel left other values than its eager launches")
        return a.elapsed_time(b) / (reps * len(seq))
    except RuntimeError:
        raise
    except Exception as e:  # measured anyway, by the slower method, and reported as such
        SHORT_TIMING["method"] = "loop of calls (graph capture failed: %s)" % type(e).__name__
        torch.cuda.synchronize()
        it = iter(range(1 << 30))
        return event_time_ms(lambda: seq[next(it) % len(seq)](), iters)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-iters", type=int, default=200)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    import paper_1812_07625_amd as P
    from workloads.device import to_dev, empty

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    cfg = W.config4()
    layers, B, T = cfg["layers"], cfg["B"], cfg["T"]
    xd = to_dev(cfg["x"], "bf16")
    wd = [to_dev(w, "bf16") for w in cfg["weights"]]
    bd = [to_dev(b) for b in cfg["biases"]]
    dwd = [empty(w.shape) for w in cfg["weights"]]
    dbd = [empty(b.shape) for b in cfg["biases"]]
    tg, il, tl = to_dev(cfg["targets"]), to_dev(cfg["in_len"]), to_dev(cfg["tgt_len"])
    Lmax = cfg["targets"].shape[1]
    ws = P.workspace(P.w2l_train_step_workspace_bytes(layers, B, T, Lmax, P.W2L_BF16))
    loss = empty((B,))

    def step():
        P.w2l_train_step(layers, wd, bd, dwd, dbd, xd, il, tg, tl, loss, None, 0, 1.0, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    lv = loss.cpu().numpy()
    assert np.all(np.isfinite(lv)), "non-finite loss in the benchmark step"
    # the same step over at least half a second of back-to-back launches, whatever --steps was: the part's clock
    # under a matrix load settles only after some tens of milliseconds, so a short burst reads differently
    n_sus = max(args.steps, int(0.5 / dt) + 1)
    for _ in range(10):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n_sus):
        step()
    torch.cuda.synchronize()
    dt_sus = (time.perf_counter() - t0) / n_sus

    frames = int(cfg["in_len"].sum())
    flops = W.step_flops(layers, B, T)

    # ---- measured ceilings: matrix pipe alone (with constant and with random operand bits: the part is
    # power-limited and the multipliers' power follows the bits that toggle), and a plain device copy
    sink = empty((2048 * 256,))
    probe_flop = [0.0]

    def probe(random_operands):
        probe_flop[0] = P.w2l_probe_mfma(sink, 2048, 2000, random_operands)

    t_probe = event_time_ms(lambda: probe(False), 3, 1)
    mfma_ceiling_const = probe_flop[0] / (t_probe * 1e-3)
    t_probe = event_time_ms(lambda: probe(True), 3, 1)
    mfma_ceiling = probe_flop[0] / (t_probe * 1e-3)
    cbuf_a = torch.empty(1 << 29, dtype=torch.uint8, device="cuda:0")
    cbuf_b = torch.empty_like(cbuf_a)
    t_copy = event_time_ms(lambda: cbuf_b.copy_(cbuf_a), 5, 2)
    copy_bw = 2.0 * cbuf_a.numel() / (t_copy * 1e-3)
    del cbuf_a, cbuf_b

    # ---- per-kernel figures at the body-layer shape (k=11, 768 -> 1536, M = B*T' = 6000),
    # through the same entry points and kernels the train step launches (operands staged into
    # the zero-haloed layout inside the call, as the step keeps them)
    L = layers[1]
    Tp = (T + layers[0]["stride"] - 1) // layers[0]["stride"]
    rng = np.random.default_rng(0)
    hx = to_dev(W.round_to_bf16(rng.standard_normal((B, Tp, L["cin"])).astype(np.float32)), "bf16")
    hdy = to_dev(W.round_to_bf16(rng.standard_normal((B, Tp, L["cout"])).astype(np.float32)), "bf16")
    hy = empty((B, Tp, L["cout"]), "bf16")
    hdx = empty((B, Tp, L["cin"]), "bf16")
    hdw = empty(cfg["weights"][1].shape)
    shp = (B, Tp, L["cin"], L["cout"], L["k"], 1, P.W2L_BF16)
    ws_f = P.workspace(P.w2l_conv1d_fwd_workspace_bytes(*shp))
    ws_d = P.workspace(P.w2l_conv1d_bwd_data_workspace_bytes(*shp))
    ws_w = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(*shp))
    gf = 2.0 * B * Tp * L["k"] * L["cin"] * L["cout"]
    kern = {}
    kern["conv1d_fwd"] = event_time_ms(lambda: P.w2l_conv1d_fwd(hx, wd[1], bd[1], hy, 1, ws_f), args.kernel_iters)
    kern["conv1d_bwd_data"] = event_time_ms(lambda: P.w2l_conv1d_bwd_data(hdy, wd[1], hdx, 1, ws_d),
                                            args.kernel_iters)
    kern["conv1d_bwd_weight"] = event_time_ms(
        lambda: P.w2l_conv1d_bwd_weight(hx, hdy, hdw, None, 1, False, ws_w), args.kernel_iters)
    # the step runs 8 body layers x (fwd, dgrad, wgrad) + the 1x1 layers: the pass that costs
    # the most per launch is the dominant kernel
    dom = max(kern, key=kern.get)
    achieved = gf / (kern[dom] * 1e-3)

    # bandwidth-bound kernels at the same layer's shape
    rows = B * Tp
    hh = empty((rows, L["cout"] // 2), "bf16")
    t_glu = graph_time_ms([lambda: P.w2l_glu_fwd(hy, hh)], args.kernel_iters, out=hh)
    glu_bytes = rows * L["cout"] * 2 + rows * (L["cout"] // 2) * 2
    hdh = to_dev(W.round_to_bf16(rng.standard_normal((rows, L["cout"] // 2)).astype(np.float32)), "bf16")
    hdy2 = empty((rows, L["cout"]), "bf16")
    t_glub = graph_time_ms([lambda: P.w2l_glu_bwd(hy, hdh, hdy2)], args.kernel_iters, out=hdy2)
    glub_bytes = rows * L["cout"] * 2 * 2 + rows * (L["cout"] // 2) * 2
    # what a plain device copy moving the same number of bytes achieves (half read, half written): at a few tens of
    # megabytes a launch is a handful of microseconds and its ramp-up and tail are a visible part of it
    def copy_rate(nbytes):
        a = torch.empty(nbytes // 2, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        t = graph_time_ms([lambda: b.copy_(a)], args.kernel_iters)
        return 2.0 * a.numel() / (t * 1e-3)

    copy_glu, copy_glub = copy_rate(glu_bytes), copy_rate(glub_bytes)
    # the same two kernels rotating over 16 sets of buffers (0.44 / 0.74 GB), so that no launch finds its
    # operands in the 256 MB memory-side cache: the figure against HBM proper
    nset = 16
    ys = [torch.empty_like(hy).copy_(hy) for _ in range(nset)]
    hs = [torch.empty_like(hh) for _ in range(nset)]
    dhs = [torch.empty_like(hdh).copy_(hdh) for _ in range(nset)]
    dys = [torch.empty_like(hdy2) for _ in range(nset)]
    t_glu_cold = graph_time_ms([(lambda i=i: P.w2l_glu_fwd(ys[i], hs[i])) for i in range(nset)], args.kernel_iters)
    t_glub_cold = graph_time_ms([(lambda i=i: P.w2l_glu_bwd(ys[i], dhs[i], dys[i])) for i in range(nset)],
                                args.kernel_iters)
    del ys, hs, dhs, dys

    # config 1: one conv layer k=11, 512 -> 1024, B=16, T=800 (147.64 GFLOP per pass; bar: 118 us = half the MFMA peak)
    c1 = W.config1()
    c1x, c1w, c1dy = to_dev(c1["x"], "bf16"), to_dev(c1["w"], "bf16"), to_dev(c1["dy"], "bf16")
    c1y, c1dx, c1dw = empty(c1["dy"].shape, "bf16"), empty(c1["x"].shape, "bf16"), empty(c1["w"].shape)
    shp1 = (c1["B"], c1["T"], c1["Cin"], c1["Cout"], c1["k"], 1, P.W2L_BF16)
    w1f = P.workspace(P.w2l_conv1d_fwd_workspace_bytes(*shp1))
    w1d = P.workspace(P.w2l_conv1d_bwd_data_workspace_bytes(*shp1))
    w1w = P.workspace(P.w2l_conv1d_bwd_weight_workspace_bytes(*shp1))
    gf1 = 2.0 * c1["B"] * c1["T"] * c1["k"] * c1["Cin"] * c1["Cout"]
    kern1 = {
        "conv1d_fwd": event_time_ms(lambda: P.w2l_conv1d_fwd(c1x, c1w, None, c1y, 1, w1f), args.kernel_iters),
        "conv1d_bwd_data": event_time_ms(lambda: P.w2l_conv1d_bwd_data(c1dy, c1w, c1dx, 1, w1d), args.kernel_iters),
        "conv1d_bwd_weight": event_time_ms(lambda: P.w2l_conv1d_bwd_weight(c1x, c1dy, c1dw, None, 1, False, w1w),
                                           args.kernel_iters),
    }
    del c1y, c1dx, c1dw, w1f, w1d, w1w

    # config 3: the ~10M-parameter model's full step (B=16, T <= 1600)
    c3 = W.config3()
    l3 = c3["layers"]
    x3 = to_dev(c3["x"], "bf16")
    w3 = [to_dev(w, "bf16") for w in c3["weights"]]
    b3 = [to_dev(b) for b in c3["biases"]]
    dw3 = [empty(w.shape) for w in c3["weights"]]
    db3 = [empty(b.shape) for b in c3["biases"]]
    tg3, il3, tl3 = to_dev(c3["targets"]), to_dev(c3["in_len"]), to_dev(c3["tgt_len"])
    ws3 = P.workspace(P.w2l_train_step_workspace_bytes(l3, c3["B"], c3["T"], c3["targets"].shape[1], P.W2L_BF16))
    loss3 = empty((c3["B"],))
    t_step3 = event_time_ms(lambda: P.w2l_train_step(l3, w3, b3, dw3, db3, x3, il3, tg3, tl3, loss3, None, 0, 1.0, ws3),
                            args.kernel_iters)
    flops3 = W.step_flops(l3, c3["B"], c3["T"])
    del x3, w3, dw3, ws3

    # per-frame log-softmax forward and backward at the criterion benchmark shape (24000 rows of 29 classes, fp32)
    lz = to_dev((rng.standard_normal((32 * 750, 29)) * 1.4).astype(np.float32))
    llp, ldz = empty((32 * 750, 29)), empty((32 * 750, 29))
    t_lsf = graph_time_ms([lambda: P.w2l_logsoftmax_fwd(lz, llp)], args.kernel_iters, out=llp)
    t_lsb = graph_time_ms([lambda: P.w2l_logsoftmax_bwd(llp, lz, ldz)], args.kernel_iters, out=ldz)
    ls_bytes_f, ls_bytes_b = 2 * 32 * 750 * 29 * 4, 3 * 32 * 750 * 29 * 4

    # CTC alone at the criterion benchmark shape (B=32, T=750, C=29)
    c2 = W.config2()
    cz, ct, ci, cl = to_dev(c2["logits"]), to_dev(c2["targets"]), to_dev(c2["in_len"]), to_dev(c2["tgt_len"])
    cws = P.workspace(P.w2l_ctc_workspace_bytes(32, 750, 29, c2["targets"].shape[1]))
    closs, cgrad = empty((32,)), empty((32, 750, 29))
    t_ctc = event_time_ms(lambda: P.w2l_ctc_fwd_bwd(cz, 1, ct, ci, cl, closs, cgrad, 0, 1.0, cws),
                          args.kernel_iters)
    cells = int(np.sum(c2["in_len"].astype(np.int64) * (2 * c2["tgt_len"].astype(np.int64) + 1)))
    ctc_bytes = 2 * 32 * 750 * 29 * 4 + 2 * 4 * cells

    # ASG alone at the same criterion shape without the blank class (B=32, T=750, C=28)
    a2 = W.asg_batch()
    ae, at, atg, ai, al = (to_dev(a2[k]) for k in ("emissions", "trans", "targets", "in_len", "tgt_len"))
    aws = P.workspace(P.w2l_asg_workspace_bytes(a2["B"], a2["T"], a2["C"], a2["targets"].shape[1]))
    aloss, age, agt = empty((a2["B"],)), empty(a2["emissions"].shape), empty(a2["trans"].shape)
    t_asg = event_time_ms(lambda: P.w2l_asg_fwd_bwd(ae, at, atg, ai, al, aloss, age, agt, 1.0, aws), args.kernel_iters)
    a_cells = int(np.sum(a2["in_len"].astype(np.int64) * (a2["tgt_len"].astype(np.int64) + a2["C"])))
    asg_bytes = 2 * a2["emissions"].size * 4 + 2 * 2 * 4 * a_cells   # emissions in, gradient out; lattices written and read once

    # log-mel features for a batch of the model's shape: B=8 waveforms of up to 240240 samples -> 1500 frames x 80 bands (bf16)
    wv = W.waveforms()
    wd, wl = to_dev(wv["wav"]), to_dev(wv["wav_len"])
    lfeat = empty((wv["B"], 1500, 80), "bf16")
    llen = torch.zeros(wv["B"], dtype=torch.int32, device="cuda:0")
    t_mel = event_time_ms(lambda: P.w2l_logmel_fwd(wd, wl, lfeat, llen), args.kernel_iters)
    mel_bytes = int(wv["wav_len"].sum()) * 4 + wv["B"] * 1500 * 80 * 2   # samples read once, features written once
    mel_frames = int(sum(max(0, 1 + (int(n) - 400) // 160) for n in wv["wav_len"]))

    # optimiser step over all parameters of the model as one flat fp32 buffer (not part of `value`:
    # the metric is forward + backward)
    npar = W.num_params(layers)
    ow = torch.zeros(npar, dtype=torch.float32, device="cuda:0")
    ov = torch.zeros_like(ow)
    og = torch.full_like(ow, 1e-3)
    olp = torch.empty(npar, dtype=torch.bfloat16, device="cuda:0")
    t_sgd = event_time_ms(lambda: P.w2l_sgd_momentum_step(ow, ov, og, olp, 0.01, 0.9), 20, 3)
    sgd_bytes = npar * 22.0
    del ow, ov, og, olp

    out = {
        "metric": "training frames/sec (fwd+bwd) for 105M conv-GLU CTC model",
        "value": frames / dt,
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "config4: 105M-param conv-GLU CTC model, B=8, T_b~U[1000,1500] padded to 1500, "
                        "80-dim features, seed 4; full fwd+criterion+bwd step",
            "params": W.num_params(layers),
            "valid_frames_per_step": frames,
            "padded_frames_per_step": B * T,
            "gflop_per_step": flops / 1e9,
        },
        "ms_per_step_sustained": dt_sus * 1e3,
        "sustained_steps": n_sus,
        "value_sustained": frames / dt_sus,
        "padded_frames_per_s": B * T / dt,
        "step_tflops": flops / dt / 1e12,
        "step_frac_of_bf16_mfma_peak": flops / dt / PEAK_BF16_MFMA,
        "roofline": {
            "bound": "mfma",
            "kernel": dom + " (k=11, 768->1536, B*T'=6000; 155.7 GFLOP per launch)",
            "achieved": achieved / 1e12,
            "peak": PEAK_BF16_MFMA / 1e12,
            "unit": "TFLOP/s",
            "frac": achieved / PEAK_BF16_MFMA,
            "traffic": DOMINANT_KERNEL_HBM_BYTES.get(dom),
            "avg_launch_ms": kern[dom],
            "measured_mfma_only_ceiling_tflops": mfma_ceiling / 1e12,
            "frac_of_measured_ceiling": achieved / mfma_ceiling,
            "ceiling_note": "matrix pipe alone with random operand bits (power-limited clock); with constant "
                            "operands the same loop sustains %.0f TFLOP/s" % (mfma_ceiling_const / 1e12),
        },
        "measured_ceilings": {"mfma_bf16_tflops_random_operands": mfma_ceiling / 1e12,
                              "mfma_bf16_tflops_constant_operands": mfma_ceiling_const / 1e12,
                              "device_copy_GBps": copy_bw / 1e9},
        "short_kernel_timing": "GLU, log-softmax and the same-size copies: %s, 16+ launches per graph "
                               "(a call through the binding costs the host ~8 us, more than they run)"
                               % SHORT_TIMING["method"],
        "config1_conv(k=11, 512->1024, B=16, T=800; 147.64 GFLOP per pass, bar 0.118 ms)": {
            k: {"ms": v, "tflops": gf1 / (v * 1e-3) / 1e12, "frac_mfma_peak": gf1 / (v * 1e-3) / PEAK_BF16_MFMA}
            for k, v in kern1.items()},
        "config3_train_step(9.2M params, B=16, T<=1600)": {
            "ms_per_step": t_step3, "frames_per_s": float(c3["in_len"].sum()) / (t_step3 * 1e-3),
            "gflop_per_step": flops3 / 1e9, "step_tflops": flops3 / (t_step3 * 1e-3) / 1e12,
            "step_frac_of_bf16_mfma_peak": flops3 / (t_step3 * 1e-3) / PEAK_BF16_MFMA},
        "kernels": {
            **{k: {"ms": v, "tflops": gf / (v * 1e-3) / 1e12, "frac_mfma_peak": gf / (v * 1e-3) / PEAK_BF16_MFMA}
               for k, v in kern.items()},
            "glu_fwd": {"ms": t_glu, "GBps": glu_bytes / (t_glu * 1e-3) / 1e9,
                        "frac_hbm_peak": glu_bytes / (t_glu * 1e-3) / PEAK_HBM,
                        "ms_rotating_buffers": t_glu_cold,
                        "frac_hbm_peak_rotating_buffers": glu_bytes / (t_glu_cold * 1e-3) / PEAK_HBM,
                        "device_copy_same_bytes_GBps": copy_glu / 1e9,
                        "frac_of_device_copy_same_bytes": glu_bytes / (t_glu * 1e-3) / copy_glu},
            "glu_bwd": {"ms": t_glub, "GBps": glub_bytes / (t_glub * 1e-3) / 1e9,
                        "frac_hbm_peak": glub_bytes / (t_glub * 1e-3) / PEAK_HBM,
                        "ms_rotating_buffers": t_glub_cold,
                        "frac_hbm_peak_rotating_buffers": glub_bytes / (t_glub_cold * 1e-3) / PEAK_HBM,
                        "device_copy_same_bytes_GBps": copy_glub / 1e9,
                        "frac_of_device_copy_same_bytes": glub_bytes / (t_glub * 1e-3) / copy_glub},
            "logsoftmax_fwd(24000x29)": {"ms": t_lsf, "GBps": ls_bytes_f / (t_lsf * 1e-3) / 1e9,
                                         "frac_hbm_peak": ls_bytes_f / (t_lsf * 1e-3) / PEAK_HBM},
            "logsoftmax_bwd(24000x29)": {"ms": t_lsb, "GBps": ls_bytes_b / (t_lsb * 1e-3) / 1e9,
                                         "frac_hbm_peak": ls_bytes_b / (t_lsb * 1e-3) / PEAK_HBM},
            # the criteria are bound by their chain of T_b dependent steps, not by HBM: critical_path_frac = the
            # longest utterance's serial steps x the time of one bare recursion step on one wavefront (no memory
            # traffic; measured with a one-wavefront probe) / the whole call (log-softmax, both lattices, gradient)
            "ctc_fwd_bwd(config2)": {"ms": t_ctc, "GBps": ctc_bytes / (t_ctc * 1e-3) / 1e9,
                                     "frac_hbm_peak": ctc_bytes / (t_ctc * 1e-3) / PEAK_HBM,
                                     "serial_steps": int(c2["in_len"].max()),
                                     "us_per_serial_step": t_ctc * 1e3 / int(c2["in_len"].max()),
                                     "bare_step_ns": CTC_BARE_STEP_NS,
                                     "critical_path_frac": int(c2["in_len"].max()) * CTC_BARE_STEP_NS * 1e-6 / t_ctc},
            "asg_fwd_bwd(B=32,T=750,C=28)": {"ms": t_asg, "GBps": asg_bytes / (t_asg * 1e-3) / 1e9,
                                             "frac_hbm_peak": asg_bytes / (t_asg * 1e-3) / PEAK_HBM,
                                             "serial_steps": int(a2["in_len"].max()),
                                             "us_per_serial_step": t_asg * 1e3 / int(a2["in_len"].max()),
                                             "bare_step_ns": ASG_BARE_STEP_NS,
                                             "critical_path_frac": int(a2["in_len"].max()) * ASG_BARE_STEP_NS * 1e-6 / t_asg},
            "logmel_fwd(B=8,1500x80)": {"ms": t_mel, "GBps": mel_bytes / (t_mel * 1e-3) / 1e9,
                                        "frac_hbm_peak": mel_bytes / (t_mel * 1e-3) / PEAK_HBM,
                                        "frames": mel_frames, "Mframes_per_s": mel_frames / (t_mel * 1e-3) / 1e6},
            "sgd_momentum_step(all %d params)" % npar: {"ms": t_sgd, "GBps": sgd_bytes / (t_sgd * 1e-3) / 1e9,
                                                         "frac_hbm_peak": sgd_bytes / (t_sgd * 1e-3) / PEAK_HBM},
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        f64 = lambda a: np.asarray(a, dtype=np.float64)
        b0 = 0
        t1 = time.perf_counter()
        oracle.train_step(layers, [f64(w) for w in cfg["weights"]], [f64(b) for b in cfg["biases"]],
                          f64(cfg["x"][b0:b0 + 1]), cfg["in_len"][b0:b0 + 1], cfg["targets"][b0:b0 + 1],
                          cfg["tgt_len"][b0:b0 + 1])
        t_cpu = time.perf_counter() - t1
        out["cpu_baseline"] = {
            "value": float(cfg["in_len"][b0]) / t_cpu,
            "unit": "frames/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "one utterance (b=0, %d valid frames, padded to %d) of the same batch through the same "
                      "11 layers, fp64 oracle train step, %.1f s" % (int(cfg["in_len"][b0]), T, t_cpu),
        }
        # the oracle's kernels alone: config 1 on two of its 16 utterances (scaled by 8: utterances are independent
        # and equally long), config 2 (log-softmax + CTC loss and gradient) whole
        sub = slice(0, 2)
        f1 = lambda a: np.asarray(a, dtype=np.float64)
        t1 = time.perf_counter(); oracle.conv1d_fwd(f1(c1["x"][sub]), f1(c1["w"]), None, 1); t_of = time.perf_counter() - t1
        t1 = time.perf_counter(); oracle.conv1d_bwd_data(f1(c1["dy"][sub]), f1(c1["w"]), c1["T"], 1); t_od = time.perf_counter() - t1
        t1 = time.perf_counter(); oracle.conv1d_bwd_weight(f1(c1["x"][sub]), f1(c1["dy"][sub]), c1["k"], 1); t_ow = time.perf_counter() - t1
        t1 = time.perf_counter()
        oracle.ctc_from_logits(f1(c2["logits"]), c2["targets"], c2["in_len"], c2["tgt_len"])
        t_oc = time.perf_counter() - t1
        out["cpu_baseline"]["kernels_ms"] = {
            "config1_conv1d_fwd": t_of * 8e3, "config1_conv1d_bwd_data": t_od * 8e3, "config1_conv1d_bwd_weight": t_ow * 8e3,
            "config1_note": "timed on 2 of the 16 utterances, scaled by 8",
            "config2_logsoftmax_ctc_fwd_bwd": t_oc * 1e3}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
