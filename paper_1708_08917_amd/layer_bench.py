"""Time one layer configuration through the C ABI (HIP events around back-to-back calls).

    python -m paper_1708_08917_amd.layer_bench --config cfg3 [--reps 100] [--backward]

Configurations: cfg1 (FC 1024x1024, k=16, batch 1), cfg2 (FC 4096x4096, k=64, batch 64),
cfg3 (9216->4096->4096 head, k=128, batch 256, both layers), cfg4 (3x3 CONV 256->256, 28x28,
batch 32, k=64; --backward adds dx, dw and the bias gradient), cfg5 (FC 16384x16384, k=256,
batch 1024; --backward adds dx and dw), head_b1 (the two head layers of cfg3 at batch 1),
head_chain_b1 (9216->4096->4096->1000 for one input, the three layers back to back), general
(block sizes that are not powers of two).
Prints one line per layer with the time per call and the algorithmic bytes/flops rates.
This is the companion of bench.py for the workloads that bench.py does not time; it is also
the program that the rocprofv3 summaries under profiles/ were collected with.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as B
from . import synth

DEV = "cuda:0"


def _time(fn, reps, warm):
    """Microseconds per call: `reps` calls captured in one HIP graph (so that the host-side
    cost of the Python binding is not in the figure), replayed between two events; the median of
    five such replays."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(reps):
                fn()
        graph.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            graph.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / reps)
    return sorted(ts)[len(ts) // 2]


def fc_work(cfg):
    F = cfg.k // 2 + 1
    lg = cfg.k.bit_length() - 1
    byts = 8 * cfg.p * cfg.q * F + 4 * cfg.batch * (cfg.n_in + cfg.n_out) + (4 * cfg.n_out if cfg.bias else 0)
    flops = 8 * cfg.p * cfg.q * (cfg.k // 2) * cfg.batch + (cfg.p + cfg.q) * cfg.batch * 5 * cfg.k * lg // 2
    return byts, flops


def bench_fc(cfg, reps, backward=False):
    w, x, b = synth.fc_inputs(cfg)
    wd, xd = torch.from_numpy(w).to(DEV), torch.from_numpy(x).to(DEV)
    bd = None if b is None else torch.from_numpy(b).to(DEV)
    wh = B.circ_precompute_spectra(wd)
    y = torch.empty(cfg.batch, cfg.n_out, device=DEV)
    ws = torch.empty(max(1, B.circ_fc_workspace_bytes(cfg.p, cfg.q, cfg.k, cfg.batch, True)), dtype=torch.uint8, device=DEV)
    epi = (B.EPI_BIAS if b is not None else 0) | (B.EPI_RELU if cfg.relu else 0)
    t = _time(lambda: B.circ_fc_forward(wh, xd, bd, y, cfg.p, cfg.q, cfg.k, epi, ws), reps, max(3, reps // 10))
    byts, flops = fc_work(cfg)
    print(f"{cfg.name}: forward {t:9.2f} us/call  {cfg.batch / t * 1e6:12.0f} vectors/s  alg {byts / t * 1e-3:7.1f} GB/s "
          f"{flops / t * 1e-6:6.2f} TFLOP/s  dense-equivalent {2.0 * cfg.n_in * cfg.n_out * cfg.batch / t * 1e-6:7.1f} TFLOP/s", flush=True)
    tp = _time(lambda: B.circ_precompute_spectra(wd, wh), 20, 3)
    print(f"{cfg.name}: precompute_spectra {tp:9.2f} us/call", flush=True)
    if cfg.k >= 8 and cfg.k & (cfg.k - 1) == 0:
        # the same layer with fp16 storage (activations, spectra) and fp32 arithmetic
        wh16 = B.circ_precompute_spectra_f16(wd)
        x16, y16 = xd.half(), torch.empty(cfg.batch, cfg.n_out, dtype=torch.float16, device=DEV)
        ws16 = torch.empty(max(1, B.circ_fc_workspace_bytes_f16(cfg.p, cfg.q, cfg.k, cfg.batch)), dtype=torch.uint8, device=DEV)
        th = _time(lambda: B.circ_fc_forward_f16(wh16, x16, bd, y16, cfg.p, cfg.q, cfg.k, epi, ws16), reps, max(3, reps // 10))
        print(f"{cfg.name}: forward, fp16 storage {th:9.2f} us/call  {cfg.batch / th * 1e6:12.0f} vectors/s  "
              f"alg {byts / 2 / th * 1e-3:7.1f} GB/s", flush=True)
    if backward:
        dy = torch.from_numpy(synth.fc_upstream_grad(cfg)).to(DEV)
        dx, dw = torch.empty_like(xd), torch.empty_like(wd)
        r = max(5, reps // 4)
        tb = _time(lambda: B.circ_fc_backward(wh, xd, dy, cfg.p, cfg.q, cfg.k, True, True, dx, dw, ws), r, 3)
        tdx = _time(lambda: B.circ_fc_backward(wh, xd, dy, cfg.p, cfg.q, cfg.k, True, False, dx, None, ws), r, 3)
        tdw = _time(lambda: B.circ_fc_backward(wh, xd, dy, cfg.p, cfg.q, cfg.k, False, True, None, dw, ws), r, 3)
        db = torch.empty(cfg.n_out, device=DEV)
        tdb = _time(lambda: B.circ_bias_grad(dy, db), r, 3)
        print(f"{cfg.name}: backward {tb:9.2f} us/call (dx only {tdx:.2f}, dw only {tdw:.2f}; bias gradient {tdb:.2f})  dense-equivalent "
              f"{4.0 * cfg.n_in * cfg.n_out * cfg.batch / tb * 1e-6:7.1f} TFLOP/s", flush=True)
        # dx + step on the cached spectra (lr = 0 keeps the weights as they are over the repetitions),
        # against dx + dw + precompute of the new weights
        tsg = _time(lambda: B.circ_fc_sgd_step(wh, xd, dy, 0.0, cfg.p, cfg.q, cfg.k, True, dx, ws), r, 3)
        print(f"{cfg.name}: sgd step {tsg:9.2f} us/call (backward + precompute: {tb + tp:.2f})", flush=True)
        if cfg.k >= 8 and cfg.k & (cfg.k - 1) == 0:
            dy16, dx16 = dy.half(), torch.empty_like(x16)
            wsb = torch.empty(max(1, B.circ_fc_backward_workspace_bytes_f16(cfg.p, cfg.q, cfg.k, cfg.batch)), dtype=torch.uint8, device=DEV)
            tbh = _time(lambda: B.circ_fc_backward_f16(wh16, x16, dy16, cfg.p, cfg.q, cfg.k, True, True, dx16, dw, wsb), r, 3)
            tdxh = _time(lambda: B.circ_fc_backward_f16(wh16, x16, dy16, cfg.p, cfg.q, cfg.k, True, False, dx16, None, wsb), r, 3)
            tdwh = _time(lambda: B.circ_fc_backward_f16(wh16, x16, dy16, cfg.p, cfg.q, cfg.k, False, True, None, dw, wsb), r, 3)
            print(f"{cfg.name}: backward, fp16 storage {tbh:9.2f} us/call (dx only {tdxh:.2f}, dw only {tdwh:.2f})", flush=True)


def bench_chain(cfgs, reps):
    """A stack of FC layers applied to the same batch through circ_chain_forward: time per
    pass over the whole stack (the per-image latency of a classifier head at batch 1)."""
    layers = []
    act = None
    for c in cfgs:
        w, x, b = synth.fc_inputs(c)
        if act is None:
            act = torch.from_numpy(x).to(DEV)
        wh = B.circ_precompute_spectra(torch.from_numpy(w).to(DEV))
        bd = None if b is None else torch.from_numpy(b).to(DEV)
        y = torch.empty(c.batch, c.n_out, device=DEV)
        ws = torch.empty(max(1, B.circ_fc_workspace_bytes(c.p, c.q, c.k, c.batch)), dtype=torch.uint8, device=DEV)
        epi = (B.EPI_BIAS if b is not None else 0) | (B.EPI_RELU if c.relu else 0)
        layers.append((wh, act, bd, y, c, epi, ws))
        act = y

    # one call of the chain entry point (the layers back to back on one stream, activations in its workspace)
    descs = [B.fc_layer(wh, bd, c.p, c.q, c.k, epi) for wh, xin, bd, y, c, epi, ws in layers]
    cws = torch.empty(B.circ_chain_workspace_bytes(descs, cfgs[0].batch), dtype=torch.uint8, device=DEV)
    x0, ylast = layers[0][1], layers[-1][3]

    def run():
        B.circ_chain_forward(descs, x0, ylast, cws)

    t = _time(run, reps, max(3, reps // 10))
    names = " -> ".join([str(cfgs[0].n_in)] + [f"{c.n_out} (k={c.k})" for c in cfgs])
    print(f"chain {names}, batch {cfgs[0].batch}: {t:9.2f} us/pass  {cfgs[0].batch / t * 1e6:10.0f} inputs/s  "
          f"{len(cfgs) / t * 1e6:10.0f} layers/s", flush=True)
    if all(c.k >= 8 and c.k & (c.k - 1) == 0 for c in cfgs):
        # the same stack with fp16 storage of activations and weight spectra
        layers16 = []
        for (wh, xin, bd, y, c, epi, ws), cfg in zip(layers, cfgs):
            w, _, _ = synth.fc_inputs(cfg)
            wh16 = B.circ_precompute_spectra_f16(torch.from_numpy(w).to(DEV))
            ws16 = torch.empty(max(1, B.circ_fc_workspace_bytes_f16(c.p, c.q, c.k, c.batch)), dtype=torch.uint8, device=DEV)
            layers16.append((wh16, xin.half(), bd, y.half(), c, epi, ws16))
        for i in range(1, len(layers16)):   # each layer reads the previous one's output buffer
            l = layers16[i]
            layers16[i] = (l[0], layers16[i - 1][3], l[2], l[3], l[4], l[5], l[6])

        def run16():
            for wh16, xin, bd, y, c, epi, ws16 in layers16:
                B.circ_fc_forward_f16(wh16, xin, bd, y, c.p, c.q, c.k, epi, ws16)

        t16 = _time(run16, reps, max(3, reps // 10))
        print(f"chain {names}, batch {cfgs[0].batch}, fp16 storage: {t16:9.2f} us/pass  {len(cfgs) / t16 * 1e6:10.0f} layers/s", flush=True)


def bench_conv(cfg, reps, backward=False):
    w, x = synth.conv_inputs(cfg)
    wd, xd = torch.from_numpy(w).to(DEV), torch.from_numpy(x).to(DEV)
    wh = B.circ_precompute_spectra(wd)
    y = torch.empty(cfg.N, cfg.C_out, cfg.H, cfg.W, device=DEV)
    nws = B.circ_conv_workspace_bytes(cfg.N, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.r, 1, cfg.pad, cfg.k)
    ws = torch.empty(nws, dtype=torch.uint8, device=DEV)
    t = _time(lambda: B.circ_conv_forward(wh, xd, None, y, cfg.C_out, cfg.r, 1, cfg.pad, cfg.k, 0, ws), reps, max(3, reps // 10))
    byts = 2 * x.nbytes + w.nbytes
    dense = 2.0 * cfg.N * cfg.H * cfg.W * cfg.r * cfg.r * cfg.C_in * cfg.C_out
    print(f"{cfg.name}: forward {t:9.2f} us/call  {cfg.N / t * 1e6:10.0f} images/s  alg {byts / t * 1e-3:7.1f} GB/s  "
          f"dense-equivalent {dense / t * 1e-6:7.1f} TFLOP/s", flush=True)
    if cfg.k >= 8 and cfg.k & (cfg.k - 1) == 0:
        x16, y16 = xd.half(), torch.empty(cfg.N, cfg.C_out, cfg.H, cfg.W, dtype=torch.float16, device=DEV)
        th = _time(lambda: B.circ_conv_forward_f16(wh, x16, None, y16, cfg.C_out, cfg.r, 1, cfg.pad, cfg.k, 0, ws), reps, max(3, reps // 10))
        print(f"{cfg.name}: forward, fp16 activations {th:9.2f} us/call  {cfg.N / th * 1e6:10.0f} images/s", flush=True)
    if backward:
        dy = torch.from_numpy(synth.conv_upstream_grad(cfg)).to(DEV)
        dx, dw, db = torch.empty_like(xd), torch.empty_like(wd), torch.empty(cfg.C_out, device=DEV)
        nwb = B.circ_conv_backward_workspace_bytes(cfg.N, cfg.C_in, cfg.C_out, cfg.H, cfg.W, cfg.r, 1, cfg.pad, cfg.k)
        wsb = torch.empty(nwb, dtype=torch.uint8, device=DEV)
        args = (wh, xd, dy, cfg.C_in, cfg.H, cfg.W, cfg.r, 1, cfg.pad, cfg.k)
        r = max(5, reps // 4)
        tb = _time(lambda: B.circ_conv_backward(*args, True, True, dx, dw, wsb), r, 3)
        tdx = _time(lambda: B.circ_conv_backward(*args, True, False, dx, None, wsb), r, 3)
        tdw = _time(lambda: B.circ_conv_backward(*args, False, True, None, dw, wsb), r, 3)
        tdb = _time(lambda: B.circ_bias_grad(dy, db), r, 3)
        print(f"{cfg.name}: backward {tb:9.2f} us/call (dx only {tdx:.2f}, dw only {tdw:.2f}; bias gradient {tdb:.2f})  "
              f"dense-equivalent {2.0 * dense / tb * 1e-6:7.1f} TFLOP/s", flush=True)
        tp = _time(lambda: B.circ_precompute_spectra(wd, wh), 20, 3)
        tsg = _time(lambda: B.circ_conv_sgd_step(wh, xd, dy, 0.0, cfg.C_in, cfg.H, cfg.W, cfg.r, 1, cfg.pad, cfg.k, True, dx,
                                                 wsb), r, 3)
        print(f"{cfg.name}: sgd step {tsg:9.2f} us/call (backward + precompute: {tb + tp:.2f})", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="all", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "head_b1", "head_chain_b1", "general", "all"])
    ap.add_argument("--reps", type=int, default=100)
    ap.add_argument("--backward", action="store_true")
    a = ap.parse_args()
    sel = lambda n: a.config in (n, "all")
    if sel("cfg1"):
        bench_fc(synth.CFG1, a.reps)
    if sel("cfg2"):
        bench_fc(synth.CFG2, a.reps)
    if sel("cfg3"):
        bench_fc(synth.CFG3_L1, a.reps)
        bench_fc(synth.CFG3_L2, a.reps)
    if sel("cfg4"):
        bench_conv(synth.CFG4, a.reps, backward=a.backward or a.config == "all")
    if sel("head_b1"):
        # the two head layers at batch 1 (single-image inference, the regime of the paper's
        # layers-per-second figures): time per layer = 1 / (layers per second)
        import dataclasses
        bench_fc(dataclasses.replace(synth.CFG3_L1, name="head_fc9216x4096_k128_b1", batch=1), a.reps)
        bench_fc(dataclasses.replace(synth.CFG3_L2, name="head_fc4096x4096_k128_b1", batch=1), a.reps)
    if sel("head_chain_b1"):
        # a whole classifier head for one input: 9216 -> 4096 -> 4096 -> 1000 (1000 = 125 blocks of 8)
        import dataclasses
        bench_chain([dataclasses.replace(synth.CFG3_L1, batch=1), dataclasses.replace(synth.CFG3_L2, batch=1),
                     synth.FcConfig("head_fc4096x1000_k8_b1", 4096, 1000, 8, 1, bias=True, relu=False, index=7)], a.reps)
    if sel("general"):
        # block sizes that are not powers of two (mixed-radix transforms): an FC layer with blocks of 100
        # and the 384-channel 13 x 13 CONV layer of an AlexNet-style network as 4 x 4 blocks of 96
        bench_fc(synth.FcConfig("fc4000_k100_b64", 4000, 4000, 100, 64, bias=True, relu=True, index=5), a.reps,
                 backward=a.backward)
        bench_conv(synth.ConvConfig("conv3x3_c384_13x13_k96_n32", 32, 384, 384, 13, 13, 3, 1, 1, 96, index=6), a.reps,
                   backward=a.backward)
        # the same layer as 6 x 6 blocks of 64 (fused kernel; rows of 13 pixels: element-wise loads), at two batch sizes
        bench_conv(synth.ConvConfig("conv3x3_c384_13x13_k64_n32", 32, 384, 384, 13, 13, 3, 1, 1, 64, index=8), a.reps,
                   backward=a.backward)
        bench_conv(synth.ConvConfig("conv3x3_c384_13x13_k64_n128", 128, 384, 384, 13, 13, 3, 1, 1, 64, index=9), a.reps,
                   backward=a.backward)
    if sel("cfg5"):
        bench_fc(synth.CFG5, max(10, a.reps // 4), backward=a.backward or a.config == "all")


if __name__ == "__main__":
    main()
