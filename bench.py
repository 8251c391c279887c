#!/usr/bin/env python3
"""Benchmark of the INT8 conv backward hot path on one MI355X.

One step = Algorithm 1 for one layer: daq_quantize_grad (statistics, discriminator, clip values,
per-channel and global int8 copies of dY) + daq_conv_bwd_filter_int8 + daq_conv_bwd_data_int8.
Inputs (fp32 dY, the saved int8 activation/filter of the forward pass, the clip state) are resident
in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--layer 0] [--rotate R]
    python bench.py --sweep --config 4     # every layer of a network, one line with per-layer times
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, GB/s

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by a copy
# kernel of known size; keyed by (workload, kernel).  See profiles/ for the runs these come from.
MEASURED_TRAFFIC = {
    ("config2", "conv_bwd_data_mfma"): 45.23e6,    # with the filter gradient's last stage on the same launch (35.6e6 alone)
    ("config2", "conv_bwd_filter_mfma"): 23.61e6,
    ("config2", "stats"): 25.78e6,
    ("config2", "count_qg"): 34.01e6,
    ("config2", "pack_vq"): 32.89e6,
}


def quantizer_for(scheme: str, dy_bf16: bool = False):
    """(callable, entry point name): daq_quantize_grad, or daq_quantize_grad_scheme bound to an ablation variant."""
    from paper_2102_04782_amd import binding as daq

    code = {"daq": daq.SCHEME_DAQ, "gq": daq.SCHEME_GQ, "gvq": daq.SCHEME_GVQ, "mcs": daq.SCHEME_MCS}[scheme]
    if dy_bf16:
        def quantize16(d, dY, st, **kw):
            return daq.quantize_grad_bf16(d, dY, st, code, **kw)

        return quantize16, f"daq_quantize_grad_bf16({scheme})"
    if scheme == "daq":
        return daq.quantize_grad, "daq_quantize_grad"

    def quantize(d, dY, st, **kw):
        return daq.quantize_grad_scheme(d, dY, st, code, **kw)

    return quantize, f"daq_quantize_grad_scheme({scheme})"


def sweep_forward(args, dev) -> int:
    """The forward entry point (daq_conv_fwd_int8: max of X and W, both layouts of q(X), packed q(W), Y) over every conv
    layer of a config, distinct shapes timed once.  Not the benchmark's metric: it produces the operands the backward
    step starts from; reported so that the figures in the design notes can be reproduced."""
    import torch

    from paper_2102_04782_amd import binding as daq
    from paper_2102_04782_amd import workloads as wl

    layers = wl.config_layers(args.config)
    steps = max(3, min(args.steps, 20))
    seen, rows_out = {}, []
    tot = {"conv": 0.0, "quantize_x": 0.0, "quantize_w": 0.0}
    for li, L in enumerate(layers):
        key = L.desc_fields()
        if key not in seen:
            d = daq.ConvDesc.make(*key)
            gen = torch.Generator(device=dev)
            gen.manual_seed(wl.seed_for(args.config, li))
            X = torch.randn(d.x_shape, device=dev, generator=gen)
            W = torch.randn(d.w_shape, device=dev, generator=gen)
            out = daq.alloc_fwd(d, dev)
            for _ in range(3):
                daq.conv_fwd_int8(d, X, W, out=out)
            torch.cuda.synchronize()
            daq.prof_begin()
            for _ in range(steps):
                daq.conv_fwd_int8(d, X, W, out=out)
            rows = daq.prof_end()
            ev = rows.pop("(empty event pair)", (0.0, 1))
            ev_us = 1e3 * ev[0] / ev[1]
            # per step: a name launched twice (fill, absmax, scale run for X and for W) counts twice
            t = {k: (1e3 * v[0] / v[1] - ev_us) * (v[1] / steps) for k, v in rows.items()}
            conv = sum(v for k, v in t.items() if k.startswith("conv"))
            qw = t.get("pack_w", 0.0)
            seen[key] = (conv, sum(t.values()) - conv - qw, qw)
            del X, W, out
        conv, qx, qw = seen[key]
        tot["conv"] += conv
        tot["quantize_x"] += qx
        tot["quantize_w"] += qw
        rows_out.append({"layer": L.name, "conv_us": round(conv, 1), "quantize_us": round(qx + qw, 1)})
    total = sum(tot.values())
    print(json.dumps({"metric": "forward entry point, kernel time (HIP events)", "value": round(1e-3 * total, 4), "unit": "ms",
                      "higher_is_better": False, "n_gpus": 1, "data": "synthetic", "dtype": "int8",
                      "config": {"workload": f"config{args.config}: all {len(layers)} conv layers, {len(seen)} distinct shapes, "
                                             f"N={layers[0].N}, daq_conv_fwd_int8 once each"},
                      "kernel_us_total": {k: round(v, 1) for k, v in tot.items()}, "layers": rows_out}))
    return 0


def sweep(args, dev) -> int:
    """Whole-network pass: the backward step of every conv layer of a config, back to back per shape.

    Inputs are generated on the GPU (random codes for the saved int8 tensors, Gaussian dY); parity of
    these shapes is the business of the tests, this only measures."""
    import torch

    from paper_2102_04782_amd import binding as daq
    from paper_2102_04782_amd import workloads as wl

    layers = wl.config_layers(args.config)
    quantize, _ = quantizer_for(args.scheme, args.dy_bf16)
    steps = max(3, min(args.steps, 20))
    seen, out_layers = {}, []
    tot_wall = tot_ops = 0.0
    tot = {"quantize": 0.0, "dW": 0.0, "dX": 0.0}
    for li, L in enumerate(layers):
        key = L.desc_fields()
        if key not in seen:
            d = daq.ConvDesc.make(*key)
            gen = torch.Generator(device=dev)
            gen.manual_seed(wl.seed_for(args.config, li))
            dY = torch.randn(d.y_shape, device=dev, generator=gen) * 1e-2
            if args.dy_bf16:
                dY = dY.to(torch.bfloat16)
            st = torch.zeros(d.Cout, device=dev)
            qx = torch.randint(-127, 128, (daq.layout_qx_cnhw(d).bytes,), dtype=torch.int8, device=dev, generator=gen)
            qw = torch.randint(-127, 128, (daq.layout_qw(d).bytes,), dtype=torch.int8, device=dev, generator=gen)
            one = torch.ones(1, device=dev)
            out = daq.alloc_quantize_grad(d, dev, want_stats=False)
            dW = torch.empty(d.w_shape, device=dev)
            dX = torch.empty(d.x_shape, device=dev)
            ws_f = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_FILTER, d)), dtype=torch.uint8, device=dev)
            ws_d = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_DATA, d)), dtype=torch.uint8, device=dev)
            ws_b = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD, d)), dtype=torch.uint8, device=dev)
            dXh, bf16_ok = None, False
            if args.dx_bf16:
                dXh = torch.empty(d.x_shape, dtype=torch.bfloat16, device=dev)
                try:   # layers without a kernel for the narrow result keep fp32
                    daq.conv_bwd_data_int8_bf16(d, out.qg, one, qw, one, dX=dXh, workspace=ws_d)
                    bf16_ok = True
                except daq.DaqError:
                    pass

            def step():
                q = quantize(d, dY, st, out=out)
                if args.dx_bf16 and bf16_ok:
                    daq.conv_bwd_filter_int8(d, qx, one, q.vq, q.s_chan, dW=dW, workspace=ws_f)
                    daq.conv_bwd_data_int8_bf16(d, q.qg, q.s_global, qw, one, dX=dXh, workspace=ws_d)
                elif args.separate:
                    daq.conv_bwd_filter_int8(d, qx, one, q.vq, q.s_chan, dW=dW, workspace=ws_f)
                    daq.conv_bwd_data_int8(d, q.qg, q.s_global, qw, one, dX=dX, workspace=ws_d)
                else:
                    daq.conv_bwd_int8(d, qx, one, q.vq, q.s_chan, q.qg, q.s_global, qw, one, dW=dW, dX=dX, workspace=ws_b)

            for _ in range(3):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            wall_us = 1e6 * (time.perf_counter() - t0) / steps
            daq.prof_begin()
            for _ in range(steps):
                step()
            rows = daq.prof_end()
            ev = rows.pop("(empty event pair)", (0.0, 1))
            ev_us = 1e3 * ev[0] / ev[1]
            t = {k: 1e3 * v[0] / v[1] - ev_us for k, v in rows.items()}
            seen[key] = (wall_us,
                         sum(v for k, v in t.items() if k in ("stats", "count_qg", "pack_vq", "pack_qg")),
                         sum(v for k, v in t.items() if k.startswith("conv_bwd_filter") or k == "dw_reduce"),
                         sum(v for k, v in t.items() if k.startswith("conv_bwd_data")))
            del dY, qx, qw, out, dW, dX, ws_f, ws_d, ws_b
        wall_us, q_us, dw_us, dx_us = seen[key]
        tot_wall += wall_us
        tot_ops += 4.0 * L.macs
        tot["quantize"] += q_us
        tot["dW"] += dw_us
        tot["dX"] += dx_us
        out_layers.append({"layer": L.name, "shape": f"N{L.N} {L.Cin}->{L.Cout} {L.Hin}x{L.Win} k{L.kH} s{L.stride} g{L.groups}",
                           "step_us": round(wall_us, 1), "quantize_us": round(q_us, 1), "dW_us": round(dw_us, 1),
                           "dX_us": round(dx_us, 1), "GOP": round(4e-9 * L.macs, 2)})
    value = tot_ops / (tot_wall * 1e-6) / 1e12
    print(json.dumps({
        "metric": "INT8 conv-backward TOPS incl. grad quantization", "value": round(value, 3), "unit": "TOP/s",
        "n_gpus": 1, "steps": steps, "warmup": 3, "ms_per_step": round(1e-3 * tot_wall, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config{args.config}: all {len(layers)} conv layers, {len(seen)} distinct shapes, "
                               f"N={layers[0].N}, one backward step each"},
        "frac_int8_mfma_peak": round(value / PEAK_INT8_TOPS, 5),
        "kernel_us_total": {k: round(v, 1) for k, v in tot.items()},
        "layers": out_layers}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--rotate", type=int, default=1, help="number of dY buffer sets cycled through (cold-cache runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=1, choices=(1, 2),
                    help="2: the two convolutions, which are independent once dY is quantized, run on two streams "
                         "(measured slower than one stream on this workload: the event waits cost more than the overlap gains)")
    ap.add_argument("--separate", action="store_true",
                    help="call daq_conv_bwd_filter_int8 and daq_conv_bwd_data_int8 one after the other instead of "
                         "daq_conv_bwd_int8 (both gradients in one call, one launch fewer)")
    ap.add_argument("--dx-bf16", action="store_true",
                    help="store the data gradient as bfloat16 (daq_conv_bwd_data_int8_bf16: an option beside the method, "
                         "which returns fp32 gradients; reported for comparison, never the default)")
    ap.add_argument("--scheme", default="daq", choices=("daq", "gq", "gvq", "mcs"),
                    help="rule for the per-channel clip values: Algorithm 1 (default) or one of the ablation study's "
                         "variants through daq_quantize_grad_scheme (global baseline, per-channel maximum, layer-wise clipping)")
    ap.add_argument("--dy-bf16", action="store_true",
                    help="hand the output gradient over as bfloat16 (daq_quantize_grad_bf16: same algorithm on the widened "
                         "values, 2 instead of 4 bytes read per element and sweep; reported for comparison, never the default)")
    ap.add_argument("--graph", type=int, default=0, choices=(0, 1),
                    help="1: capture one step into a HIP graph and time replays of it")
    ap.add_argument("--sweep", action="store_true",
                    help="time the step of every layer of --config (distinct shapes once) and report the network total")
    ap.add_argument("--forward", action="store_true",
                    help="with --sweep: time the forward entry point (daq_conv_fwd_int8) of every layer instead of the backward step")
    ap.add_argument("--copy-calib-mib", type=int, default=0,
                    help="after the timed region, run 5 device-to-device copies of this many MiB: the plain copy "
                         "kernel of known size that scales rocprofv3's FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2102_04782_amd import binding as daq
    from paper_2102_04782_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    daq.lib()  # fail loudly if the HIP library is missing
    if args.sweep:
        return sweep_forward(args, dev) if args.forward else sweep(args, dev)
    quantize, quantize_name = quantizer_for(args.scheme, args.dy_bf16)

    layer, X, W, dY, st = wl.make_inputs(args.config, args.layer)
    d = daq.ConvDesc.make(*layer.desc_fields())
    X_d, W_d = torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev)
    fwd = daq.conv_fwd_int8(d, X_d, W_d)            # produces the saved q(X), q(W), s_X, s_W
    del X_d
    R = max(1, args.rotate)
    dYs = [torch.from_numpy(dY).to(dev)] + [torch.from_numpy(dY).to(dev).clone() for _ in range(R - 1)]
    if args.dy_bf16:
        dYs = [g.to(torch.bfloat16) for g in dYs]
        dY = dYs[0].float().cpu().numpy()   # what the oracle of the cpu_baseline leg sees: the widened values
    states = [torch.from_numpy(st.copy()).to(dev) for _ in range(R)]
    outs = [daq.alloc_quantize_grad(d, dev, want_stats=False) for _ in range(R)]
    dWs = [torch.empty(d.w_shape, dtype=torch.float32, device=dev) for _ in range(R)]
    dXs = [torch.empty(d.x_shape, dtype=torch.float32, device=dev) for _ in range(R)]
    ws_f = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_FILTER, d)), dtype=torch.uint8, device=dev)
    ws_d = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_DATA, d)), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD, d)), dtype=torch.uint8, device=dev)
    combined = not args.separate and args.streams == 1 and not args.dx_bf16
    dXh = torch.empty(d.x_shape, dtype=torch.bfloat16, device=dev) if args.dx_bf16 else None
    main_s = torch.cuda.Stream()
    side_s = torch.cuda.Stream() if args.streams == 2 else None

    def step(i: int, fork: bool = True):
        # Algorithm 1 for one layer.  dW needs the per-channel copy, dX the global copy: after the quantizer
        # the two convolutions share no data.  fork=False is the plain reference schedule: the three entry points
        # one after the other on one stream.
        r = i % R
        q = quantize(d, dYs[r], states[r], out=outs[r], stream=main_s)
        if combined and fork:
            daq.conv_bwd_int8(d, fwd.qx_cnhw, fwd.s_x, q.vq, q.s_chan, q.qg, q.s_global, fwd.qw, fwd.s_w,
                              dW=dWs[r], dX=dXs[r], workspace=ws_b, stream=main_s)
        elif args.dx_bf16 and fork:
            daq.conv_bwd_filter_int8(d, fwd.qx_cnhw, fwd.s_x, q.vq, q.s_chan, dW=dWs[r], workspace=ws_f, stream=main_s)
            daq.conv_bwd_data_int8_bf16(d, q.qg, q.s_global, fwd.qw, fwd.s_w, dX=dXh, workspace=ws_d, stream=main_s)
        elif side_s is not None and fork:
            side_s.wait_stream(main_s)
            daq.conv_bwd_data_int8(d, q.qg, q.s_global, fwd.qw, fwd.s_w, dX=dXs[r], workspace=ws_d, stream=side_s)
            daq.conv_bwd_filter_int8(d, fwd.qx_cnhw, fwd.s_x, q.vq, q.s_chan, dW=dWs[r], workspace=ws_f, stream=main_s)
            main_s.wait_stream(side_s)
        else:
            daq.conv_bwd_filter_int8(d, fwd.qx_cnhw, fwd.s_x, q.vq, q.s_chan, dW=dWs[r], workspace=ws_f, stream=main_s)
            daq.conv_bwd_data_int8(d, q.qg, q.s_global, fwd.qw, fwd.s_w, dX=dXs[r], workspace=ws_d, stream=main_s)

    torch.cuda.synchronize()
    graphs = None
    if args.graph:
        # one captured step per buffer set; every replay is checked against the eager result below
        with torch.cuda.stream(main_s):
            step(0)
        torch.cuda.synchronize()
        graphs = []
        for r in range(R):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph, stream=main_s):
                step(r)
            graphs.append(gph)
        torch.cuda.synchronize()

    def run(i: int):
        if graphs is not None:
            graphs[i % R].replay()
        else:
            step(i)

    for i in range(args.warmup):
        run(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / args.steps

    # the schedule under test must reproduce the plain single-stream result bit for bit (state: same input each time)
    chk_state = torch.from_numpy(st.copy()).to(dev)
    states[0].copy_(chk_state)
    torch.cuda.synchronize()
    run(0)
    torch.cuda.synchronize()
    got = (dWs[0].clone(), dXs[0].clone() if dXh is None else dXh.clone(), outs[0].vq.clone(), outs[0].qg.clone())
    states[0].copy_(chk_state)
    torch.cuda.synchronize()
    step(0, fork=False)
    torch.cuda.synchronize()
    want_dX = dXs[0] if dXh is None else dXs[0].to(torch.bfloat16)   # torch rounds to nearest even too
    same = all(torch.equal(a, b) for a, b in zip(got, (dWs[0], want_dX, outs[0].vq, outs[0].qg)))
    if not same:
        print("bench.py: the timed schedule does not reproduce the single-stream result", file=sys.stderr)
        return 3

    # per-kernel durations: K steps of the timed schedule on one stream with a HIP event pair around every launch
    daq.prof_begin()
    for i in range(args.steps):
        step(i, fork=combined or args.dx_bf16)
    rows = daq.prof_end()
    torch.cuda.synchronize()

    if args.copy_calib_mib > 0:
        ca = torch.zeros(args.copy_calib_mib << 20, dtype=torch.uint8, device=dev)
        cb = torch.empty_like(ca)
        for _ in range(5):
            cb.copy_(ca)
        torch.cuda.synchronize()
        del ca, cb

    E_Y = int(np.prod(d.y_shape))
    eb_y = 2.0 if args.dy_bf16 else 4.0   # bytes read per element of dY and sweep
    E_X = int(np.prod(d.x_shape))
    E_W = int(np.prod(d.w_shape))
    ops_per_conv = 2.0 * layer.macs
    ops_per_step = 2.0 * ops_per_conv          # dX + dW
    # algorithmic bytes / ops of one launch of each kernel
    alg_bytes = {
        "stats": eb_y * E_Y,
        "count_qg": (eb_y + 1.0) * E_Y if daq.layout_qg(d).kind == daq.LAYOUT_NHWC else eb_y * E_Y,
        "pack_vq": (eb_y + 1.0) * E_Y,
        "pack_qg": (eb_y + 1.0) * E_Y,
    }
    # convolutions: int8 operands read once, fp32 result written once
    conv_bytes = {"conv_bwd_data": E_Y + E_W + (2.0 if args.dx_bf16 else 4.0) * E_X, "conv_bwd_filter": E_X + E_Y + 4.0 * E_W}
    ridge = PEAK_INT8_TOPS * 1e12 / (PEAK_HBM_GBS * 1e9)   # ops per byte above which the MFMA peak binds
    kernels = {}
    # what an event pair adds by itself (measured by the library with empty pairs), removed from every span
    ev_ms, ev_n = rows.pop("(empty event pair)", (0.0, 0))
    ev_us = 1e3 * ev_ms / ev_n if ev_n else 0.0
    for name, (total_ms, launches) in list(rows.items()):
        rows[name] = (max(total_ms - 1e-3 * ev_us * launches, 1e-6), launches)
    for name, (total_ms, launches) in rows.items():
        avg_us = 1e3 * total_ms / max(launches, 1)
        per_step = launches / args.steps
        entry = {"avg_us": round(avg_us, 3), "launches_per_step": per_step}
        if name in alg_bytes:
            entry["GBps"] = round(alg_bytes[name] / (avg_us * 1e-6) / 1e9, 1)
        if name.startswith("conv_bwd"):
            entry["TOPs"] = round(ops_per_conv / (avg_us * 1e-6) / 1e12, 2)
        kernels[name] = entry
    dom = max(rows.items(), key=lambda kv: kv[1][0])[0] if rows else None
    roofline = None
    if dom is not None:
        avg_s = 1e-3 * rows[dom][0] / max(rows[dom][1], 1)
        if dom in alg_bytes:
            ach = alg_bytes[dom] / avg_s / 1e9
            roofline = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(ach / PEAK_HBM_GBS, 4)}
        else:
            # a convolution is priced on the roofline its arithmetic intensity puts it under
            cb = next((b for k, b in conv_bytes.items() if dom.startswith(k)), None)
            if cb is not None and ops_per_conv / cb < ridge:
                ach = cb / avg_s / 1e9
                roofline = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS,
                            "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4),
                            "ops_per_byte": round(ops_per_conv / cb, 1)}
            else:
                ach = ops_per_conv / avg_s / 1e12
                roofline = {"kernel": dom, "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_INT8_TOPS,
                            "unit": "TOP/s", "frac": round(ach / PEAK_INT8_TOPS, 4)}
        roofline["traffic"] = MEASURED_TRAFFIC.get((f"config{args.config}", dom))
        roofline["avg_us"] = round(1e6 * avg_s, 3)

    value = ops_per_step / (ms_per_step * 1e-3) / 1e12
    quant_us = sum(v["avg_us"] * v["launches_per_step"] for k, v in kernels.items()
                   if k in ("fill", "stats", "count_qg", "pack_vq", "pack_qg"))
    result = {
        "metric": "INT8 conv-backward TOPS incl. grad quantization",
        "value": round(value, 3),
        "unit": "TOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"config{args.config}:{layer.name} N={layer.N} {layer.Cin}->{layer.Cout} "
                               f"{layer.Hin}x{layer.Win} k{layer.kH} s{layer.stride} p{layer.pad}",
                   "rotate": R, "rounding": "nearest", "k": 1.0, "A": 0.8, "lambda": 0.3,
                   "streams": args.streams, "hip_graph": bool(args.graph),
                   "dX": "bf16" if args.dx_bf16 else "fp32", "dY": "bf16" if args.dy_bf16 else "fp32",
                   "scheme": args.scheme,
                   "calls": f"{quantize_name} + daq_conv_bwd_int8" if combined else
                            f"{quantize_name} + daq_conv_bwd_filter_int8 + daq_conv_bwd_data_int8"},
        "frac_int8_mfma_peak": round(value / PEAK_INT8_TOPS, 5),
        "quant_GBps_effective_6B": round(6.0 * E_Y / (quant_us * 1e-6) / 1e9, 1) if quant_us else None,
        "quant_us": round(quant_us, 2),
        "event_pair_overhead_us": round(ev_us, 3),
        "kernels": kernels,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        from oracle import daq_ref as ref

        rd = ref.ConvDesc(*layer.desc_fields())
        qX = daq.layout_qx_cnhw(d).unpack(fwd.qx_cnhw)
        qW = daq.layout_qw(d).unpack_plain(d, fwd.qw)
        s_x, s_w = float(fwd.s_x.item()), float(fwd.s_w.item())
        # bounded sample: shrink the batch until the oracle needs roughly <= 30 s
        n_s = layer.N
        while n_s > 1 and 2.0 * layer.macs * n_s / layer.N > 60e9:
            n_s //= 2
        sub = wl.shrink(layer, n_s)
        rds = ref.ConvDesc(*sub.desc_fields())
        # whole passes of the same step on the sample until about ten seconds of CPU work have been timed
        passes, cpu_s = 0, 0.0
        while cpu_s < 10.0 and passes < 64:
            t0 = time.perf_counter()
            rq = ref.quantize_grad(dY[:n_s], st, want_fragile=False,
                                   scheme={"daq": ref.SCHEME_DAQ, "gq": ref.SCHEME_GQ, "gvq": ref.SCHEME_GVQ, "mcs": ref.SCHEME_MCS}[args.scheme])
            ref.conv_bwd_filter_int8(rds, qX[:n_s], s_x, rq.vq, rq.s_chan)
            ref.conv_bwd_data_int8(rds, rq.qg, rq.s_global, qW, s_w)
            cpu_s += time.perf_counter() - t0
            passes += 1
        result["cpu_baseline"] = {
            "value": round(passes * 2.0 * 2.0 * sub.macs / cpu_s / 1e12, 6), "unit": "TOP/s", "cores": ref.num_threads(),
            "kind": "oracle",
            "sample": f"same layer, first {n_s} of {layer.N} images, {passes} passes of the whole step ({cpu_s:.1f} s)"}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
