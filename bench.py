#!/usr/bin/env python3
"""Benchmark of the INT8 conv backward hot path on one MI355X.

One step = the backward pass (Algorithm 1) of EVERY conv layer of a network, last layer first: per layer the
quantizer (statistics, discriminator, clip values, per-channel and global int8 copies of dY, stochastic rounding as
the paper prescribes for gradients), then the data gradient (daq_conv_bwd_data_int8) and, on a second stream, the
filter gradient (daq_conv_bwd_filter_int8): the two share no data, and nothing downstream in a backward pass waits
for dW.  The quantizer is daq_quantize_grad_split, which already hands to the second stream the launches that only
the filter gradient needs.  (--streams 1: every launch on one stream, daq_quantize_grad_ex and both gradients
through daq_conv_bwd_int8; that step is timed as well and reported beside the headline.)  Every layer has its own tensors, as
in a real backward pass: fp32 dY, the int8 activation / filter and their scales saved by the forward entry point, the
clip state, the results.  All of it is resident in HBM before the timed region starts.  The default workload is
ResNet-50 at batch 64 (53 conv layers, 2.8 GB of fp32 dY per step, far beyond the 256 MB Infinity Cache, so every
sweep starts cold).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--rounding stochastic|nearest] [--streams 2|1]
    python bench.py --config 2              # a single layer; its buffers are rotated through enough copies to stay cold
    python bench.py --config 3 --layer 0    # one layer of a config
    python bench.py --sweep --config 4      # every distinct layer shape on its own, one line with per-layer times
    python bench.py --sweep --forward       # the forward entry point over the same layers
    python bench.py --ceilings              # what the GPU delivers: int8 MFMA loop, streaming read / write / copy
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, GB/s
COLD_BYTES = 512 << 20    # a workload whose dY is smaller is replicated until the copies exceed twice the Infinity Cache

QUANT_KERNELS = ("stats", "count_qg", "pack_vq", "pack_qg", "layer_stats", "layer_decide", "chan_resident", "global_copy")
SCHEMES = {"daq": 0, "gq": 1, "gvq": 2, "mcs": 3}
SCHEDULES = {"auto": 0, "three_sweeps": 1, "early_copy": 2, "channel_resident": 3}


# ------------------------------------------------------------------------------------------------ helpers

def measured_traffic(config: int):
    """HBM bytes per step and kernel from the committed rocprofv3 counter summary of this workload, if there is one:
    rows `| kernel | launches | FETCH bytes | WRITE bytes |` of profiles/hbm_traffic_config<N>_network.md."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_config{config}_network.md")
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        m = re.match(r"\|\s*([a-z_0-9]+)\s*\|\s*(\d+)\s*\|\s*([0-9.eE+]+)\s*\|\s*([0-9.eE+]+)\s*\|", line)
        if m:
            out[m.group(1)] = (int(m.group(2)), float(m.group(3)) + float(m.group(4)))
    return out


def traced_avg_us(config: int):
    """Average launch duration per kernel family under the tracer, from the committed rocprofv3 --kernel-trace summary
    of this workload: rows `| kernel | launches per step | us per step | share | avg us | ...` of
    profiles/kernel_trace_config<N>_network.md."""
    path = os.path.join(ROOT, "profiles", f"kernel_trace_config{config}_network.md")
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        m = re.match(r"\|\s*([a-z_0-9]+)\s*\|\s*\d+\s*\|\s*[0-9.]+\s*\|\s*[0-9.]+ %\s*\|\s*([0-9.]+)\s*\|", line)
        if m:
            out[m.group(1)] = float(m.group(2))
    return out


def kernel_work(layer, d, name: str, dy_bytes: float, dx_bytes: float, qg_nhwc: bool, early: bool = False):
    """(algorithmic HBM bytes, int8 operations) of one launch of kernel `name` on `layer`.

    Quantizer sweeps: dY read once per sweep plus the int8 bytes the sweep writes.  `early`: the counting sweep also wrote
    the per-channel copy, and the packing launch after it only repairs the channels whose class was guessed wrong (no
    bytes are attributed to it).  Convolutions: int8 operands read once, result written once; ops = 2 x true
    multiply-accumulates."""
    import numpy as np

    E_Y = float(np.prod(d.y_shape))
    E_X = float(np.prod(d.x_shape))
    E_W = float(np.prod(d.w_shape))
    ops = 2.0 * layer.macs
    if name == "stats":
        return dy_bytes * E_Y, 0.0
    if name == "count_qg":
        return (dy_bytes + (1.0 if qg_nhwc else 0.0) + (1.0 if early else 0.0)) * E_Y, 0.0
    if name == "pack_vq" and early:
        return 0.0, 0.0
    if name in ("pack_vq", "pack_qg", "chan_resident", "global_copy"):
        return (dy_bytes + 1.0) * E_Y, 0.0
    if name.startswith("conv_bwd_data"):
        return E_Y + E_W + dx_bytes * E_X, ops
    if name.startswith("conv_bwd_filter"):
        return E_X + E_Y + 4.0 * E_W, ops
    return 0.0, 0.0


def prof_rows_us(rows, steps):
    """daq_prof_end rows -> {kernel: (us per launch, launches per step)}, with the event pair's own cost removed."""
    ev = rows.pop("(empty event pair)", (0.0, 1))
    ev_us = 1e3 * ev[0] / max(ev[1], 1)
    return {k: (max(1e3 * v[0] / v[1] - ev_us, 1e-3), v[1] / steps) for k, v in rows.items()}, ev_us


class LayerState:
    """Everything one layer's backward step touches, resident on the device."""
    pass


def build_network(args, dev, config, want_sample):
    """Synthetic tensors of every layer (times `rotate` replicas): X = |N(0,1)|, W Kaiming-normal through the forward
    entry point (which saves q(X'), q(W), s_X, s_W), dY mixed bell-shaped / long-tailed per channel, clip state from a
    plausible previous iteration.  Drawn on the device with the recipe of workloads.py; parity on these shapes is the
    business of the tests."""
    import torch

    from paper_2102_04782_amd import binding as daq
    from paper_2102_04782_amd import workloads as wl

    layers = wl.config_layers(config)
    first = 0
    if args.layer >= 0:   # one layer of the config on its own (per-layer profiles); it keeps its seed
        if args.layer >= len(layers):
            raise SystemExit(f"bench.py: config {config} has {len(layers)} layers")
        first, layers = args.layer, layers[args.layer:args.layer + 1]
    dy_total = sum(4 * L.N * L.Cout * L.Ho * L.Wo for L in layers)
    R = args.rotate if args.rotate > 0 else max(1, -(-COLD_BYTES // dy_total))
    n_s = max(1, layers[0].N // 16)
    net, sample = [], []
    for r in range(R):
        for li, L in enumerate(layers):
            d = daq.ConvDesc.make(*L.desc_fields())
            seed = wl.seed_for(config, first + li) + 7919 * r
            gen = torch.Generator(device=dev)
            gen.manual_seed(seed)
            X = torch.randn(d.x_shape, device=dev, generator=gen)
            if config != 1:
                X.abs_()
            std = 0.1 if config == 1 else (2.0 / (L.Cout * L.kH * L.kW)) ** 0.5
            W = torch.randn(d.w_shape, device=dev, generator=gen) * std
            f = daq.conv_fwd_int8(d, X, W)
            del X, W
            s = LayerState()
            s.layer, s.d, s.index = L, d, li
            s.qx_cnhw, s.qw, s.s_x, s.s_w = f.qx_cnhw, f.qw, f.s_x, f.s_w
            dY = wl.make_dY_device(L, seed, dev)
            rho = torch.rand(L.Cout, device=dev, generator=gen) * 0.5 + 0.5
            s.state0 = (rho * dY.abs().amax(dim=(0, 2, 3))).contiguous()
            s.state = s.state0.clone()
            if want_sample and r == 0:
                Ln = daq.layout_qx_nhwc(d)
                qx = f.qx_nhwc[:Ln.N * Ln.H * Ln.W * Ln.c_pitch].view(Ln.N, Ln.H, Ln.W, Ln.c_pitch)[:n_s, :, :, :Ln.C]
                sample.append(dict(layer=wl.shrink(L, min(n_s, L.N)), qX=qx.permute(0, 3, 1, 2).contiguous().cpu().numpy(),
                                   qW=daq.layout_qw(d).unpack_plain(d, f.qw).copy(), s_x=float(f.s_x.item()),
                                   s_w=float(f.s_w.item()), dY=dY[:n_s].float().cpu().numpy(), st=s.state0.cpu().numpy()))
            s.dY = dY.to(torch.bfloat16) if args.dy_bf16 else dY
            del f, dY
            s.out = daq.alloc_quantize_grad(d, dev, want_stats=False)
            s.dW = torch.empty(d.w_shape, device=dev)
            s.dX = torch.empty(d.x_shape, device=dev)
            s.ws_f = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_FILTER, d)), dtype=torch.uint8, device=dev)
            s.ws_d = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_DATA, d)), dtype=torch.uint8, device=dev)
            s.ws_b = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD, d)), dtype=torch.uint8, device=dev)
            s.dXh, s.bf16_ok = None, False
            if args.dx_bf16:
                s.dXh = torch.empty(d.x_shape, dtype=torch.bfloat16, device=dev)
                try:   # layers without a kernel for the narrow result keep fp32
                    daq.conv_bwd_data_int8_bf16(d, s.out.qg, s.s_w, s.qw, s.s_w, dX=s.dXh, workspace=s.ws_d)
                    s.bf16_ok = True
                except daq.DaqError:
                    pass
            net.append(s)
    torch.cuda.synchronize()
    return layers, net, R, sample


def layer_step(args, s, mode, seed):
    """Algorithm 1 for one layer."""
    from paper_2102_04782_amd import binding as daq

    if getattr(args, "given_stats", False):
        # the producer of dY has the channel statistics: one sweep over dY is left (daq_quantize_grad_from_stats)
        q = daq.quantize_grad_from_stats(s.d, s.dY, s.ch_absmax, s.ch_sum, s.ch_sumsq, s.state, args.side, SCHEMES[args.scheme],
                                         SCHEDULES[args.schedule], mode=mode, seed=seed, out=s.out)
        daq.conv_bwd_filter_int8(s.d, s.qx_cnhw, s.s_x, q.vq, q.s_chan, dW=s.dW, workspace=s.ws_f, stream=args.side)
        daq.conv_bwd_data_int8(s.d, q.qg, q.s_global, s.qw, s.s_w, dX=s.dX, workspace=s.ws_d)
        return
    if args.streams == 2:
        # the filter gradient needs the per-channel copy, the data gradient the global one: the two share no data, and
        # the filter gradient (off the critical path of a backward pass) runs on a second stream, ordered there behind
        # the quantizer's launches that it needs (the quantizer makes that stream wait for its own)
        q = daq.quantize_grad_split(s.d, s.dY, s.state, args.side, SCHEMES[args.scheme], SCHEDULES[args.schedule], mode=mode,
                                    seed=seed, out=s.out)
        daq.conv_bwd_filter_int8(s.d, s.qx_cnhw, s.s_x, q.vq, q.s_chan, dW=s.dW, workspace=s.ws_f, stream=args.side)
        if s.bf16_ok:
            daq.conv_bwd_data_int8_bf16(s.d, q.qg, q.s_global, s.qw, s.s_w, dX=s.dXh, workspace=s.ws_d)
        else:
            daq.conv_bwd_data_int8(s.d, q.qg, q.s_global, s.qw, s.s_w, dX=s.dX, workspace=s.ws_d)
        return
    q = daq.quantize_grad_ex(s.d, s.dY, s.state, SCHEMES[args.scheme], SCHEDULES[args.schedule], mode=mode, seed=seed, out=s.out)
    if s.bf16_ok:
        daq.conv_bwd_filter_int8(s.d, s.qx_cnhw, s.s_x, q.vq, q.s_chan, dW=s.dW, workspace=s.ws_f)
        daq.conv_bwd_data_int8_bf16(s.d, q.qg, q.s_global, s.qw, s.s_w, dX=s.dXh, workspace=s.ws_d)
    elif args.separate:
        daq.conv_bwd_filter_int8(s.d, s.qx_cnhw, s.s_x, q.vq, q.s_chan, dW=s.dW, workspace=s.ws_f)
        daq.conv_bwd_data_int8(s.d, q.qg, q.s_global, s.qw, s.s_w, dX=s.dX, workspace=s.ws_d)
    else:
        daq.conv_bwd_int8(s.d, s.qx_cnhw, s.s_x, q.vq, q.s_chan, q.qg, q.s_global, s.qw, s.s_w, dW=s.dW, dX=s.dX,
                          workspace=s.ws_b)


def timed_run(args, net, n_layers, R, mode, steps, warmup):
    """W untimed + K timed network steps between synchronisations; (seconds per step, per-step event times in ms)."""
    import torch

    def step(i):
        r = i % R
        for s in reversed(net[r * n_layers:(r + 1) * n_layers]):   # backward order: last layer first
            layer_step(args, s, mode, seed=i)
        if args.streams == 2:
            torch.cuda.current_stream().wait_stream(args.side)    # the step ends when both streams have

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall / steps, step


def step_statistics(step, n):
    """Median and minimum of n single steps, each bracketed by events on the stream the library launches on."""
    import torch

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record()
    for i in range(n):
        step(i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(n))
    return ms[len(ms) // 2], ms[0]


def profile_pass(args, net, n_layers, R, mode, steps):
    """Per layer and kernel: average launch duration from HIP event pairs around every launch (daq_prof_*), taken inside
    whole network steps so that every kernel meets the caches as in the timed region."""
    from paper_2102_04782_amd import binding as daq

    per = [dict() for _ in range(n_layers)]
    ev_sum = 0.0
    for i in range(steps):
        r = i % R
        for s in reversed(net[r * n_layers:(r + 1) * n_layers]):
            daq.prof_begin()
            layer_step(args, s, mode, seed=i)
            rows, ev_us = prof_rows_us(daq.prof_end(), 1)
            ev_sum += ev_us
            for k, (us, n) in rows.items():
                a = per[s.index].setdefault(k, [0.0, 0.0])
                a[0] += us * n
                a[1] += n
    for p in per:
        for k in p:
            p[k] = (p[k][0] / p[k][1], p[k][1] / steps)   # us per launch, launches per step
    return per, ev_sum / max(1, steps * n_layers)


# ------------------------------------------------------------------------------------------------ modes

def run_network(args, dev) -> int:
    import numpy as np
    import torch

    from paper_2102_04782_amd import binding as daq

    config = args.config
    layers, net, R, sample = build_network(args, dev, config, want_sample=not args.no_cpu_baseline)
    nL = len(layers)
    modes = {"stochastic": daq.ROUND_STOCHASTIC, "nearest": daq.ROUND_NEAREST}
    other = "nearest" if args.rounding == "stochastic" else "stochastic"
    ops_per_step = sum(4.0 * L.macs for L in layers)          # dX + dW, 2 ops per multiply-accumulate
    E_Y_total = sum(float(np.prod(L.y_shape)) for L in layers)

    sec, step = timed_run(args, net, nL, R, modes[args.rounding], args.steps, args.warmup)
    if args.only_timed:
        # for runs under rocprofv3: nothing but the warm-up and the timed steps is launched after the set-up, so every
        # dispatch of a backward kernel belongs to one of W + K identical steps
        if args.copy_calib_mib > 0:   # the plain copy of known size that scales the FETCH_SIZE / WRITE_SIZE readings
            ca = torch.zeros(args.copy_calib_mib << 20, dtype=torch.uint8, device=dev)
            cb = torch.empty_like(ca)
            for _ in range(5):
                cb.copy_(ca)
            torch.cuda.synchronize()
        print(json.dumps({"metric": "INT8 conv-backward TOPS incl. grad quantization", "value": round(ops_per_step / sec / 1e12, 3),
                          "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(1e3 * sec, 5),
                          "config": {"workload": f"config{config}" + (f": {layers[0].name}" if nL == 1 else f": all {nL} conv layers"),
                                     "rounding": args.rounding, "streams": args.streams}}))
        return 0
    n_stat = max(100, args.steps) if sec * max(100, args.steps) < 30.0 else args.steps
    med_ms, min_ms = step_statistics(step, n_stat)
    sec_other, _ = timed_run(args, net, nL, R, modes[other], args.steps, min(args.warmup, 3))
    # the same steps with the other stream count, reported beside the headline; the per-kernel pass below always runs on
    # one stream, where a launch's duration is its own
    head_streams = args.streams
    args.streams, args.side = (1, None) if head_streams == 2 else (2, torch.cuda.Stream())
    sec_alt, _ = timed_run(args, net, nL, R, modes[args.rounding], args.steps, min(args.warmup, 3))
    # and with the channel statistics of dY handed over by its producer (computed here, before the timed region, as a
    # fused producer would have them): what is left of the quantizer is one sweep.  Reported beside the headline only.
    sec_given = None
    if not (args.dy_bf16 or args.dx_bf16 or args.scheme != "daq"):
        for s_ in net:
            g64 = s_.dY.double()
            s_.ch_absmax = s_.dY.abs().amax(dim=(0, 2, 3)).float().contiguous()
            s_.ch_sum = g64.sum(dim=(0, 2, 3)).contiguous()
            s_.ch_sumsq = (g64 * g64).sum(dim=(0, 2, 3)).contiguous()
            del g64
        args.streams, args.side, args.given_stats = 2, torch.cuda.Stream(), True
        sec_given, _ = timed_run(args, net, nL, R, modes[args.rounding], args.steps, min(args.warmup, 3))
        args.given_stats = False
    args.streams, args.side = 1, None
    sec_one = sec if head_streams == 1 else sec_alt

    # the two ways of calling the convolutions must agree bit for bit (first layer of the network, timed tensors)
    s0 = net[0]
    dW2 = daq.conv_bwd_filter_int8(s0.d, s0.qx_cnhw, s0.s_x, s0.out.vq, s0.out.s_chan)
    dX2 = daq.conv_bwd_data_int8(s0.d, s0.out.qg, s0.out.s_global, s0.qw, s0.s_w)
    dW1, dX1 = daq.conv_bwd_int8(s0.d, s0.qx_cnhw, s0.s_x, s0.out.vq, s0.out.s_chan, s0.out.qg, s0.out.s_global, s0.qw, s0.s_w)
    torch.cuda.synchronize()
    if not (torch.equal(dW1, dW2) and torch.equal(dX1, dX2)):
        print("bench.py: daq_conv_bwd_int8 does not reproduce the two separate calls", file=sys.stderr)
        return 3
    del dW1, dW2, dX1, dX2

    per, ev_us = profile_pass(args, net, nL, R, modes[args.rounding], max(2, min(args.steps, 10)))
    dy_b = 2.0 if args.dy_bf16 else 4.0
    kernels, phases = {}, {"quantize": 0.0, "dW": 0.0, "dX": 0.0}
    floors = {"quantize": 0.0, "dW": 0.0, "dX": 0.0}   # per phase: sum over launches of max(ops / int8 peak, algorithmic bytes / HBM peak)
    layer_rows = []
    for li, L in enumerate(layers):
        d = net[li].d
        qg_nhwc = daq.layout_qg(d).kind == daq.LAYOUT_NHWC
        row = {"layer": L.name, "shape": f"N{L.N} {L.Cin}->{L.Cout} {L.Hin}x{L.Win} k{L.kH} s{L.stride} g{L.groups}"}
        for k, (us, n) in per[li].items():
            dx_b = 2.0 if (net[li].bf16_ok and k.startswith("conv_bwd_data")) else 4.0
            # the library's rule for the early per-channel copy (gradients of 8 Mi elements and more, NHWC global copy,
            # rows of an even number of pixels); a layer without a channel-resident launch took the sweeps
            early = (args.scheme == "daq" and qg_nhwc and "chan_resident" not in per[li] and L.Wo % 2 == 0 and
                     (args.schedule == "early_copy" or (args.schedule == "auto" and float(np.prod(d.y_shape)) >= 8 * 2 ** 20)))
            b, o = kernel_work(L, d, k, dy_b, dx_b, qg_nhwc, early)
            e = kernels.setdefault(k, {"us": 0.0, "launches": 0.0, "bytes": 0.0, "ops": 0.0})
            e["us"] += us * n
            e["launches"] += n
            e["bytes"] += b * n
            e["ops"] += o * n
            ph = "quantize" if k in QUANT_KERNELS else "dW" if (k.startswith("conv_bwd_filter") or k == "dw_reduce") else "dX"
            phases[ph] += us * n
            row[ph + "_us"] = round(row.get(ph + "_us", 0.0) + us * n, 1)
            row.setdefault("kernels_us", {})[k] = round(us * n, 1)
            fl = 1e6 * n * max(o / (PEAK_INT8_TOPS * 1e12), b / (PEAK_HBM_GBS * 1e9))
            floors[ph] += fl
            row[ph + "_roofline_us"] = round(row.get(ph + "_roofline_us", 0.0) + fl, 2)
        # fraction of the layer's roofline min(int8 peak, ops/byte x HBM peak) each phase reaches: floor time / measured time
        row["frac_of_roofline"] = {ph: round(row[ph + "_roofline_us"] / row[ph + "_us"], 3) for ph in ("quantize", "dW", "dX")
                                   if row.get(ph + "_us", 0.0) > 0}
        layer_rows.append(row)
    ridge = PEAK_INT8_TOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    traffic = measured_traffic(config) if (args.rounding == "stochastic" and args.layer < 0 and not (args.dy_bf16 or args.dx_bf16 or args.separate or args.scheme != "daq" or args.schedule != "auto")) else {}
    table = {}
    for k, e in kernels.items():
        t = e["us"] * 1e-6
        ent = {"us_per_step": round(e["us"], 1), "launches_per_step": round(e["launches"], 2)}
        if e["bytes"] > 0:
            ent["GBps"] = round(e["bytes"] / t / 1e9, 1)
        if e["ops"] > 0:
            ent["TOPs"] = round(e["ops"] / t / 1e12, 1)
        table[k] = ent
    dom = max(kernels.items(), key=lambda kv: kv[1]["us"])[0]
    e = kernels[dom]
    n_l = max(e["launches"], 1e-9)
    avg_s = e["us"] * 1e-6 / n_l
    if e["ops"] > 0 and e["ops"] / e["bytes"] >= ridge:
        ach = e["ops"] / n_l / avg_s / 1e12
        roofline = {"kernel": dom, "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                    "frac": round(ach / PEAK_INT8_TOPS, 4)}
    else:
        ach = e["bytes"] / n_l / avg_s / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBS, 4)}
        if e["ops"] > 0:
            roofline["ops_per_byte"] = round(e["ops"] / e["bytes"], 1)
    tr = traffic.get(dom)
    roofline["traffic"] = round(tr[1] / max(tr[0], 1), 1) if tr else None
    roofline["algorithmic_bytes_per_launch"] = round(e["bytes"] / n_l, 1)
    roofline["avg_us"] = round(1e6 * avg_s, 3)
    roofline["launches_per_step"] = round(e["launches"], 2)
    # the same kernel's average in the committed rocprofv3 trace of this workload (one stream).  Launches are about 2 us
    # longer under the tracer than between HIP events, for every kernel family - the traced step as a whole is 12 % longer
    # than the untraced one - so both are given, and the fraction that follows from the tracer's figure beside them.
    tr_us = traced_avg_us(config).get(dom) if traffic else None
    roofline["rocprofv3_avg_us"] = tr_us
    roofline["frac_at_rocprofv3_avg"] = round(roofline["frac"] * 1e6 * avg_s / tr_us, 4) if tr_us else None

    value = ops_per_step / sec / 1e12
    L0 = layers[0]
    result = {
        "metric": "INT8 conv-backward TOPS incl. grad quantization",
        "value": round(value, 3),
        "unit": "TOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(1e3 * sec, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": f"config{config}: " + (f"all {nL} conv layers of the network" if nL > 1 else L0.name) +
                               f", N={L0.N}, one backward step (quantize + dW + dX) per layer and step",
                   "rounding": args.rounding, "k": 1.0, "A": 0.8, "lambda": 0.3, "buffer_sets": R,
                   "dY_bytes_per_step": int(dy_b * E_Y_total), "cold": bool(R * dy_b * E_Y_total >= COLD_BYTES),
                   "dX": "bf16 where served" if args.dx_bf16 else "fp32", "dY": "bf16" if args.dy_bf16 else "fp32",
                   "scheme": args.scheme, "schedule": args.schedule, "streams": head_streams,
                   "calls": "daq_quantize_grad_split + daq_conv_bwd_data_int8, and daq_conv_bwd_filter_int8 on the second stream"
                            if head_streams == 2 else "daq_quantize_grad_ex + " + (
                       "daq_conv_bwd_filter_int8 + daq_conv_bwd_data_int8" if (args.separate or args.dx_bf16) else "daq_conv_bwd_int8")},
        "frac_int8_mfma_peak": round(value / PEAK_INT8_TOPS, 5),
        "step_ms_median": round(med_ms, 5), "step_ms_min": round(min_ms, 5), "stat_steps": n_stat,
        other: {"ms_per_step": round(1e3 * sec_other, 5), "value": round(ops_per_step / sec_other / 1e12, 3)},
        ("one_stream" if head_streams == 2 else "two_streams"): {
            "ms_per_step": round(1e3 * sec_alt, 5), "value": round(ops_per_step / sec_alt / 1e12, 3),
            "what": "every launch on one stream" if head_streams == 2 else "filter gradients on a second stream"},
        "producer_statistics": None if sec_given is None else {
            "ms_per_step": round(1e3 * sec_given, 5), "value": round(ops_per_step / sec_given / 1e12, 3),
            "what": "not the headline: daq_quantize_grad_from_stats, |g|max / sum / sum of squares per channel supplied by the "
                    "producer of dY (computed before the timed region), two streams"},
        "phase_us_per_step": {k: round(v, 1) for k, v in phases.items()},
        "phase_note": "sums of single launch durations measured on one stream",
        "launch_gap_us_per_step": round(1e6 * sec_one - sum(phases.values()), 1),
        "quant_GBps_effective_6B": round(6.0 * E_Y_total / (phases["quantize"] * 1e-6) / 1e9, 1) if phases["quantize"] else None,
        "event_pair_overhead_us": round(ev_us, 3),
        "kernels": table,
        "roofline": roofline,
    }
    result["frac_of_roofline_by_phase"] = {ph: round(floors[ph] / phases[ph], 3) for ph in phases if phases[ph] > 0}
    if args.layers:
        result["layers"] = layer_rows

    if not args.no_cpu_baseline:
        from oracle import daq_ref as ref

        # bounded sample: every layer of the network at 1/16 of the batch, whole passes until about ten seconds are timed
        passes, cpu_s = 0, 0.0
        s_ops = sum(4.0 * smp["layer"].macs for smp in sample)
        while cpu_s < 10.0 and passes < 16:
            t0 = time.perf_counter()
            for smp in reversed(sample):
                rd = ref.ConvDesc(*smp["layer"].desc_fields())
                rq = ref.quantize_grad(smp["dY"], smp["st"], mode=ref.ROUND_STOCHASTIC if args.rounding == "stochastic" else ref.ROUND_NEAREST,
                                       seed=passes, want_fragile=False, scheme=SCHEMES[args.scheme])
                ref.conv_bwd_filter_int8(rd, smp["qX"], smp["s_x"], rq.vq, rq.s_chan)
                ref.conv_bwd_data_int8(rd, rq.qg, rq.s_global, smp["qW"], smp["s_w"])
            cpu_s += time.perf_counter() - t0
            passes += 1
        result["cpu_baseline"] = {
            "value": round(passes * s_ops / cpu_s / 1e12, 6), "unit": "TOP/s", "cores": ref.num_threads(), "kind": "oracle",
            "sample": f"every layer of the workload at the first {sample[0]['layer'].N} of {L0.N} images, {passes} "
                      f"pass(es) of the whole step ({cpu_s:.1f} s); a rate, so no extrapolation is involved"}
    print(json.dumps(result))
    return 0


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
            rows, _ = prof_rows_us(daq.prof_end(), steps)
            t = {k: us * n for k, (us, n) in rows.items()}
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
    """Every distinct layer shape of a config on its own: its step repeated back to back (a small layer then finds its
    tensors in the caches - the per-layer figures of the design notes; the default mode is the cold whole-network run)."""
    import torch

    from paper_2102_04782_amd import binding as daq
    from paper_2102_04782_amd import workloads as wl

    layers = wl.config_layers(args.config)
    mode = daq.ROUND_STOCHASTIC if args.rounding == "stochastic" else daq.ROUND_NEAREST
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
            s = LayerState()
            s.layer, s.d, s.index = L, d, li
            s.dY = torch.randn(d.y_shape, device=dev, generator=gen) * 1e-2
            if args.dy_bf16:
                s.dY = s.dY.to(torch.bfloat16)
            s.state = torch.zeros(d.Cout, device=dev)
            f = daq.conv_fwd_int8(d, torch.randn(d.x_shape, device=dev, generator=gen).abs_(),
                                  torch.randn(d.w_shape, device=dev, generator=gen))
            s.qx_cnhw, s.qw, s.s_x, s.s_w = f.qx_cnhw, f.qw, f.s_x, f.s_w
            del f
            s.out = daq.alloc_quantize_grad(d, dev, want_stats=False)
            s.dW = torch.empty(d.w_shape, device=dev)
            s.dX = torch.empty(d.x_shape, device=dev)
            s.ws_f = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_FILTER, d)), dtype=torch.uint8, device=dev)
            s.ws_d = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD_DATA, d)), dtype=torch.uint8, device=dev)
            s.ws_b = torch.empty(max(256, daq.workspace_bytes(daq.OP_CONV_BWD, d)), dtype=torch.uint8, device=dev)
            s.dXh, s.bf16_ok = None, False
            if args.dx_bf16:
                s.dXh = torch.empty(d.x_shape, dtype=torch.bfloat16, device=dev)
                try:
                    daq.conv_bwd_data_int8_bf16(d, s.out.qg, s.s_w, s.qw, s.s_w, dX=s.dXh, workspace=s.ws_d)
                    s.bf16_ok = True
                except daq.DaqError:
                    pass
            for i in range(3):
                layer_step(args, s, mode, i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                layer_step(args, s, mode, i)
            torch.cuda.synchronize()
            wall_us = 1e6 * (time.perf_counter() - t0) / steps
            daq.prof_begin()
            for i in range(steps):
                layer_step(args, s, mode, i)
            rows, _ = prof_rows_us(daq.prof_end(), steps)
            t = {k: us * n for k, (us, n) in rows.items()}
            seen[key] = (wall_us,
                         sum(v for k, v in t.items() if k in QUANT_KERNELS),
                         sum(v for k, v in t.items() if k.startswith("conv_bwd_filter") or k == "dw_reduce"),
                         sum(v for k, v in t.items() if k.startswith("conv_bwd_data")))
            del s
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
                               f"N={layers[0].N}, each shape's step repeated back to back (warm)", "rounding": args.rounding},
        "frac_int8_mfma_peak": round(value / PEAK_INT8_TOPS, 5),
        "kernel_us_total": {k: round(v, 1) for k, v in tot.items()},
        "layers": out_layers}))
    return 0


def ceilings(args, dev) -> int:
    """What this GPU delivers on the two resources everything here is priced against."""
    import torch

    from paper_2102_04782_amd import binding as daq

    sink = torch.zeros(64, dtype=torch.int32, device=dev)
    nbytes = 1 << 30
    a = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=dev)
    b = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    small = torch.zeros(24 << 20, dtype=torch.uint8, device=dev)

    def timed(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        best = 1e30
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, 1e-3 * e0.elapsed_time(e1))
        return best

    out = {}
    ops = [0.0]

    def mfma():
        ops[0] = daq.ceiling_mfma_i8(256 * 8, 20000, sink)
    t = timed(mfma, 5)
    out["mfma_i8_32x32x32_TOPs"] = round(ops[0] / t / 1e12, 1)
    for name, mode, src, dst, n, traffic in (("read_1GiB", 0, a, None, nbytes, 1), ("write_1GiB", 1, None, b, nbytes, 1),
                                             ("copy_1GiB", 2, a, b, nbytes, 2), ("read_24MiB_cache_resident", 0, small, None, 24 << 20, 1)):
        best = {}
        for blocks in (256, 512, 768, 1024, 2048, 4096, 8192, 16384):   # fewer, longer workgroups stream faster on this chip
            t = timed(lambda: daq.ceiling_stream(mode, src, dst, n, blocks, sink))
            best[blocks] = traffic * n / t / 1e9
        k = max(best, key=best.get)
        out[name + "_GBps"] = round(best[k], 1)
        out[name + "_blocks"] = k
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(200):
        daq.ceiling_stream(0, small, None, 16, 1, sink)
    e1.record()
    torch.cuda.synchronize()
    out["empty_kernel_back_to_back_us"] = round(1e3 * e0.elapsed_time(e1) / 200, 2)
    print(json.dumps({"metric": "machine ceilings", "unit": "see keys", "n_gpus": 1,
                      "peaks": {"int8_mfma_TOPs": PEAK_INT8_TOPS, "hbm_GBps": PEAK_HBM_GBS}, "measured": out,
                      "note": "copy counts bytes read + bytes written; best of 10 launches, HIP events"}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload 1-5: 1 tiny layer, 2 and 3 single ResNet-50 layers, 4 = ResNet-50 at batch 64, 5 = MobileNetV2 at batch 128")
    ap.add_argument("--layer", type=int, default=-1, help="restrict the workload to this layer of the config (0-based)")
    ap.add_argument("--rounding", default="stochastic", choices=("stochastic", "nearest"),
                    help="rounding of the gradient quantizer in the reported step (the paper prescribes stochastic rounding "
                         "for gradients); the other mode is timed as well and reported beside it")
    ap.add_argument("--rotate", type=int, default=0,
                    help="buffer sets cycled through; 0 = as many as it takes for the dY tensors in flight to exceed 512 MiB")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", action="store_true", help="add the per-layer table to the JSON line")
    ap.add_argument("--separate", action="store_true",
                    help="call daq_conv_bwd_filter_int8 and daq_conv_bwd_data_int8 one after the other instead of "
                         "daq_conv_bwd_int8 (both gradients in one call, one launch fewer)")
    ap.add_argument("--dx-bf16", action="store_true",
                    help="store the data gradient as bfloat16 (daq_conv_bwd_data_int8_bf16: an option beside the method, "
                         "which returns fp32 gradients; reported for comparison, never the default)")
    ap.add_argument("--scheme", default="daq", choices=tuple(SCHEMES),
                    help="rule for the per-channel clip values: Algorithm 1 (default) or one of the ablation study's variants")
    ap.add_argument("--only-timed", action="store_true",
                    help="set-up, warm-up and the timed steps only, short JSON line: for runs under rocprofv3")
    ap.add_argument("--copy-calib-mib", type=int, default=0,
                    help="with --only-timed: afterwards run 5 device-to-device copies of this many MiB, the plain copy "
                         "kernel of known size that scales rocprofv3's FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--streams", type=int, default=2, choices=(1, 2),
                    help="2 (default): a layer's filter gradient, which nothing downstream in a backward pass waits for, and "
                         "the quantizer launches only it needs run on a second stream beside the data gradient and the "
                         "next layer's quantizer; 1: every launch on one stream.  The other count is timed too and reported beside")
    ap.add_argument("--schedule", default="auto", choices=tuple(SCHEDULES),
                    help="how the quantizer shares its sweeps over dY among its launches (daq_quantize_grad_ex); same results")
    ap.add_argument("--dy-bf16", action="store_true",
                    help="hand the output gradient over as bfloat16 (same algorithm on the widened values; reported for "
                         "comparison, never the default)")
    ap.add_argument("--sweep", action="store_true",
                    help="time the step of every distinct layer shape of --config on its own and report the network total")
    ap.add_argument("--forward", action="store_true",
                    help="with --sweep: time the forward entry point (daq_conv_fwd_int8) of every layer instead")
    ap.add_argument("--ceilings", action="store_true", help="measure the int8 MFMA and streaming ceilings of this GPU")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        return 2

    import torch

    from paper_2102_04782_amd import binding as daq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    daq.lib()  # fail loudly if the HIP library is missing
    args.side = torch.cuda.Stream() if args.streams == 2 else None
    if args.ceilings:
        return ceilings(args, dev)
    if args.sweep:
        return sweep_forward(args, dev) if args.forward else sweep(args, dev)
    return run_network(args, dev)


if __name__ == "__main__":
    sys.exit(main())
