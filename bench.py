#!/usr/bin/env python3
"""Benchmark of the HOT linear-layer backward hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
forward-time activation compression, the g_x path and the g_w path of one
linear layer (Sec. 5.1, 5.2, 5.2.1).  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
INT8_PEAK_TOPS = 5000.0     # MI355X dense int8 MFMA
BF16_PEAK_TOPS = 2500.0     # MI355X dense bf16 MFMA (gw_bits = 16 variant)


def stage_model(L, O, I, n, r, gx_bits, per_token, gw_bits=8, Lr=None):
    """Algorithmic work per launch of every kernel role: HBM bytes for the
    transform/quantise kernels, integer ops (and compulsory bytes) for the GEMMs."""
    Lr = L // n * r if Lr is None else Lr
    cb = gx_bits / 8.0
    wb = gw_bits / 8.0
    m = {
        "act_col_absmax": dict(bound="hbm", bytes=4 * L * I),
        "act_col_quant": dict(bound="hbm", bytes=4 * L * I + wb * Lr * I),
        "w_col_absmax": dict(bound="hbm", bytes=4 * O * I),
        "w_col_quant": dict(bound="hbm", bytes=4 * O * I + cb * O * I),
        "gy_row_quant": dict(bound="hbm", bytes=4 * L * O + cb * L * O + 4 * L),
        "w_and_gy_row_quant": dict(bound="hbm", bytes=4 * L * O + cb * L * O + 4 * L + 4 * O * I + cb * O * I),
        "gy_row_absmax": dict(bound="hbm", bytes=4 * L * O),
        "gy_row_quant2": dict(bound="hbm", bytes=4 * L * O + cb * L * O),
        "gyT_col_absmax": dict(bound="hbm", bytes=4 * L * O),
        "gyT_col_quant": dict(bound="hbm", bytes=4 * L * O + wb * Lr * O),
        "gy_fused_absmax": dict(bound="hbm", bytes=4 * L * O + (4 * L * ((O + 127) // 128) if per_token else 0)),
        "gy_fused_quant": dict(bound="hbm", bytes=4 * L * O + cb * L * O + Lr * O + 4 * L),
        "gx_igemm": dict(bound="mfma", ops=2 * L * O * I, bytes=cb * (L * O + I * O) + 4 * L * I),
        "gw_igemm": dict(bound="mfma", ops=2 * O * I * Lr, bytes=wb * Lr * (O + I) + 4 * O * I,
                         peak=BF16_PEAK_TOPS if gw_bits == 16 else INT8_PEAK_TOPS),
    }
    return m


def profiled_traffic(workload, role):
    """HBM bytes per launch (fetched + written) of a kernel role, from the committed
    rocprofv3 counter summary of this workload (FETCH_SIZE / WRITE_SIZE, scaled by a copy
    of known size); None when no summary covers it."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"hbm_traffic_{workload}.txt")
    try:
        with open(path) as fh:
            for line in fh:
                f = line.split()
                if len(f) == 4 and f[0] == "traffic_bytes" and f[1] == role:
                    return int(f[2]) + int(f[3])
    except OSError:
        pass
    return None


def run_sweep(torch, hot, hot_inputs, wl, quantizer_flag):
    """Forward-time compression of every layer of a workload, then the backward of every
    layer (a chain when the workload says so: each g_x is the next lower layer's g_y).
    Returns per-layer times (HIP events on the launch stream), buffer bytes and peak memory."""
    n, r = wl.block, wl.keep
    cfg = hot.Config(block=n, keep=r)
    depth = int(wl.extra.get("depth", 0))
    chain = depth > 0
    layers = [(f"{d}.{l.name}", l) for d in range(depth) for l in wl.layers] if chain \
        else [(l.name, l) for l in wl.layers]
    torch.cuda.reset_peak_memory_stats()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    acts, rows = [], []
    ws = torch.empty(max(hot.hot_workspace_bytes(cfg, l.L, l.O, l.I) for _, l in layers),
                     dtype=torch.uint8, device="cuda")
    fp32_bytes = act_bytes = 0
    for name, l in layers:           # "forward": only what the backward will need is kept
        x = hot_inputs.make_x(wl.x_kind, l.L, l.I, 0, f"{wl.name}.{name}", "cuda")
        act = hot.alloc_act_buffer(cfg, l.L, l.I)
        e0, e1 = ev(), ev()
        e0.record()
        hot.hot_compress_activation(cfg, x, act, ws)
        e1.record()
        torch.cuda.synchronize()
        rows.append(dict(layer=name, L=l.L, O=l.O, I=l.I, compress_us=round(e0.elapsed_time(e1) * 1e3, 1)))
        acts.append(act)
        fp32_bytes += 4 * l.L * l.I
        act_bytes += act.numel()
        del x
    g_y = None
    for k in range(len(layers) - 1, -1, -1):
        name, l = layers[k]
        w = hot_inputs.make_w(l.O, l.I, 0, f"{wl.name}.{name}", "cuda")
        if g_y is None or not chain:
            g_y = hot_inputs.make_gy(wl.gy_kind, l.L, l.O, 0, f"{wl.name}.{name}", "cuda")
        quant = quantizer_flag or wl.quantizer
        row = rows[k]
        if quant == "select":
            choice, m_tok, m_ten = hot.hot_select_quantizer(cfg, g_y, ws)
            quant = "token" if choice == hot.HOT_Q_PER_TOKEN else "tensor"
            row.update(mse_token=m_tok, mse_tensor=m_ten)
        q = hot.HOT_Q_PER_TOKEN if quant == "token" else hot.HOT_Q_PER_TENSOR
        g_x = torch.empty((l.L, l.I), device="cuda")
        g_w = torch.empty((l.O, l.I), device="cuda")
        e0, e1 = ev(), ev()
        e0.record()
        hot.hot_linear_backward(cfg, g_y, w, acts[k], q, g_x, g_w, ws)
        e1.record()
        torch.cuda.synchronize()
        bw_us = e0.elapsed_time(e1) * 1e3
        Lr = cfg.reduced_tokens(l.L)
        row.update(gy_quantizer=quant, backward_us=round(bw_us, 1),
                   backward_TOPS=round((2.0 * l.L * l.O * l.I + 2.0 * l.O * l.I * Lr) / bw_us / 1e6, 1),
                   finite=bool(torch.isfinite(g_x).all().item() and torch.isfinite(g_w).all().item()))
        acts[k] = None
        g_y = g_x if chain else None
        del w, g_w
    total_us = sum(x["compress_us"] + x["backward_us"] for x in rows)
    ops = sum(2.0 * l.L * l.O * l.I + 2.0 * l.O * l.I * (l.L // n * r) for _, l in layers)
    return dict(workload=wl.name, layers=rows, total_us=round(total_us, 1),
                effective_TOPS=round(ops / total_us / 1e6, 1),
                act_buffer_bytes=act_bytes, act_fp32_bytes=fp32_bytes,
                peak_device_bytes=int(torch.cuda.max_memory_allocated()))


def probe_peaks(torch, hot):
    """Plain HBM read / write rate and raw int8 matrix rate of this machine (context only)."""
    out = {}
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(kind, buf, iters, reps):
        hot.hot_debug_probe(kind, buf, iters)
        torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            hot.hot_debug_probe(kind, buf, iters)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps * 1e-3

    for mb in (155, 1024):
        buf = torch.zeros(mb * 1000 * 1000 // 4, dtype=torch.float32, device="cuda")
        nbytes = buf.numel() * 4 - 4096
        out[f"hbm_read_GBps_{mb}MB"] = round(nbytes / timed(0, buf, 1, 10) / 1e9, 1)
        out[f"hbm_write_GBps_{mb}MB"] = round(nbytes / timed(1, buf, 1, 10) / 1e9, 1)
        del buf
    buf = torch.zeros(1 << 20, dtype=torch.int32, device="cuda")
    iters = 4000
    ops = 2.0 * 32 * 32 * 32 * 16 * iters * 256 * 4
    out["mfma_i8_TOPS_constant_operands"] = round(ops / timed(2, buf, iters, 3) / 1e12, 1)
    out["mfma_i8_TOPS_random_operands"] = round(ops / timed(3, buf, iters, 6) / 1e12, 1)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_vitb_fc1")
    ap.add_argument("--quantizer", default=None, choices=[None, "token", "tensor"])
    ap.add_argument("--cpu-sample-tokens", type=int, default=0,
                    help="tokens of the workload the oracle is timed on (0 = all of them)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="repeat the oracle on the sample until about this much CPU wall time")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--backward", default="auto", choices=["auto", "separate", "shared", "unfused"],
                    help="how hot_linear_backward produces the two views of g_y: the library's "
                         "choice (default), always the two separate paths, or the shared g_y "
                         "passes wherever they exist")
    ap.add_argument("--gemm", type=int, default=0,
                    help="work distribution of the GEMMs: 0 = the library's choice (default), 1 = one "
                         "workgroup per output tile, s >= 2 = s K slices wherever a split applies")
    ap.add_argument("--probe-peaks", action="store_true",
                    help="instead of the workload, time plain HBM read/write and a register-only "
                         "int8 matrix loop, and print them as JSON")
    ap.add_argument("--gw-bits", type=int, default=8, choices=[8, 16],
                    help="g_w operands: 8 = INT8 (the paper), 16 = bfloat16 variant")
    ap.add_argument("--sample-tokens", type=int, default=0,
                    help="tile the token axis per sample of this many tokens (197 for the ViT "
                         "workloads) instead of as one run")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the timed step, run every layer of the workload once (compress "
                         "all, then backward all; chained where the workload is a chain) and print "
                         "per-layer times, buffer bytes and peak device memory as JSON")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of g_y (for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs the HOT backward on ONE GPU; "
                         "--gpus N with N > 1 is not supported.\n")
        return 2

    import torch
    import hot_inputs
    import paper_2503_21261_amd as hot

    hot.lib()  # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    if args.probe_peaks:
        print(json.dumps(probe_peaks(torch, hot)))
        return 0
    wl = hot_inputs.WORKLOADS[args.workload]
    hot.hot_debug_set_gemm_mode(args.gemm)
    if args.sweep:
        hot.hot_debug_set_backward_strategy({"auto": 0, "separate": 1, "shared": 2, "unfused": 3}[args.backward])
        run_sweep(torch, hot, hot_inputs, wl, args.quantizer)   # warm-up: code objects, allocator
        print(json.dumps(run_sweep(torch, hot, hot_inputs, wl, args.quantizer)))
        return 0
    layer = wl.layers[0]
    L, O, I, n, r = layer.L, layer.O, layer.I, wl.block, wl.keep
    quant = args.quantizer or ("token" if wl.quantizer in ("token", "select") else "tensor")
    per_token = quant == "token"
    cfg = hot.Config(block=n, keep=r, gw_bits=args.gw_bits, sample_tokens=args.sample_tokens)

    x, w, gy = hot_inputs.make_layer(wl, layer, seed=0, device="cuda")
    ws = hot.alloc_workspace(cfg, L, O, I)
    act = hot.alloc_act_buffer(cfg, L, I)
    gx = torch.empty((L, I), device="cuda")
    gw = torch.empty((O, I), device="cuda")
    q = hot.HOT_Q_PER_TOKEN if per_token else hot.HOT_Q_PER_TENSOR
    stream = torch.cuda.current_stream()
    hot.hot_debug_set_backward_strategy({"auto": 0, "separate": 1, "shared": 2, "unfused": 3}[args.backward])

    def step():
        hot.hot_compress_activation(cfg, x, act, ws, stream=stream)
        hot.hot_linear_backward(cfg, gy, w, act, q, gx, gw, ws, stream=stream)

    if args.calibrate_copy:
        scratch = torch.empty_like(gy)
        for _ in range(5):
            scratch.copy_(gy)
        torch.cuda.synchronize()
        del scratch

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # same steps again with HIP events around every kernel (on the launch stream)
    hot.hot_debug_profile_begin()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = hot.hot_debug_profile_end()

    model = stage_model(L, O, I, n, r, cfg.gx_bits, per_token, cfg.gw_bits, cfg.reduced_tokens(L))
    kernels = {}
    for name, (ms, cnt) in prof.items():
        avg_us = ms * 1e3 / cnt
        k = dict(avg_us=round(avg_us, 3), launches_per_step=cnt / args.steps)
        mdl = model.get(name)
        if mdl:
            k["bound"] = mdl["bound"]
            k["GBps"] = round(mdl["bytes"] / (avg_us * 1e-6) / 1e9, 1)
            if "ops" in mdl:
                k["TOPS"] = round(mdl["ops"] / (avg_us * 1e-6) / 1e12, 2)
            # fraction of the published peak that bounds this kernel (HBM 8 TB/s or the MFMA peak)
            k["frac"] = round(k["TOPS"] / mdl.get("peak", INT8_PEAK_TOPS) if mdl["bound"] == "mfma"
                              else k["GBps"] / HBM_PEAK_GBS, 4)
        kernels[name] = k
    dominant = max((k for k in kernels if k in model), key=lambda k: kernels[k]["avg_us"])
    d, dm = kernels[dominant], model[dominant]
    if dm["bound"] == "hbm":
        roof = dict(kernel=dominant, bound="hbm", achieved=d["GBps"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(d["GBps"] / HBM_PEAK_GBS, 4), traffic=None,
                    algorithmic_bytes=int(dm["bytes"]), avg_us=d["avg_us"])
    else:
        peak = dm.get("peak", INT8_PEAK_TOPS)
        roof = dict(kernel=dominant, bound="mfma", achieved=d["TOPS"], peak=peak, unit="TOP/s",
                    frac=round(d["TOPS"] / peak, 4), traffic=None,
                    algorithmic_ops=int(dm["ops"]), avg_us=d["avg_us"])

    if quant == "token" and args.backward == "auto" and args.gw_bits == 8 and not args.sample_tokens:   # what the counter runs measured
        roof["traffic"] = profiled_traffic(wl.name, dominant)
    Lr = cfg.reduced_tokens(L)
    ops_step = 2 * L * O * I + 2 * O * I * Lr          # integer ops actually executed
    value = ops_step / (ms_per_step * 1e-3) / 1e12

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        Ls = L if args.cpu_sample_tokens <= 0 else min(L, max(n, args.cpu_sample_tokens // n * n))
        xs, gys, wh = x[:Ls].cpu().numpy(), gy[:Ls].cpu().numpy(), w.cpu().numpy()
        oracle.lib()
        if cfg.sample_tokens:     # the oracle's per-sample definition: zero tokens after every sample
            Ls = L
            xs, gys = x.cpu().numpy(), gy.cpu().numpy()
            xs_t, gys_t = oracle.pad_samples(xs, cfg.sample_tokens, n), oracle.pad_samples(gys, cfg.sample_tokens, n)
        else:
            xs_t, gys_t = xs, gys
        reps, dt = 0, 0.0
        while reps < 1 or (dt < args.cpu_seconds and reps < 64):
            t0 = time.perf_counter()
            oracle.backward_gx(gys, wh, n, bits=cfg.gx_bits, per_token=per_token, taps=False)
            if cfg.gw_bits == 16:
                oracle.backward_gw_bf16(gys_t, oracle.compress_activation_bf16(xs_t, n, r), n, r)
            else:
                codes, sx = oracle.compress_activation(xs_t, n, r)
                oracle.backward_gw(gys_t, codes, sx, n, r, taps=False)
            dt += time.perf_counter() - t0
            reps += 1
        ops_s = 2 * Ls * O * I + 2 * O * I * cfg.reduced_tokens(Ls)
        cpu = dict(value=round(ops_s * reps / dt / 1e12, 6), unit="TOPS", cores=oracle.threads(), kind="oracle",
                   sample=f"{'all' if Ls == L else 'first ' + str(Ls) + ' of'} {L} tokens of {wl.name} "
                          f"(compress + g_x + g_w), {reps} passes in {dt:.1f} s",
                   seconds_per_pass=round(dt / reps, 3))

    out = {
        "metric": "HOT linear-backward effective TOPS (integer ops executed / step time)",
        "value": round(value, 3), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "us_per_step": round(ms_per_step * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8" if cfg.gw_bits == 8 else "int8 (g_x) + bf16 (g_w)",
        "data": "synthetic",
        "config": {"workload": wl.name, "L": L, "O": O, "I": I, "block": n, "keep": r,
                   "gx_bits": cfg.gx_bits, "gw_bits": cfg.gw_bits, "gy_quantizer": quant,
                   "sample_tokens": cfg.sample_tokens,
                   "step": "compress_activation + linear_backward (g_x and g_w; g_y views: %s; GEMM work "
                           "distribution: %s)" % (args.backward, {0: "auto", 1: "tile"}.get(args.gemm, "K split %d" % args.gemm))},
        "act_buffer_bytes": hot.hot_act_buffer_bytes(cfg, L, I), "act_fp32_bytes": 4 * L * I,
        "roofline": roof, "cpu_baseline": cpu, "kernels": kernels,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
