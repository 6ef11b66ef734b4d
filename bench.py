#!/usr/bin/env python3
"""Benchmark of the HOT linear-layer backward hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input: forward-time
activation compression of every layer of a workload (Sec. 5.2.1), then the g_x and g_w
paths of every layer (Sec. 5.1, 5.2), top layer first; in a chain each layer's g_x is the
g_y of the layer below.  All inputs are resident in HBM before the timed region.

With no --workload the headline is the largest single-GPU workload (the ViT-L chain at
201728 tokens, 48 layers per step) and the four smaller configurations are run the same
way and reported under "workloads".  Prints ONE JSON line.
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
HEADLINE = "cfg5_vitl_chain"
OTHERS = ["cfg1_single_512x768x768", "cfg2_vitb_fc1", "cfg3_vitb_block_b256", "cfg4_llm7b_mlp"]
STRATEGY = {"auto": 0, "separate": 1, "shared": 2, "unfused": 3}


def stage_model(L, O, I, n, r, gx_bits, per_token, gw_bits=8, Lr=None):
    """Algorithmic work per launch of every kernel role: HBM bytes for the
    transform/quantise kernels, operations and compulsory bytes for the GEMMs."""
    Lr = L // n * r if Lr is None else Lr
    cb = gx_bits / 8.0
    wb = gw_bits / 8.0
    return {
        "act_col_absmax": dict(bytes=4 * L * I),
        "act_col_quant": dict(bytes=4 * L * I + wb * Lr * I),
        "w_col_absmax": dict(bytes=4 * O * I),
        "w_col_quant": dict(bytes=4 * O * I + cb * O * I),
        "gy_row_quant": dict(bytes=4 * L * O + cb * L * O + 4 * L),
        "w_and_gy_row_quant": dict(bytes=4 * L * O + cb * L * O + 4 * L + 4 * O * I + cb * O * I),
        "gy_row_absmax": dict(bytes=4 * L * O),
        "gy_row_quant2": dict(bytes=4 * L * O + cb * L * O),
        "gyT_col_absmax": dict(bytes=4 * L * O),
        "gyT_col_quant": dict(bytes=4 * L * O + wb * Lr * O),
        "gy_fused_absmax": dict(bytes=4 * L * O + (4 * L * ((O + 127) // 128) if per_token else 0)),
        "gy_fused_quant": dict(bytes=4 * L * O + cb * L * O + Lr * O + 4 * L),
        "gx_igemm": dict(ops=2 * L * O * I, bytes=cb * (L * O + I * O) + 4 * L * I, peak=INT8_PEAK_TOPS),
        "gw_igemm": dict(ops=2 * O * I * Lr, bytes=wb * Lr * (O + I) + 4 * O * I,
                         peak=BF16_PEAK_TOPS if gw_bits == 16 else INT8_PEAK_TOPS),
    }


def kernel_entry(mdl, avg_us, launches_per_step):
    """One row of the per-kernel table.  A transform kernel is priced against the HBM peak.
    A GEMM is priced against whichever of its two lower bounds is the larger: operations at
    the matrix peak of its operand type, or compulsory bytes (operands once, output once) at
    the HBM peak: the g_x GEMM of a layer with few output features writes more fp32 output
    than its operations can cover."""
    k = dict(avg_us=round(avg_us, 3), launches_per_step=launches_per_step)
    if not mdl:
        return k
    t = avg_us * 1e-6
    k["GBps"] = round(mdl["bytes"] / t / 1e9, 1)
    if "ops" in mdl:
        k["TOPS"] = round(mdl["ops"] / t / 1e12, 2)
        t_mfma = mdl["ops"] / (mdl["peak"] * 1e12)
        t_hbm = mdl["bytes"] / (HBM_PEAK_GBS * 1e9)
        k["bound"] = "mfma" if t_mfma >= t_hbm else "hbm"
        k["frac"] = round(max(t_mfma, t_hbm) / t, 4)
        k["frac_mfma"] = round(t_mfma / t, 4)
        k["peak_TOPS"] = mdl["peak"]
    else:
        k["bound"] = "hbm"
        k["frac"] = round(k["GBps"] / HBM_PEAK_GBS, 4)
    return k


def profiled_traffic(workload, key):
    """HBM bytes per launch (fetched + written) of a kernel, from the committed rocprofv3
    counter summary of this workload (FETCH_SIZE / WRITE_SIZE runs, scaled by a copy of known
    size); (None, None) when no summary covers it."""
    rel = os.path.join("profiles", f"hbm_traffic_{workload}.txt")
    try:
        with open(os.path.join(ROOT, rel)) as fh:
            for line in fh:
                f = line.split()
                if len(f) == 4 and f[0] == "traffic_bytes" and f[1] == key:
                    return int(f[2]) + int(f[3]), rel
    except OSError:
        pass
    return None, None


class Job:
    """One workload with everything a step needs resident on the device."""

    def __init__(self, torch, hot, hot_inputs, wl, args):
        self.torch, self.hot, self.wl = torch, hot, wl
        n, r = wl.block, wl.keep
        self.cfg = hot.Config(block=n, keep=r, gw_bits=args.gw_bits, sample_tokens=args.sample_tokens)
        depth = int(wl.extra.get("depth", 0))
        self.chain = depth > 0
        self.layers = [(f"{d}.{l.name}", l) for d in range(depth) for l in wl.layers] if self.chain \
            else [(l.name, l) for l in wl.layers]
        cfg = self.cfg
        self.ws = torch.empty(max(hot.hot_workspace_bytes(cfg, l.L, l.O, l.I) for _, l in self.layers),
                              dtype=torch.uint8, device="cuda")
        self.x, self.w, self.gy, self.act, self.gx, self.gw, self.quant = [], [], [], [], [], [], []
        shared_out = {}
        for k, (name, l) in enumerate(self.layers):
            tag = f"{wl.name}.{name}"
            self.x.append(hot_inputs.make_x(wl.x_kind, l.L, l.I, 0, tag, "cuda"))
            self.w.append(hot_inputs.make_w(l.O, l.I, 0, tag, "cuda"))
            top = k == len(self.layers) - 1
            self.gy.append(hot_inputs.make_gy(wl.gy_kind, l.L, l.O, 0, tag, "cuda")
                           if (top or not self.chain) else None)
            self.act.append(hot.alloc_act_buffer(cfg, l.L, l.I))
            # outputs of layers of one shape share a buffer in a chain (a g_x is consumed by the
            # next call and nothing else), otherwise each layer has its own
            key = (l.L, l.O, l.I) if self.chain else k
            if key not in shared_out:
                shared_out[key] = (torch.empty((l.L, l.I), device="cuda"), torch.empty((l.O, l.I), device="cuda"))
            self.gx.append(shared_out[key][0])
            self.gw.append(shared_out[key][1])
            self.quant.append(args.quantizer or wl.quantizer)
        self.selected = {}
        for k, (name, l) in enumerate(self.layers):     # calibration, before training (Sec. 5.2.2)
            if self.quant[k] == "select":
                choice, m_tok, m_ten = hot.hot_select_quantizer(cfg, self.gy[k], self.ws)
                self.quant[k] = "token" if choice == hot.HOT_Q_PER_TOKEN else "tensor"
                self.selected[name] = dict(choice=self.quant[k], mse_token=m_tok, mse_tensor=m_ten)
        self.q = [hot.HOT_Q_PER_TOKEN if q == "token" else hot.HOT_Q_PER_TENSOR for q in self.quant]
        self.stream = torch.cuda.current_stream()
        self.ops = sum(2.0 * l.L * l.O * l.I + 2.0 * l.O * l.I * cfg.reduced_tokens(l.L) for _, l in self.layers)
        self.act_bytes = sum(a.numel() for a in self.act)
        self.fp32_bytes = sum(4 * l.L * l.I for _, l in self.layers)

    def compress(self, k):
        self.hot.hot_compress_activation(self.cfg, self.x[k], self.act[k], self.ws, stream=self.stream)

    def backward(self, k):
        g_y = self.gy[k] if self.gy[k] is not None else self.gx[k + 1]
        self.hot.hot_linear_backward(self.cfg, g_y, self.w[k], self.act[k], self.q[k], self.gx[k], self.gw[k],
                                     self.ws, stream=self.stream)

    def step(self):
        for k in range(len(self.layers)):
            self.compress(k)
        for k in range(len(self.layers) - 1, -1, -1):
            self.backward(k)

    def timed(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def timed_graph(self, steps, warmup):
        """The same step recorded once into a HIP graph (hot_config.replayable: launch tags from
        an epoch in the workspace, one more one-thread launch per call) and replayed: what a
        launch-bound step costs without the host's launch overhead.  ms per replay."""
        torch = self.torch
        eager_cfg = self.cfg
        self.cfg = self.hot.Config(block=eager_cfg.block, keep=eager_cfg.keep, gw_bits=eager_cfg.gw_bits,
                                   sample_tokens=eager_cfg.sample_tokens, replayable=True)
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                self.stream = side
                self.step()            # launch plans are made on first use
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                self.stream = torch.cuda.current_stream()
                self.step()
            torch.cuda.synchronize()
            for _ in range(warmup):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / steps
        finally:
            self.cfg = eager_cfg
            self.stream = torch.cuda.current_stream()

    def kernel_table(self, steps):
        """The same steps with HIP events around every kernel (recorded on the launch stream),
        one layer call at a time; kernels are keyed "<layer>.<role>", layers of a chain that
        share a shape pooled under the layer's name."""
        hot, cfg = self.hot, self.cfg
        acc = {}
        self.launch_sequence = []   # "<layer>.<role>" of every launch of one step, in order

        def take(lname, prof):
            for role, (ms, cnt) in prof.items():
                a = acc.setdefault((lname, role), [0.0, 0])
                a[0] += ms
                a[1] += cnt

        for step in range(steps):
            for k, (name, l) in enumerate(self.layers):
                hot.hot_debug_profile_begin()
                self.compress(k)
                take(name.split(".")[-1], hot.hot_debug_profile_end())
                if step == 0:
                    self.launch_sequence += [f"{name.split('.')[-1]}.{r}" for r in hot.hot_debug_profile_sequence()]
            for k in range(len(self.layers) - 1, -1, -1):
                hot.hot_debug_profile_begin()
                self.backward(k)
                take(self.layers[k][0].split(".")[-1], hot.hot_debug_profile_end())
                if step == 0:
                    lname = self.layers[k][0].split(".")[-1]
                    self.launch_sequence += [f"{lname}.{r}" for r in hot.hot_debug_profile_sequence()]
        shapes = {name.split(".")[-1]: (l, self.quant[k]) for k, (name, l) in enumerate(self.layers)}
        table = {}
        for (lname, role), (ms, cnt) in acc.items():
            l, quant = shapes[lname]
            mdl = stage_model(l.L, l.O, l.I, cfg.block, cfg.keep, cfg.gx_bits, quant == "token", cfg.gw_bits,
                              cfg.reduced_tokens(l.L)).get(role)
            e = kernel_entry(mdl, ms * 1e3 / cnt, cnt / steps)
            e["step_us"] = round(ms * 1e3 / steps, 1)
            if mdl:
                e["algorithmic_bytes"] = int(mdl["bytes"])
                if "ops" in mdl:
                    e["algorithmic_ops"] = int(mdl["ops"])
            table[f"{lname}.{role}"] = e
        return table

    def layer_table(self):
        """Per-layer times of one more step (HIP events around each call) and output sanity."""
        torch = self.torch
        ev = lambda: torch.cuda.Event(enable_timing=True)
        rows = {}
        marks = []
        for k in range(len(self.layers)):
            e0, e1 = ev(), ev()
            e0.record()
            self.compress(k)
            e1.record()
            marks.append((k, "compress_us", e0, e1))
        for k in range(len(self.layers) - 1, -1, -1):
            e0, e1 = ev(), ev()
            e0.record()
            self.backward(k)
            e1.record()
            marks.append((k, "backward_us", e0, e1))
        torch.cuda.synchronize()
        for k, what, e0, e1 in marks:
            lname = self.layers[k][0].split(".")[-1]
            row = rows.setdefault(lname, dict(layers=0, compress_us=0.0, backward_us=0.0))
            row[what] += e0.elapsed_time(e1) * 1e3
            if what == "compress_us":
                row["layers"] += 1
        out = {}
        for lname, row in rows.items():
            l = next(l for name, l in self.layers if name.split(".")[-1] == lname)
            quant = next(self.quant[k] for k, (name, _) in enumerate(self.layers) if name.split(".")[-1] == lname)
            ops = 2.0 * l.L * l.O * l.I + 2.0 * l.O * l.I * self.cfg.reduced_tokens(l.L)
            bw = row["backward_us"] / row["layers"]
            out[lname] = dict(L=l.L, O=l.O, I=l.I, layers=row["layers"], gy_quantizer=quant,
                              compress_us=round(row["compress_us"] / row["layers"], 1),
                              backward_us=round(bw, 1), backward_TOPS=round(ops / bw / 1e6, 1))
        finite = all(bool(torch.isfinite(t).all().item()) for t in set(self.gx) | set(self.gw))
        return out, finite


def summarise(job, ms_per_step, table, layers, finite, torch):
    cfg, wl = job.cfg, job.wl
    out = dict(workload=wl.name, layers_per_step=len(job.layers), us_per_step=round(ms_per_step * 1e3, 2),
               effective_TOPS=round(job.ops / (ms_per_step * 1e-3) / 1e12, 2),
               block=cfg.block, keep=cfg.keep, gx_bits=cfg.gx_bits, gw_bits=cfg.gw_bits,
               act_buffer_bytes=job.act_bytes, act_fp32_bytes=job.fp32_bytes,
               act_ratio=round(job.act_bytes / job.fp32_bytes, 4),
               peak_device_bytes=int(torch.cuda.max_memory_allocated()),
               outputs_finite=finite, layers=layers, kernels=table, launch_sequence=job.launch_sequence)
    if job.selected:
        out["select_quantizer"] = job.selected
    return out


def pick_roofline(workload, table):
    """The kernel the roofline object describes: among the kernels whose average launch is
    within 10 % of the longest one, the one with the lowest fraction of its bound."""
    priced = {k: v for k, v in table.items() if "frac" in v}
    longest = max(v["avg_us"] for v in priced.values())
    key = min((k for k, v in priced.items() if v["avg_us"] >= 0.9 * longest), key=lambda k: priced[k]["frac"])
    d = priced[key]
    traffic, source = profiled_traffic(workload, key)
    if d["bound"] == "hbm":
        roof = dict(kernel=key, bound="hbm", achieved=d["GBps"], peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=d["frac"], traffic=traffic, algorithmic_bytes=d["algorithmic_bytes"], avg_us=d["avg_us"])
    else:
        roof = dict(kernel=key, bound="mfma", achieved=d["TOPS"], peak=d["peak_TOPS"], unit="TOP/s",
                    frac=d["frac"], traffic=traffic, algorithmic_ops=d["algorithmic_ops"], avg_us=d["avg_us"])
    if traffic is not None:
        roof["traffic_source"] = f"{source} (rocprofv3 counter runs of an earlier session, not of this run)"
    return roof


def run_sweep(torch, hot, hot_inputs, wl, quantizer_flag):
    """Streamed form of one step, for the peak-memory figure: inputs are generated layer by
    layer and only what the backward needs (the compressed activations) is kept.
    Returns per-layer times (HIP events), buffer bytes and peak memory."""
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
        out[f"hbm_write_streaming_hint_GBps_{mb}MB"] = round(nbytes / timed(4, buf, 1, 10) / 1e9, 1)
        del buf
    buf = torch.zeros(1 << 20, dtype=torch.int32, device="cuda")
    iters = 4000
    ops = 2.0 * 32 * 32 * 32 * 16 * iters * 256 * 4
    out["mfma_i8_TOPS_constant_operands"] = round(ops / timed(2, buf, iters, 3) / 1e12, 1)
    out["mfma_i8_TOPS_random_operands"] = round(ops / timed(3, buf, iters, 6) / 1e12, 1)

    # What a streaming read costs right behind another kernel: behind a 1 GB write (whose tail
    # is still on its way from the memory-side cache to HBM), a 50 MB write, a 1 GB read and a
    # register-only matrix loop of about 0.5 ms.  Median of 8, the read alone timed.
    a = torch.zeros(1000 * 1000 * 1000 // 4, dtype=torch.float32, device="cuda")
    b = torch.zeros(1000 * 1000 * 1000 // 4, dtype=torch.float32, device="cuda")
    nbytes = a.numel() * 4 - 4096
    before = {"idle": None, "read_1GB": (0, b, 1), "write_1GB": (1, b, 1),
              "write_50MB": (1, b[:50 * 1000 * 1000 // 4], 1), "matrix_loop": (3, buf, 1500)}
    for name, pre in before.items():
        ts = []
        for _ in range(8):
            torch.cuda.synchronize()
            time.sleep(0.01)
            if pre is not None:
                hot.hot_debug_probe(*pre)
            ev0.record()
            hot.hot_debug_probe(0, a, 1)
            ev1.record()
            torch.cuda.synchronize()
            ts.append(ev0.elapsed_time(ev1) * 1e-3)
        out[f"hbm_read_GBps_1GB_behind_{name}"] = round(nbytes / sorted(ts)[len(ts) // 2] / 1e9, 1)
    return out


def cpu_baseline(job, seconds, sample_tokens):
    """The oracle, as it stands, on a bounded sample of the workload: the first tokens of one
    layer of every shape (compress + g_x + g_w), repeated for about `seconds` of wall time."""
    import oracle
    oracle.lib()
    cfg, n, r = job.cfg, job.cfg.block, job.cfg.keep
    seen, sample = set(), []
    for k in range(len(job.layers) - 1, -1, -1):
        name, l = job.layers[k]
        if (l.O, l.I) in seen:
            continue
        seen.add((l.O, l.I))
        if cfg.sample_tokens:     # the oracle's per-sample definition: zero tokens after every sample
            Ls = l.L
        else:
            Ls = l.L if sample_tokens <= 0 else min(l.L, max(n, sample_tokens // n * n))
        gy = job.gy[k] if job.gy[k] is not None else job.gx[k + 1]
        sample.append((name, l, Ls, job.x[k][:Ls].cpu().numpy(), gy[:Ls].cpu().numpy(), job.w[k].cpu().numpy(),
                       job.quant[k] == "token"))
    reps, dt, ops = 0, 0.0, 0.0
    while reps < 1 or (dt < seconds and reps < 64):
        t0 = time.perf_counter()
        for name, l, Ls, xs, gys, wh, per_token in sample:
            oracle.backward_gx(gys, wh, n, bits=cfg.gx_bits, per_token=per_token, taps=False)
            if cfg.sample_tokens:
                xs_t, gys_t = oracle.pad_samples(xs, cfg.sample_tokens, n), oracle.pad_samples(gys, cfg.sample_tokens, n)
            else:
                xs_t, gys_t = xs, gys
            if cfg.gw_bits == 16:
                oracle.backward_gw_bf16(gys_t, oracle.compress_activation_bf16(xs_t, n, r), n, r)
            else:
                codes, sx = oracle.compress_activation(xs_t, n, r)
                oracle.backward_gw(gys_t, codes, sx, n, r, taps=False)
        dt += time.perf_counter() - t0
        reps += 1
    ops = sum(2.0 * Ls * l.O * l.I + 2.0 * l.O * l.I * cfg.reduced_tokens(Ls) for _, l, Ls, *_ in sample)
    what = ", ".join(f"{'all' if Ls == l.L else 'first ' + str(Ls) + ' of'} {l.L} tokens of {name} ({l.O}x{l.I})"
                     for name, l, Ls, *_ in sample)
    return dict(value=round(ops * reps / dt / 1e12, 6), unit="TOPS", cores=oracle.threads(), kind="oracle",
                sample=f"{job.wl.name}: {what}; compress + g_x + g_w of each, {reps} passes in {dt:.1f} s; the "
                       f"oracle's rate on the sample stands for its rate on the whole step (cost is linear in tokens)",
                seconds_per_pass=round(dt / reps, 3))


def run_job(torch, hot, hot_inputs, wl, args, want_cpu):
    torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    job = Job(torch, hot, hot_inputs, wl, args)
    ms = job.timed(args.steps, args.warmup)
    # a step recorded into a HIP graph and replayed, for the workloads where launches matter
    ms_graph, graph_error = None, None
    if len(job.layers) <= 4 and ms < 5.0:
        try:
            ms_graph = job.timed_graph(args.steps, args.warmup)
        except Exception as e:      # context figure only: never lose the measurement over it
            graph_error = f"{type(e).__name__}: {e}"[:200]
            torch.cuda.synchronize()
    table = job.kernel_table(max(1, min(args.steps, 5 if len(job.layers) > 8 else 20)))
    layers, finite = job.layer_table()
    res = summarise(job, ms, table, layers, finite, torch)
    if ms_graph is not None:
        res["graph_replay_us_per_step"] = round(ms_graph * 1e3, 2)
    if graph_error is not None:
        res["graph_replay_error"] = graph_error
    cpu = None
    if want_cpu:
        cpu = cpu_baseline(job, args.cpu_seconds, args.cpu_sample_tokens or (16384 if len(job.layers) > 1 else 0))
    del job
    return res, ms, cpu


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    help="run this workload only (default: the ViT-L chain as the headline and the four "
                         "smaller configurations under 'workloads')")
    ap.add_argument("--quantizer", default=None, choices=[None, "token", "tensor"])
    ap.add_argument("--cpu-sample-tokens", type=int, default=0,
                    help="tokens per layer the oracle is timed on (0 = 16384 for multi-layer workloads, "
                         "all tokens for single layers)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="repeat the oracle on the sample until about this much CPU wall time")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--backward", default="auto", choices=list(STRATEGY),
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
                    help="instead of the timed steps, run the streamed form of one step (inputs generated "
                         "layer by layer) and print per-layer times, buffer bytes and peak memory as JSON")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of 154.9 MB (for scaling rocprofv3 byte counters)")
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
    hot.hot_debug_set_gemm_mode(args.gemm)
    hot.hot_debug_set_backward_strategy(STRATEGY[args.backward])
    if args.sweep:
        wl = hot_inputs.WORKLOADS[args.workload or HEADLINE]
        run_sweep(torch, hot, hot_inputs, wl, args.quantizer)   # warm-up: code objects, allocator
        print(json.dumps(run_sweep(torch, hot, hot_inputs, wl, args.quantizer)))
        return 0
    if args.calibrate_copy:
        a = torch.empty(12608 * 3072, device="cuda")
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    head_wl = hot_inputs.WORKLOADS[args.workload or HEADLINE]
    others = {}
    streamed_peak = None
    if args.workload is None:
        # the peak-memory figure of the headline: a streamed step, before its inputs are made resident
        streamed_peak = run_sweep(torch, hot, hot_inputs, head_wl, args.quantizer)["peak_device_bytes"]
        for name in OTHERS:
            res, _, _ = run_job(torch, hot, hot_inputs, hot_inputs.WORKLOADS[name], args, False)
            others[name] = res
    head, ms_per_step, cpu = run_job(torch, hot, hot_inputs, head_wl, args, not args.no_cpu_baseline)
    roof = pick_roofline(head_wl.name, head["kernels"])

    cfg = hot.Config(block=head_wl.block, keep=head_wl.keep, gw_bits=args.gw_bits, sample_tokens=args.sample_tokens)
    out = {
        "metric": "HOT linear-backward effective TOPS (integer ops executed / step time)",
        "value": head["effective_TOPS"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "us_per_step": head["us_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8" if cfg.gw_bits == 8 else "int8 (g_x) + bf16 (g_w)",
        "data": "synthetic",
        "config": {"workload": head_wl.name, "layers_per_step": head["layers_per_step"],
                   "layers": {k: [v["L"], v["O"], v["I"]] for k, v in head["layers"].items()},
                   "block": cfg.block, "keep": cfg.keep, "gx_bits": cfg.gx_bits, "gw_bits": cfg.gw_bits,
                   "gy_quantizer": {k: v["gy_quantizer"] for k, v in head["layers"].items()},
                   "sample_tokens": cfg.sample_tokens,
                   "step": "compress_activation of every layer, then linear_backward (g_x and g_w) of every layer, "
                           "top first%s; g_y views: %s; GEMM work distribution: %s"
                           % (" (each g_x is the next g_y)" if head_wl.extra.get("depth") else "", args.backward,
                              {0: "auto", 1: "tile"}.get(args.gemm, "K split %d" % args.gemm))},
        "act_buffer_bytes": head["act_buffer_bytes"], "act_fp32_bytes": head["act_fp32_bytes"],
        "peak_device_bytes": head["peak_device_bytes"],
        "peak_device_bytes_streamed": streamed_peak,
        "outputs_finite": head["outputs_finite"],
        "roofline": roof, "cpu_baseline": cpu, "layers": head["layers"], "kernels": head["kernels"],
        "launch_sequence": head["launch_sequence"],
    }
    if "select_quantizer" in head:
        out["select_quantizer"] = head["select_quantizer"]
    if "graph_replay_us_per_step" in head:
        out["graph_replay_us_per_step"] = head["graph_replay_us_per_step"]
    if others:
        out["workloads"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
