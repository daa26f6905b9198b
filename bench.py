#!/usr/bin/env python3
"""Benchmark of the residual-expanded quantized layer on one MI355X.

A step is one pass of the whole hot path -- activation quantization, integer
contraction over all kept rows of all K orders, de-quantizing epilogue, member
sum -- over one batch of synthetic input that is already resident in HBM (the
expansion itself is built once, offline, before the timed region).

Prints ONE JSON line.  `value` is effective integer TOPS of the headline
workload (2*T*in*(stored rows) / step time); `sweep` adds the other token counts
of the same layer and the decode-sized HBM roofline; `cpu_baseline` is the CPU
checker timed on a bounded sample of the same workload on this machine's host cores.
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

# Kernel arguments in device memory (a switch of the HIP runtime, read when it is loaded, i.e. before
# torch is imported): with the default, host-resident arguments, every eagerly launched kernel spends
# about 3 us fetching them before its first instruction (the 16-token contraction: 15.2 us against
# 11.8 us between its start and stop events).  Kernels replayed from a HIP graph do not pay this.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

INT8_MFMA_PEAK_TOPS = 5000.0    # MI355X dense int8, vendor figure (5.0 POP/s)
HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, vendor figure (8 TB/s)
LLC_BYTES = 256 << 20           # Infinity Cache: rotate over more expansion bytes than this

# HBM-side bytes per step of the contraction launches come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this script (each counter scaled by what it reads for a 1 GiB device copy).  Counters cannot
# be read from inside this process: the figures live in profiles/hbm_traffic.txt, next to the summaries
# they were taken from, one line "workload tokens fetch_bytes write_bytes" per profiled workload.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic():
    out = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                line = line.split("#", 1)[0].split()
                if len(line) == 4:
                    out[(line[0], int(line[1]))] = float(line[2]) + float(line[3])
    except OSError:
        pass
    return out


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="untimed steps run for this long before the warm-up steps of every measurement: the chip "
                         "raises its clocks only under sustained load (the 4096-token kernel takes 235 us in the first "
                         "milliseconds after an idle period and 205 us from about 25 ms on)")
    ap.add_argument("--workload", default="c4",
                    help="c4 (LLM-7B linear, ternary K=4) | c5 (gated MLP, int4 K=4) | c3 | c2 | c1 | "
                         "chain (residual stack of 8 layers, ternary K=8, as member chains) | "
                         "stack (decode stack: 8 layers of the c4 shape, 11008x4096 and back, as one chain)")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the rows of the other workloads (c5 at 1, 16, 4096 tokens; the decode stack at 1, 16)")
    ap.add_argument("--resident", type=int, default=1,
                    help="decode-sized chains as one resident launch: 0 never, 1 automatic, 2 whenever possible")
    ap.add_argument("--tokens", type=int, default=0, help="override the headline token count")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 tiled MFMA, 2 weight streaming")
    ap.add_argument("--token-tile", type=int, default=0,
                    help="token-tile height of the tiled kernel: 16, 32, 64 (0 = automatic)")
    ap.add_argument("--stream-split", type=int, default=0,
                    help="workgroups per bin of the weight-streaming kernel (0 = automatic)")
    ap.add_argument("--no-graph", action="store_true", help="time the steps eagerly instead of as one HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a 1 GiB device copy 5 times (reference for the FETCH_SIZE/WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
              "(no collectives or sharding are part of it)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2311_15806_amd import workloads as wl
    import paper_2311_15806_amd.binding as pipe   # raises if the HIP library is missing

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    pipe.pipe_set_kernel(args.kernel)
    pipe.pipe_set_stream_split(args.stream_split)
    pipe.pipe_set_token_tile(args.token_tile)
    pipe.pipe_set_decode_resident(args.resident)
    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB
        b = torch.empty_like(a)
        a.fill_(1.0)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": a.numel() * 4, "calibrate_copy_bytes_written": a.numel() * 4}))
        return

    WORKLOADS = {"c1": wl.C1, "c2": wl.C2, "c3": wl.C3, "c4": wl.C4, "c5": wl.C5, "chain": wl.CHAIN, "stack": wl.DECODE_STACK}
    chain_act = {"none": pipe.PIPE_ACT_NONE, "relu": pipe.PIPE_ACT_RELU, "gelu": pipe.PIPE_ACT_GELU}
    traffic = measured_traffic()

    class Runner:
        """One workload: its expansions (built once, offline step a0; further copies for rotation), input, step."""

        def __init__(self, name):
            self.name = name
            cfg = self.cfg = WORKLOADS[name]
            t0 = time.time()
            # the decode stack repeats two shapes: the layers share the two fp32 weights, every layer has
            # its own expansion (its own codes in HBM)
            n_w = 2 if name == "stack" else len(cfg.layers)
            self.Ws = [torch.from_numpy(wl.make_weight(cfg, i)).to(dev) for i in range(n_w)]
            torch.cuda.synchronize()
            t1 = time.time()
            self.exps = [self.build()]
            torch.cuda.synchronize()
            self.expand_s = time.time() - t1
            self.gen_s = t1 - t0
            self.stream_bytes = sum(e.packed_bytes for e in self.exps[0])
            self.macs_per_token = sum(e.macs_per_token() for e in self.exps[0])
            self.T_max = cfg.tokens if cfg.kind == "conv2d" else (16 if name == "stack" else 4096)
            self.x_full = wl.make_input(cfg if cfg.kind == "conv2d" else wl.with_tokens(cfg, self.T_max))
            self.xd_full = torch.from_numpy(self.x_full).to(dev)
            self.split = list(cfg.split) if len(cfg.split) > 1 else None
            self.static_sx = 0.0   # > 0: the activation scale is given (the paper's static ranges) instead of max|x| / 127
            self.given = None      # chain: per layer the given scales of the tensors entering it (static ranges), or None

        def build(self):
            cfg = self.cfg
            if cfg.kind == "conv2d":       # the convolution as an implicit GEMM: the expansion is stored tap-major
                c, l = cfg.conv, cfg.layers[0]
                return [pipe.pipe_expand_conv2d(self.Ws[0], c["C"], c["kh"], c["kw"], l.bits, l.K, l.gamma, l.group)]
            return [pipe.pipe_expand(self.Ws[i % len(self.Ws)], l.bits, l.K, l.gamma, l.group) for i, l in enumerate(cfg.layers)]

        def free(self):
            for es in self.exps:
                for e in es:
                    e.free()
            self.exps = []

        def step_fn(self, e, xd, out=None, split="default"):
            cfg = self.cfg
            split = self.split if split == "default" else split
            if cfg.kind == "linear" and self.static_sx > 0:
                return pipe.pipe_forward(e[0], xd, s_x=self.static_sx, split=split, out=out)
            if cfg.kind == "chain":
                if self.given is not None:
                    layers = [(e[i], None, chain_act[c[0]], c[1], c[2], 0, 0, 1, 0, self.given[i]) for i, c in enumerate(cfg.chain)]
                    return pipe.pipe_chain_forward(layers, xd, s_x=self.static_sx, split=split, out=out)
                layers = [(e[i], None, chain_act[c[0]], c[1], c[2]) for i, c in enumerate(cfg.chain)]
                return pipe.pipe_chain_forward(layers, xd, split=split, out=out)
            if cfg.kind == "linear":
                return pipe.pipe_forward(e[0], xd, split=split, out=out)
            if cfg.kind == "conv2d":
                c = cfg.conv
                return pipe.pipe_forward_conv2d(e[0], xd, c["kh"], c["kw"], c["stride"], c["pad"], split=split, out=out)
            act = pipe.PIPE_ACT_GELU if cfg.kind == "mlp_gelu" else pipe.PIPE_ACT_SILU_GATED
            if self.given is not None:
                return pipe.pipe_mlp_forward_given_scales(e[0], e[1], act, xd, self.static_sx, self.given, split=split, out=out)
            return pipe.pipe_mlp_forward(e[0], e[1], act, xd, split=split, out=out)

        def io_bytes(self, T):
            """Bytes the contraction launches of one step must move besides the packed codes:
            int8 activations in, fp32 results out (hidden activations of an MLP: out and back in)."""
            cfg = self.cfg
            M = len(self.split) if self.split else 1
            b = 0
            for i, l in enumerate(cfg.layers):
                last = i == len(cfg.layers) - 1
                b += T * l.in_features * (1 if i == 0 else M)
                b += 4 * T * l.out_features * (1 if last else M)
                if cfg.chain is not None and cfg.chain[i][1] >= 0:     # the skip tensor is read once more
                    b += 4 * T * l.out_features * (1 if cfg.chain[i][1] == 0 else M)
            return b

        def measure(self, T, steps, warmup, rotate, settle_ms=None, graph=True):
            """Times `steps` passes; returns dict with step time and contraction-kernel time."""
            cfg, exps = self.cfg, self.exps
            settle_ms = args.settle_ms if settle_ms is None else settle_ms
            xd = self.xd_full if cfg.kind == "conv2d" else self.xd_full[:T].contiguous()
            out = torch.empty((T, cfg.layers[-1].out_features), dtype=torch.float32, device=dev)
            copies = 1
            if rotate:
                copies = max(2, -(-int(1.25 * LLC_BYTES) // max(self.stream_bytes, 1)))
                while len(exps) < copies:
                    exps.append(self.build())
            step_fn = self.step_fn
            # sustained load first (clocks settle), then the W warm-up steps
            t_s, i_s = time.perf_counter(), 0
            while (time.perf_counter() - t_s) * 1e3 < settle_ms:
                for _ in range(8):
                    step_fn(exps[i_s % copies], xd, out)
                    i_s += 1
                torch.cuda.synchronize()
            for i in range(warmup):
                step_fn(exps[i % copies], xd, out)
            torch.cuda.synchronize()
            # ---- K steps, eager, contraction kernels bracketed by events on the launch stream ----
            pipe.pipe_timing_read()
            pipe.pipe_timing_enable(True)
            torch.cuda.synchronize()
            t_a = time.perf_counter()
            for i in range(steps):
                step_fn(exps[i % copies], xd, out)
            torch.cuda.synchronize()
            t_b = time.perf_counter()
            pipe.pipe_timing_enable(False)
            k_ms, k_n = pipe.pipe_timing_read()
            step_ms = (t_b - t_a) * 1e3 / steps
            mode = "eager"
            # a resident launch whose wait for other workgroups ran out ends with wrong results: no figure from such a run
            if pipe.pipe_resident_status() != 0:
                raise RuntimeError("a resident launch ran into its wait limit: the timings of this run are void")
            # ---- the same K steps as ONE HIP graph: decode-sized steps are launch bound, and the small
            # layers' five launches leave gaps as long as their kernels when launched eagerly --------
            if graph and not args.no_graph:
                try:
                    side = torch.cuda.Stream()
                    side.wait_stream(torch.cuda.current_stream())
                    with torch.cuda.stream(side):          # the library keeps its scratch per stream: warm the capture stream
                        for i in range(max(2, copies)):
                            step_fn(exps[i % copies], xd, out)
                    torch.cuda.current_stream().wait_stream(side)
                    torch.cuda.synchronize()
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side):
                        for i in range(steps):
                            step_fn(exps[i % copies], xd, out)
                    t_s = time.perf_counter()      # capture left the chip idle: load it again before the timed replay
                    g.replay()
                    torch.cuda.synchronize()
                    while (time.perf_counter() - t_s) * 1e3 < settle_ms:
                        g.replay()
                        torch.cuda.synchronize()
                    t_a = time.perf_counter()
                    g.replay()
                    torch.cuda.synchronize()
                    t_b = time.perf_counter()
                    with torch.cuda.stream(side):
                        if pipe.pipe_resident_status() != 0:
                            raise RuntimeError("a resident launch of the graph ran into its wait limit")
                    step_ms = (t_b - t_a) * 1e3 / steps
                    mode = "hipgraph"
                except Exception as ex:      # keep the eager number
                    mode = "eager (graph capture failed: %s)" % type(ex).__name__
            per_step_kernel_ms = k_ms / steps
            ops = 2.0 * T * self.macs_per_token
            alg_bytes = self.stream_bytes + self.io_bytes(T)
            return dict(tokens=T, ms_per_step=step_ms, kernel_ms_per_step=per_step_kernel_ms,
                        kernel_launches_per_step=k_n / steps, step_mode=mode,
                        eff_tops=ops / (step_ms * 1e-3) / 1e12,
                        kernel_eff_tops=ops / (per_step_kernel_ms * 1e-3) / 1e12 if k_ms > 0 else None,
                        tokens_per_s=T / (step_ms * 1e-3),
                        kernel_gbs=alg_bytes / (per_step_kernel_ms * 1e-3) / 1e9 if k_ms > 0 else None,
                        step_gbs=alg_bytes / (step_ms * 1e-3) / 1e9,
                        alg_bytes=alg_bytes, expansion_copies=copies)

    def fractions(r):
        """Roofline fractions of a row: the contraction kernels alone and the whole step."""
        r["mfma_frac"] = (r["kernel_eff_tops"] or 0) / INT8_MFMA_PEAK_TOPS
        r["hbm_frac"] = (r["kernel_gbs"] or 0) / HBM_PEAK_GBS
        r["step_mfma_frac"] = r["eff_tops"] / INT8_MFMA_PEAK_TOPS
        r["step_hbm_frac"] = r["step_gbs"] / HBM_PEAK_GBS
        return {k: (round(v, 6) if isinstance(v, float) else v) for k, v in r.items()}

    run = Runner(args.workload)
    cfg, Ws, exps = run.cfg, run.Ws, run.exps
    x_full, xd_full, split = run.x_full, run.xd_full, run.split
    stream_bytes, macs_per_token, expand_s, gen_s = run.stream_bytes, run.macs_per_token, run.expand_s, run.gen_s
    T_head = args.tokens or cfg.tokens
    measure, step_fn = run.measure, run.step_fn

    T0 = cfg.tokens if cfg.kind == "conv2d" else T_head
    # the same workload from an idle chip first (no sustained load before it, 5 warm-up steps, 50
    # eager steps): what a burst after an idle period sees, reported next to the settled figure
    cold = measure(T0, min(50, args.steps), min(5, args.warmup), rotate=(T0 <= 128), settle_ms=0.0, graph=False)
    head = measure(T0, args.steps, args.warmup, rotate=(T0 <= 128))

    # the same step with a given activation scale (Sec. 4.1: the paper quantizes activations with static
    # ranges): no max|x| reduction in the step.  Reported next to the headline, which keeps the dynamic scale.
    static = None
    if cfg.kind == "linear":
        run.static_sx = float(xd_full[:T0].abs().max().item()) / 127.0
        r = measure(T0, args.steps, args.warmup, rotate=(T0 <= 128))
        run.static_sx = 0.0
        static = {"ms_per_step": r["ms_per_step"], "eff_tops": r["eff_tops"], "tokens_per_s": r["tokens_per_s"],
                  "step_mode": r["step_mode"]}

    # the dominant kernel's roofline (its own launch duration) and, next to it, the same figure over
    # the whole step (activation quantization included)
    mfma_bound = T0 > 128
    one_launch = head["kernel_launches_per_step"] <= 1.0 and cfg.kind in ("chain", "mlp_gelu", "mlp_gated") and T0 <= 16
    if mfma_bound:
        roofline = dict(bound="mfma", achieved=head["kernel_eff_tops"], peak=INT8_MFMA_PEAK_TOPS, unit="TOP/s",
                        frac=(head["kernel_eff_tops"] or 0) / INT8_MFMA_PEAK_TOPS, traffic=None,
                        kernel="gemm_tiled_kernel", kernel_ms=head["kernel_ms_per_step"],
                        step_achieved=head["eff_tops"], step_frac=head["eff_tops"] / INT8_MFMA_PEAK_TOPS)
    else:
        roofline = dict(bound="hbm", achieved=head["kernel_gbs"], peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=(head["kernel_gbs"] or 0) / HBM_PEAK_GBS, traffic=None,
                        kernel=("chain_resident_kernel" if one_launch else
                                "gemm_stream_kernel" if cfg.layers[0].K <= 4 else "gemm_stream_multi_kernel"),
                        kernel_ms=head["kernel_ms_per_step"],
                        step_achieved=head["step_gbs"], step_frac=head["step_gbs"] / HBM_PEAK_GBS)

    roofline["traffic"] = traffic.get((args.workload, T0))
    roofline["algorithmic_bytes"] = head["alg_bytes"]

    sweep = []
    if not args.no_sweep and cfg.kind not in ("conv2d", "chain"):
        for T in (1, 16, 64, 256, 2048, 4096):
            if T == T0:
                r = dict(head)
            else:
                r = measure(T, max(10, args.steps // 2), 3, rotate=(T <= 128))
            if T <= 128:
                # same batch with ONE expansion copy: codes stay in the Infinity Cache between steps
                rr = measure(T, max(10, args.steps // 2), 3, rotate=False)
                r["resident_ms_per_step"] = rr["ms_per_step"]
                r["resident_kernel_ms_per_step"] = rr["kernel_ms_per_step"]
                r["resident_kernel_gbs"] = rr["kernel_gbs"]
            sweep.append(fractions(r))

    # ---- the other workloads' rows: the largest config (gated MLP) at decode and prefill sizes, and the
    # decode stack (8 layers of this run's headline shape in one chain), each with both rooflines
    extra = []
    if not args.no_extra and not args.no_sweep and args.workload == "c4":
        for name, tokens in (("c5", (1, 16, 4096)), ("stack", (1, 16))):
            other = Runner(name)
            for T in tokens:
                r = other.measure(T, max(10, args.steps // 2), 3, rotate=(T <= 128))
                r["workload"] = other.cfg.name
                r["traffic"] = traffic.get((name, T))
                if other.cfg.kind == "chain":
                    # the same step with the paper's static activation ranges: every layer's input scale is given
                    # (here: the scales the dynamic run found), so no maxima are exchanged between the layers
                    xd = other.xd_full[:T].contiguous()
                    layers = [(other.exps[0][i], None, chain_act[c[0]], c[1], c[2]) for i, c in enumerate(other.cfg.chain)]
                    _, acts = pipe.pipe_chain_forward(layers, xd, split=other.split, return_acts=True)
                    other.given = [None] + [[float(a[m].abs().max().item()) / 127.0 for m in range(a.shape[0])] for a in acts]
                    other.static_sx = float(xd.abs().max().item()) / 127.0
                    rs = other.measure(T, max(10, args.steps // 2), 3, rotate=True)
                    other.given, other.static_sx = None, 0.0
                    r["static_ranges"] = {"ms_per_step": rs["ms_per_step"], "kernel_ms_per_step": rs["kernel_ms_per_step"],
                                          "step_gbs": rs.get("step_gbs"), "hbm_frac": (rs.get("step_gbs") or 0.0) / HBM_PEAK_GBS}
                elif other.cfg.kind in ("mlp_gelu", "mlp_gated") and T <= 128:
                    xd = other.xd_full[:T].contiguous()
                    act = pipe.PIPE_ACT_GELU if other.cfg.kind == "mlp_gelu" else pipe.PIPE_ACT_SILU_GATED
                    _, hh = pipe.pipe_mlp_forward(other.exps[0][0], other.exps[0][1], act, xd, split=other.split, return_hidden=True)
                    other.given = [float(hh[m].abs().max().item()) / 127.0 for m in range(hh.shape[0])]
                    other.static_sx = float(xd.abs().max().item()) / 127.0
                    rs = other.measure(T, max(10, args.steps // 2), 3, rotate=True)
                    other.given, other.static_sx = None, 0.0
                    r["static_ranges"] = {"ms_per_step": rs["ms_per_step"], "kernel_ms_per_step": rs["kernel_ms_per_step"],
                                          "step_gbs": rs.get("step_gbs"), "hbm_frac": (rs.get("step_gbs") or 0.0) / HBM_PEAK_GBS}
                extra.append(fractions(r))
            other.free()
            del other
            torch.cuda.empty_cache()

    # ---- the run-time comparison of the ensembles (a chain workload only): the same network and
    # the same K under the groupings of the paper's run-time table, and the unexpanded K = 1 net
    ensemble_ms = None
    if cfg.kind == "chain" and not args.no_sweep:
        ensemble_ms = {}
        xd = xd_full[:T0].contiguous()
        out_t = torch.empty((T0, cfg.layers[-1].out_features), dtype=torch.float32, device=dev)
        K = cfg.layers[0].K

        def timed(e, sp):
            t_s = time.perf_counter()
            while (time.perf_counter() - t_s) * 1e3 < args.settle_ms:      # sustained load first, as in measure()
                for _ in range(4):
                    step_fn(e, xd, out_t, split=sp)
                torch.cuda.synchronize()
            for _ in range(3):
                step_fn(e, xd, out_t, split=sp)
            torch.cuda.synchronize()
            n_it = max(10, args.steps // 2)
            pipe.pipe_timing_read()
            pipe.pipe_timing_enable(True)
            ta = time.perf_counter()
            for _ in range(n_it):
                step_fn(e, xd, out_t, split=sp)
            torch.cuda.synchronize()
            tb = time.perf_counter()
            pipe.pipe_timing_enable(False)
            k_ms, _ = pipe.pipe_timing_read()
            return {"ms_per_step": round((tb - ta) * 1e3 / n_it, 4), "contraction_ms_per_step": round(k_ms / n_it, 4)}

        groupings = [[K]]
        if K % 2 == 0:
            groupings.append([K // 2] * 2)
        if K >= 3:
            groupings.append([-(-K // 3)] * (K % 3 or 3) + [K // 3] * (3 - (K % 3 or 3)) if K % 3 else [K // 3] * 3)
        if K % 4 == 0:
            groupings.append([K // 4] * 4)
        for sp in groupings:
            ensemble_ms[str(sp)] = timed(exps[0], sp if len(sp) > 1 else None)
        e1 = [pipe.pipe_expand(Ws[i], l.bits, 1, l.gamma, l.group) for i, l in enumerate(cfg.layers)]
        ensemble_ms["[1] (K = 1, no expansion)"] = timed(e1, None)
        for e in e1:
            e.free()

    # ---- CPU checker on a bounded sample of the same workload ------------------------------
    cpu = None
    if not args.no_cpu:
        from oracle import pipe_oracle as po
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        O_s = cfg.layers[0].out_features
        l0 = cfg.layers[0]
        if cfg.kind == "linear" or args.workload == "stack":
            T_s = min(T0, 4096)
            Wn = Ws[0][:O_s].cpu().numpy()
            ex = po.expand(Wn, l0.bits, l0.K, l0.gamma, l0.group)
            xs = x_full[:T_s]
            passes, dt = 0, 0.0
            while dt < 10.0 and passes < 64:       # about 10 s of CPU work
                tc = time.perf_counter()
                po.forward(ex, xs, split=split)
                dt += time.perf_counter() - tc
                passes += 1
            macs = passes * po.expansion_macs(ex, T_s)
            sample = ("%d passes of forward (quantize, contract, de-quantize) over all %d output channels and "
                      "%d tokens%s; expansion built outside the timer"
                      % (passes, O_s, T_s, " of the stack's first layer" if args.workload == "stack" else ""))
        elif cfg.kind == "chain":
            l0 = cfg.layers[0]
            small = wl.residual_stack(l0.out_features // 4, (len(cfg.layers) - 2) // 2, cfg.layers[-1].out_features // 4,
                                      l0.bits, l0.K, l0.gamma, l0.group, 512, cfg.split, name=cfg.name + "_small")
            exs = [po.expand(wl.make_weight(small, i), l.bits, l.K, l.gamma, l.group) for i, l in enumerate(small.layers)]
            layers_o = [po.ChainLayer(e, None, c[0], c[1], c[2]) for e, c in zip(exs, small.chain)]
            xs = wl.make_input(small)
            passes, dt = 0, 0.0
            while dt < 10.0 and passes < 64:
                tc = time.perf_counter()
                po.chain_forward(layers_o, xs, split=split)
                dt += time.perf_counter() - tc
                passes += 1
            macs = passes * sum(po.expansion_macs(e, small.tokens) for e in exs)
            sample = "%d passes over the reduced copy %s, %d tokens" % (passes, small.name, small.tokens)
        else:
            small = wl.scaled(cfg, out_div=2, in_div=1, tokens=512) if cfg.kind != "conv2d" else cfg
            Wsm = [wl.make_weight(small, i) for i in range(len(small.layers))]
            exs = [po.expand(Wsm[i], l.bits, l.K, l.gamma, l.group) for i, l in enumerate(small.layers)]
            xs = wl.make_input(small)
            passes, dt = 0, 0.0
            while dt < 10.0 and passes < 64:
                tc = time.perf_counter()
                if cfg.kind == "conv2d":
                    c = small.conv
                    po.forward_conv2d(exs[0], xs, c["kh"], c["kw"], c["stride"], c["pad"], split=split)
                else:
                    po.mlp_forward(exs[0], exs[1], "gelu" if cfg.kind == "mlp_gelu" else "gated", xs, split=split)
                dt += time.perf_counter() - tc
                passes += 1
            macs = passes * sum(po.expansion_macs(e, small.tokens) for e in exs)
            sample = "%d passes over the reduced copy %s, %d tokens" % (passes, small.name, small.tokens)
        cpu = dict(value=2.0 * macs / dt / 1e12, unit="TOPS", cores=int(cores), kind="oracle",
                   sample=sample, seconds=dt)

    # ---- data-free diagnostic (not part of a step): spectral norm of layer 0's fp32 weight by
    # power iteration; every iteration reads W twice, the last product once more
    sn_iters = 20
    pipe.pipe_spectral_norm(Ws[0], 2)
    torch.cuda.synchronize()
    t_sn = time.perf_counter()
    sigma0 = pipe.pipe_spectral_norm(Ws[0], sn_iters)     # synchronizes
    t_sn = time.perf_counter() - t_sn
    sn_bytes = (2 * sn_iters + 1) * Ws[0].numel() * 4
    spectral = {"layer": 0, "iters": sn_iters, "sigma": sigma0, "ms": t_sn * 1e3, "achieved_gbs": sn_bytes / t_sn / 1e9,
                "frac_of_hbm_peak": sn_bytes / t_sn / 1e9 / HBM_PEAK_GBS}

    out = {
        "metric": "effective int TOPS of the residual-expanded layer (2*T*in*stored_rows / step time)",
        "value": head["eff_tops"],
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_ms": args.settle_ms,          # untimed load before the warm-up steps (clocks)
        "hip_force_dev_kernarg": os.environ.get("HIP_FORCE_DEV_KERNARG"),
        "step_mode": head["step_mode"],       # the K timed steps as one HIP graph, or launched eagerly
        "static_activation_scale": static,
        "cold_start": {"ms_per_step": cold["ms_per_step"], "kernel_ms": cold["kernel_ms_per_step"],
                       "steps": min(50, args.steps), "warmup": min(5, args.warmup), "step_mode": cold["step_mode"]},
        "ms_per_step": head["ms_per_step"],
        "tokens_per_s": head["tokens_per_s"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": cfg.name, "tokens": T0, "layers": [[l.out_features, l.in_features] for l in cfg.layers],
                   "bits": cfg.layers[0].bits, "K": cfg.layers[0].K, "gamma": cfg.layers[0].gamma,
                   "group": cfg.layers[0].group, "split": list(cfg.split),
                   "macs_per_token": macs_per_token, "expansion_bytes": stream_bytes},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "sweep": sweep,
        "other_workloads": extra,
        "ensemble_ms_per_step": ensemble_ms,
        "spectral_norm": spectral,
        # reference rates of this chip (not targets): MFMA-only loop with constant operands, with
        # ternary codes x random int8 (what C4 feeds the pipe), with random int8 x int8; plain
        # streaming read of 2 GiB with the weight-streaming kernel's access pattern
        "mfma_probe_tops": pipe.pipe_mfma_probe(20000, 0),
        "mfma_probe_tops_ternary_x_int8": pipe.pipe_mfma_probe(20000, 1),
        "mfma_probe_tops_int8_x_int8": pipe.pipe_mfma_probe(20000, 2),
        # the same on v_mfma_i32_32x32x32_i8 (twice the work per operand byte, but a lower sustained rate)
        "mfma_probe_tops_32x32x32_ternary_x_int8": pipe.pipe_mfma_probe(20000, 11),
        "hbm_probe_gbs": pipe.pipe_hbm_probe(1 << 31),
        # the same step counted as if all K orders were dense (2*T*in*out*K): NOT the roofline numerator
        "dense_equivalent_tops": 2.0 * T0 * sum(l.in_features * l.out_features * l.K for l in cfg.layers)
                                 / (head["ms_per_step"] * 1e-3) / 1e12,
        "expand_seconds": expand_s,
        "input_generation_seconds": gen_s,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
