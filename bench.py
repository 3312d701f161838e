#!/usr/bin/env python3
"""Benchmark of the binary-decomposition mixed-precision convolution on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input:
for every case of the workload (a layer shape at one (k_w, k_a) pair) the
activation bit-plane packing followed by the AND+popcount convolution with its
fused shift-accumulate and scale/offset epilogue.  Weight packing is done once
before timing (it is an offline step in the paper's deployment flow, Sec. 4.3).
All inputs are resident in HBM before the timed region starts.

Prints ONE JSON line (the README lists the fields).
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

# Integer-ALU roofline of the AND+popcount inner product on MI355X: 256 CUs x 64
# int32 lanes per clock x 2.4 GHz = 39.3 T lane-ops/s; 32 binary MACs cost two
# lane-ops (v_and_b32 + accumulating v_bcnt_u32_b32) and count as 64 binary ops.
ALU_LANE_OPS = 256 * 64 * 2.4e9
PEAK_BINARY_TOPS = ALU_LANE_OPS / 2 * 64 / 1e12      # 1258.3
HBM_PEAK_GBS = 8000.0

WORKLOADS = {"tiny": 1, "cifar20": 2, "resnet18": 3, "resnet50": 4, "fc": 5, "resnet18_five": 6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet18", choices=sorted(WORKLOADS))
    ap.add_argument("--kernel-reps", type=int, default=50, help="back-to-back launches per case for per-kernel timing (after 10 warm-up launches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma", action="store_true", help="skip the int8 matrix-core comparison timing")
    ap.add_argument("--no-requant", action="store_true", help="skip timing the fused re-quantising call")
    ap.add_argument("--no-two-stage", action="store_true", help="skip timing the literal two-stage form")
    ap.add_argument("--no-quantizers", action="store_true", help="skip timing the quantiser / aggregation kernels")
    ap.add_argument("--no-chain", action="store_true", help="skip timing the chained ResNet-20-shaped stack")
    ap.add_argument("--only", default=None, metavar="LAYER,KW,KA",
                    help="restrict the workload to one case (layer index and bitwidths), e.g. 0,2,2")
    ap.add_argument("--traffic-pass", action="store_true",
                    help="no timing: one copy of known size (256 MiB) and one pass of the workload, to be run under "
                         "`rocprofv3 --pmc FETCH_SIZE` and again under `--pmc WRITE_SIZE`")
    ap.add_argument("--traffic-reps", type=int, default=1,
                    help="with --traffic-pass: passes of the workload (rotating buffers); the last one is warm")
    ap.add_argument("--cases-out", default=None, help="write the per-case table (JSON) here")
    ap.add_argument("--variant", type=int, default=0, help="conv kernel variant (0 = library heuristic)")
    return ap.parse_args()


ROTATE_BYTES = 256 << 20      # working set every timed loop cycles through (more than the last-level cache)
MAX_SLOTS = 32


class Pools:
    """Flat device pools that the cases cut their rotating buffer sets from."""

    def __init__(self, cases, dev):
        import torch
        import paper_2003_07577_amd as ebs
        need_out = need_pa = 0
        for c in cases:
            L = c.layer
            r = n_slots(c)
            need_out = max(need_out, r * L.N * L.OH * L.OW * L.K)
            need_pa = max(need_pa, r * (ebs.ebs_packed_activations_bytes(L.N, L.H, L.W, L.C, c.k_a) // 4 + 64))
        self.acc = torch.empty(need_out, dtype=torch.int32, device=dev)
        self.out = torch.empty(need_out, dtype=torch.float32, device=dev)
        self.pa = torch.empty(need_pa, dtype=torch.int32, device=dev)


def n_slots(case):
    """Rotating buffer sets of a case: enough that input + output of consecutive launches cover ROTATE_BYTES."""
    return max(2, min(MAX_SLOTS, -(-ROTATE_BYTES // conv_bytes(case))))


class CaseBuffers:
    """Device-resident tensors of one case (torch owns memory only).  Packed activations and the two
    outputs exist n_slots() times, cut from shared pools; every pack / conv call moves on to the next
    set, so that back-to-back launches neither re-read nor re-write lines that are still in a cache."""

    def __init__(self, case, inputs, pools, dev):
        import torch
        import paper_2003_07577_amd as ebs
        L = case.layer
        self.case = case
        self.a = torch.from_numpy(inputs["a"]).to(dev)
        q = torch.from_numpy(inputs["q"]).to(dev)
        pa_words = ebs.ebs_packed_activations_bytes(L.N, L.H, L.W, L.C, case.k_a) // 4
        pa_pitch = (pa_words + 63) // 64 * 64
        self.pw = torch.empty(ebs.ebs_packed_weights_bytes(L.K, L.C, L.R, L.S, case.k_w) // 4,
                              dtype=torch.int32, device=dev)
        ebs.ebs_pack_weights(q, L.K, L.C, L.R, L.S, case.k_w, self.pw)          # offline step
        self.scale = torch.from_numpy(inputs["scale"]).to(dev)
        self.offset = None if inputs["offset"] is None else torch.from_numpy(inputs["offset"]).to(dev)
        self.per_channel = inputs["per_channel"]
        n_out = L.N * L.OH * L.OW * L.K
        r = n_slots(case)
        self.slots = [(pools.pa[i * pa_pitch:i * pa_pitch + pa_words], pools.acc[i * n_out:(i + 1) * n_out],
                       pools.out[i * n_out:(i + 1) * n_out]) for i in range(r)]
        self.i = 0
        self.pa, self.acc, self.out = self.slots[0]

    def next_slot(self):
        self.i = (self.i + 1) % len(self.slots)
        self.pa, self.acc, self.out = self.slots[self.i]

    def pack_all(self, ebs, stream):
        """Fills every slot's packed activations (the pools are shared between cases)."""
        for _ in self.slots:
            self.next_slot()
            self.pack(ebs, stream)

    def pack(self, ebs, stream):
        L = self.case.layer
        ebs.ebs_pack_activations(self.a, L.N, L.H, L.W, L.C, self.case.k_a, self.pa, stream)

    def conv(self, ebs, stream, variant=0):
        L, c = self.case.layer, self.case
        ebs.ebs_mixed_conv2d_variant(variant, self.pa, self.pw, L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad,
                                     c.k_w, c.k_a, self.scale, self.offset, self.per_channel, self.acc, self.out,
                                     stream)


def conv_bytes(case):
    """Algorithmic HBM bytes of one convolution launch: packed operands once, int32+fp32 outputs once."""
    L = case.layer
    cw = (L.C + 31) // 32
    return (L.N * (L.H + 2) * (L.W + 2) * cw * case.k_a * 4 + ((L.K + 15) // 16 * 16) * L.R * L.S * cw * case.k_w * 4
            + L.N * L.OH * L.OW * L.K * 8)


def pack_bytes(case):
    L = case.layer
    cw = (L.C + 31) // 32
    return L.N * L.H * L.W * L.C + L.N * (L.H + 2) * (L.W + 2) * cw * case.k_a * 4


def gpu_clocks():
    """Shader and memory clock states as the driver reports them (the starred entry is the current one)."""
    import glob
    out = {}
    for name in ("pp_dpm_sclk", "pp_dpm_mclk"):
        for path in sorted(glob.glob(f"/sys/class/drm/card*/device/{name}")):
            try:
                out[name] = " ".join(open(path).read().split())
                break
            except OSError:
                continue
    return out or None


def source_digest():
    """Digest of the HIP sources the library is built from: measured profiles are stamped with it."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2003_07577_amd", "csrc", "*"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def read_traffic(workload):
    """HBM bytes per convolution launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two
    separate runs, scaled by a copy kernel of known size); the committed summary holds the figure
    and the digest of the sources it was measured on.  Returns (bytes or None, note)."""
    path = os.path.join(ROOT, "profiles", f"bd_conv_{workload}_hbm_traffic.txt")
    value = stamp = None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                value = float(line.split(":")[1].split()[0])
            if line.startswith("source_digest:"):
                stamp = line.split(":")[1].split()[0]
    except OSError:
        return None, "no committed traffic summary for this workload"
    now = source_digest()
    if stamp != now:
        return None, f"committed traffic summary was measured on sources {stamp}, these are {now}: not used"
    return value, f"profiles/bd_conv_{workload}_hbm_traffic.txt, sources {stamp}"


def measured_peaks(ebs, torch, dev, stream):
    """What the machine sustains for the two resources the kernels are bound by (library probes):
    the AND + accumulating-bitcount pair on registers only, and a 256 MiB copy / fill."""
    def timed(f, reps):
        f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            f()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps
    blocks, trips = 256 * 8, 2000
    seed = torch.randint(0, 2 ** 31 - 1, (512,), dtype=torch.int32, device=dev)
    sink = torch.zeros(blocks * 256, dtype=torch.int32, device=dev)
    t = min(timed(lambda: ebs.ebs_probe_and_bcnt(seed, sink, blocks, trips, stream), 5) for _ in range(3))
    alu = ebs.ebs_probe_and_bcnt_pairs(blocks, trips) * 64 / t / 1e12
    n = 256 << 20
    src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty(n, dtype=torch.uint8, device=dev)
    t_copy = min(timed(lambda: ebs.ebs_probe_copy(src, dst, n, 8192, stream), 5) for _ in range(3))
    t_fill = min(timed(lambda: ebs.ebs_probe_copy(None, dst, n, 8192, stream), 5) for _ in range(3))
    # period of back-to-back launches of a kernel that does next to nothing (one work-group copying 4 KiB):
    # what every launch of a stream costs at least, whatever the kernel
    t_empty = min(timed(lambda: ebs.ebs_probe_copy(src, dst, 4096, 1, stream), 200) for _ in range(3))
    return {"alu_binary_tops": round(alu, 1), "hbm_copy_gbs": round(2 * n / t_copy / 1e9, 1),
            "hbm_fill_gbs": round(n / t_fill / 1e9, 1), "launch_period_floor_us": round(t_empty * 1e6, 2),
            "how": "ebs_probe_and_bcnt (register-only AND + accumulating bitcount, 2048 work-groups) and "
                   "ebs_probe_copy on 256 MiB (copy counts read + written bytes; fill = write only)"}


def cpu_baseline(cases):
    """The oracle as it stands, timed on the host cores: each distinct layer shape once
    (its time does not depend on the bitwidths), aggregated over the cases of the workload."""
    import numpy as np
    import oracle
    import ebs_workloads as wl
    oracle.build()
    per_layer = {}
    layers = []
    for c in cases:
        if c.layer not in per_layer:
            per_layer[c.layer] = []
            layers.append((c.layer, wl.make_inputs(c)))
    t_begin = time.time()
    passes = 0
    while passes == 0 or (time.time() - t_begin < 12.0 and passes < 50):   # about 10-20 s of CPU work
        for L, inp in layers:
            t0 = time.time()
            oracle.conv2d_levels(inp["a"], inp["q"], L.stride, L.pad)
            per_layer[L].append(time.time() - t0)
        passes += 1
        print(f"[cpu_baseline] pass {passes} done at {time.time() - t_begin:.1f}s", file=sys.stderr, flush=True)
    total_cpu_s = sum(sum(v) for v in per_layer.values())
    per_layer = {L: sum(v) / len(v) for L, v in per_layer.items()}
    covered = [c for c in cases if c.layer in per_layer]
    ops = sum(c.binary_ops for c in covered)
    secs = sum(per_layer[c.layer] for c in covered)
    macs = sum(L.int_macs for L in per_layer)
    return {
        "value": ops / secs / 1e12, "unit": "TOP/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": (f"direct integer conv, each of {len(per_layer)} layer shapes of the workload at full batch "
                   f"per pass ({macs / 1e9:.1f} G int-MACs), {passes} passes, {total_cpu_s:.1f}s in all; time is bitwidth-independent, "
                   f"so the rate is aggregated over the {len(covered)} (layer, k_w, k_a) cases like the GPU value"),
        "int_gmacs_per_s": macs / sum(per_layer.values()) / 1e9,
    }



def vendor_int8_gemm_us(torch, dev, M, K, N):
    """Microseconds per call of the vendor library's int8 GEMM (int32 result) on an M x K x N problem, timed as 20
    calls in a captured graph replayed five times; None where this build of the framework has no such call."""
    try:
        a = torch.randint(-8, 8, (M, K), dtype=torch.int8, device=dev)
        b = torch.randint(-8, 8, (K, N), dtype=torch.int8, device=dev)
        c = torch.empty((M, N), dtype=torch.int32, device=dev)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            torch._int_mm(a, b, out=c)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(20):
                    torch._int_mm(a, b, out=c)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(5):
            graph.replay()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) * 1e3 / 100
    except Exception:
        return None

def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    import ebs_workloads as wl
    import paper_2003_07577_amd as ebs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    ebs.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()

    cfg = WORKLOADS[args.workload]
    cases = wl.config_cases(cfg)
    if args.only:
        li, kw, ka = (int(v) for v in args.only.split(","))
        cases = [c for c in cases if (c.layer_index, c.k_w, c.k_a) == (li, kw, ka)]
        if not cases:
            print("--only matches no case", file=sys.stderr)
            sys.exit(1)
    pools = Pools(cases, dev)
    bufs = []
    for c in cases:
        bufs.append(CaseBuffers(c, wl.make_inputs(c), pools, dev))
    torch.cuda.synchronize()

    if args.traffic_pass:
        n = 256 << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty(n, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        ebs.ebs_probe_copy(src, dst, n, 4096, stream)
        torch.cuda.synchronize()
        for _ in range(max(1, args.traffic_reps)):
            for b in bufs:
                b.next_slot()
                b.pack(ebs, stream)
                b.conv(ebs, stream, args.variant)
                torch.cuda.synchronize()
        print(json.dumps({"traffic_pass": True, "passes": max(1, args.traffic_reps), "copy_bytes": n, "cases": len(bufs), "source_digest": source_digest()}))
        return

    def step():
        for b in bufs:
            b.next_slot()
            b.pack(ebs, stream)
            b.conv(ebs, stream, args.variant)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.time()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.time() - t0
    ms_total = e0.elapsed_time(e1)
    ms_per_step = ms_total / args.steps
    ops_per_step = sum(c.binary_ops for c in cases)
    value = ops_per_step / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel timing, live, with events on the launch stream
    table = []
    conv_us_sum = pack_us_sum = 0.0
    conv_ops = 0
    conv_bytes_sum = pack_bytes_sum = 0
    for b in bufs:
        c = b.case
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        b.pack_all(ebs, stream)                  # the pools are shared: every slot gets this case's input
        for _ in range(10):
            b.next_slot()
            b.conv(ebs, stream, args.variant)
        ev[0].record(stream)
        for _ in range(args.kernel_reps):
            b.next_slot()
            b.pack(ebs, stream)
        ev[1].record(stream)
        # the convolution launches in five batches: the mean over all of them is the figure used,
        # the fastest batch is kept beside it in the per-case table
        nb = 5 if args.kernel_reps >= 5 else 1
        per = args.kernel_reps // nb
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(nb)]
        for i in range(nb):
            for _ in range(per if i + 1 < nb else args.kernel_reps - per * (nb - 1)):
                b.next_slot()
                b.conv(ebs, stream, args.variant)
            marks[i].record(stream)
        ev[2] = marks[-1]
        torch.cuda.synchronize()
        pack_us = ev[0].elapsed_time(ev[1]) * 1e3 / args.kernel_reps
        conv_us = ev[1].elapsed_time(ev[2]) * 1e3 / args.kernel_reps
        edges = [ev[1]] + marks
        conv_us_min = min(edges[i].elapsed_time(edges[i + 1]) * 1e3 / (per if i + 1 < nb else args.kernel_reps - per * (nb - 1))
                          for i in range(nb))
        conv_us_sum += conv_us
        pack_us_sum += pack_us
        conv_ops += c.binary_ops
        conv_bytes_sum += conv_bytes(c)
        pack_bytes_sum += pack_bytes(c)
        tops = c.binary_ops / conv_us / 1e6
        t_alu = c.binary_ops / PEAK_BINARY_TOPS / 1e6
        t_hbm = conv_bytes(c) / HBM_PEAK_GBS / 1e3
        table.append({
            "case": c.tag, "layer": c.layer.name, "k_w": c.k_w, "k_a": c.k_a,
            "conv_us": round(conv_us, 2), "conv_us_min_batch": round(conv_us_min, 2), "pack_us": round(pack_us, 2),
            "binary_tops": round(tops, 1), "alu_frac": round(tops / PEAK_BINARY_TOPS, 4),
            "conv_hbm_gbs": round(conv_bytes(c) / conv_us / 1e3, 1),
            "pack_hbm_gbs": round(pack_bytes(c) / pack_us / 1e3, 1), "pack_bytes": pack_bytes(c),
            "binding_roof": "alu" if t_alu >= t_hbm else "hbm",
            "roof_us": round(max(t_alu, t_hbm), 2),
            "frac_of_binding_roof": round(max(t_alu, t_hbm) / conv_us, 4),
            "rotating_sets": len(b.slots),
        })
    achieved = conv_ops / conv_us_sum / 1e6
    roofline = {
        "kernel": "bd_conv (AND+popcount convolution, all launches of the workload)",
        "bound": "alu", "achieved": round(achieved, 2), "peak": round(PEAK_BINARY_TOPS, 1), "unit": "TOP/s",
        "frac": round(achieved / PEAK_BINARY_TOPS, 4), "traffic": None,
        "avg_launch_us": round(conv_us_sum / len(bufs), 2),
        "hbm_gbs_algorithmic": round(conv_bytes_sum / conv_us_sum / 1e3, 1),
        # per case, against the roof that binds it (ALU, or HBM at 8 TB/s where the 8 B per output take longer)
        "min_case_frac": min(r["frac_of_binding_roof"] for r in table),
        "max_case_frac": max(r["frac_of_binding_roof"] for r in table),
        "min_case_alu_frac": min(r["alu_frac"] for r in table),
        "cases_below_half": [f'{r["layer"]} ({r["k_w"]},{r["k_a"]}) {r["frac_of_binding_roof"]}' for r in table
                             if r["frac_of_binding_roof"] < 0.5],
        "timing": f"{args.kernel_reps} back-to-back launches per case after 10 warm-up launches, inputs and outputs "
                  f"rotating over >= {ROTATE_BYTES >> 20} MiB",
    }
    peaks = measured_peaks(ebs, torch, dev, stream)
    roofline["measured_peak"] = peaks
    roofline["frac_of_measured"] = round(achieved / peaks["alu_binary_tops"], 4)
    pack_roof = {
        "kernel": "pack_activations", "bound": "hbm", "achieved": round(pack_bytes_sum / pack_us_sum / 1e3, 1),
        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(pack_bytes_sum / pack_us_sum / 1e3 / HBM_PEAK_GBS, 4),
        "avg_launch_us": round(pack_us_sum / len(bufs), 2),
    }
    # large and small inputs apart: below a few MB a launch is as short as the launch period itself
    for name, sel in (("large_inputs", lambda r: r["pack_bytes"] >= 8 << 20), ("small_inputs", lambda r: r["pack_bytes"] < 8 << 20)):
        rows = [r for r in table if sel(r)]
        if rows:
            us = sum(r["pack_us"] for r in rows)
            by = sum(r["pack_bytes"] for r in rows)
            pack_roof[name] = {"cases": len(rows), "avg_launch_us": round(us / len(rows), 2),
                               "achieved": round(by / us / 1e3, 1), "frac": round(by / us / 1e3 / HBM_PEAK_GBS, 4)}
    pack_roof["launch_period_floor_us"] = peaks["launch_period_floor_us"]

    # ---- measured comparison: the same layers on the int8 matrix cores (no binary decomposition);
    #      its time does not depend on the bitwidths, so each layer shape is timed once
    mfma = None
    if not args.no_mfma:
        per_layer = {}
        for b in bufs:
            L = b.case.layer
            if L in per_layer or L.C % 32 != 0:
                continue
            import paper_2003_07577_amd as ebs_mod
            wl_inp = wl.make_inputs(b.case)
            qd = torch.from_numpy(wl_inp["q"]).to(dev)
            f = lambda: ebs_mod.ebs_mixed_conv2d_mfma_i8(b.a, qd, L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad,
                                                          b.scale, b.offset, b.per_channel, b.acc, b.out, stream)
            f()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record(stream)
            for _ in range(args.kernel_reps):
                f()
            ev[1].record(stream)
            torch.cuda.synchronize()
            per_layer[L] = ev[0].elapsed_time(ev[1]) * 1e3 / args.kernel_reps
        covered = [b.case for b in bufs if b.case.layer in per_layer]
        if covered:
            t_us = sum(per_layer[c.layer] for c in covered)
            macs = sum(L.int_macs for L in per_layer)
            mfma = {
                "kernel": "ebs_mixed_conv2d_mfma_i8 (comparison only, not the default path)",
                "equivalent_binary_tops": round(sum(c.binary_ops for c in covered) / t_us / 1e6, 1),
                "int8_tmacs": round(macs / sum(per_layer.values()) / 1e6, 1),
                "frac_of_int8_mfma_peak": round(2 * macs / sum(per_layer.values()) / 1e6 / 5000.0, 4),
                "layer_us": {L.name: round(t, 1) for L, t in per_layer.items()},
            }
            for r in table:
                L = [c.layer for c in cases if c.tag == r["case"]][0]
                if L in per_layer:
                    r["mfma_i8_us"] = round(per_layer[L], 2)
            # the vendor library's int8 GEMM on each layer's GEMM shape, as context for the kernel above
            vendor = {L.name: vendor_int8_gemm_us(torch, dev, L.N * L.OH * L.OW, L.R * L.S * L.C, L.K) for L in per_layer}
            if all(v is not None for v in vendor.values()):
                mfma["vendor_int8_gemm_us"] = {k: round(v, 1) for k, v in vendor.items()}
                mfma["vendor_int8_gemm"] = ("torch._int_mm (the vendor GEMM library) on the layer as a plain GEMM, positions x "
                                            "(filter taps * input channels) x output channels, operands already in matrix "
                                            "form (no im2col pass, no epilogue), 20 launches in a captured graph")

    # ---- fused re-quantise + re-pack epilogue (replaces conv's 8 B/output and the next pack call)
    requant = None
    if not args.no_requant:
        t_us = 0.0
        for b, r in zip(bufs, table):
            c, L = b.case, b.case.layer
            kn = c.k_a
            nxt = torch.empty(ebs.ebs_packed_activations_bytes(L.N, L.OH, L.OW, L.K, kn) // 4, dtype=torch.int32, device=dev)
            f = lambda: ebs.ebs_mixed_conv2d_requant(b.pa, b.pw, L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad,
                                                      c.k_w, c.k_a, b.scale, b.offset, b.per_channel, 6.0, kn, nxt, stream)
            f()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record(stream)
            for _ in range(5):
                f()
            ev[1].record(stream)
            torch.cuda.synchronize()
            us = ev[0].elapsed_time(ev[1]) * 1e3 / 5
            r["requant_us"] = round(us, 2)
            t_us += us
            del nxt
        requant = {
            "kernel": "ebs_mixed_conv2d_requant (conv + next layer's quantiser + bit-plane packing + zero ring, one kernel)",
            "binary_tops": round(conv_ops / t_us / 1e6, 1), "frac_of_alu_roof": round(conv_ops / t_us / 1e6 / PEAK_BINARY_TOPS, 4),
            "vs_pack_plus_conv": round((conv_us_sum + pack_us_sum) / t_us, 3),
        }

    # ---- the literal two-stage form (partial products through memory, then the depthwise
    #      power-of-two recombination), timed on the same cases as the fused kernel
    two_stage = None
    if not args.no_two_stage:
        max_planes = max(ebs.ebs_partial_products_bytes(c.layer.N, c.layer.H, c.layer.W, c.layer.K, c.layer.R, c.layer.S,
                                                        c.layer.stride, c.layer.pad, c.k_w, c.k_a) for c in cases)
        planes = torch.empty(max_planes // 4, dtype=torch.int32, device=dev)
        s1_us = s2_us = 0.0
        p_bytes = 0
        for b, r in zip(bufs, table):
            c, L = b.case, b.case.layer
            f1 = lambda: ebs.ebs_binary_conv_planes(b.pa, b.pw, L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad,
                                                    c.k_w, c.k_a, planes, stream)
            f2 = lambda: ebs.ebs_pow2_depthwise(planes, L.N * L.OH * L.OW, L.K, c.k_w, c.k_a, b.scale, b.offset,
                                                b.per_channel, b.acc, b.out, stream)
            f1()
            f2()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            ev[0].record(stream)
            for _ in range(5):
                f1()
            ev[1].record(stream)
            for _ in range(5):
                f2()
            ev[2].record(stream)
            torch.cuda.synchronize()
            u1 = ev[0].elapsed_time(ev[1]) * 1e3 / 5
            u2 = ev[1].elapsed_time(ev[2]) * 1e3 / 5
            r["stage1_us"], r["stage2_us"] = round(u1, 2), round(u2, 2)
            s1_us += u1
            s2_us += u2
            p_bytes += L.N * L.OH * L.OW * L.K * c.k_w * c.k_a * 4
        del planes
        two_stage = {
            "kernel": "ebs_binary_conv_planes + ebs_pow2_depthwise (comparison only: P goes through HBM)",
            "binary_tops": round(conv_ops / (s1_us + s2_us) / 1e6, 1),
            "stage1_binary_tops": round(conv_ops / s1_us / 1e6, 1),
            "stage2_hbm_gbs": round((p_bytes + 8 * sum(c.layer.N * c.layer.OH * c.layer.OW * c.layer.K for c in cases)) / s2_us / 1e3, 1),
            "partial_product_bytes_per_step": p_bytes,
            "fused_speedup": round((s1_us + s2_us) / conv_us_sum, 3),
        }

    # ---- quantisers (Eq. 1a-1c) and aggregated quantisation functions (Eq. 6-7) on tensors of the
    #      workload's largest layer: its input activations and the largest filter bank
    quant = None
    if not args.no_quantizers:
        La = max((c.layer for c in cases), key=lambda L: L.N * L.H * L.W * L.C)
        Lw = max((c.layer for c in cases), key=lambda L: L.K * L.R * L.S * L.C)
        na, nw = La.N * La.H * La.W * La.C, Lw.K * Lw.R * Lw.S * Lw.C
        gen = torch.Generator(device=dev).manual_seed(1234)
        xa = (torch.randn(na, device=dev, generator=gen).abs_() * 3.0)
        xw = torch.randn(nw, device=dev, generator=gen) * 0.3
        lva = torch.empty(na, dtype=torch.uint8, device=dev)
        lvw = torch.empty(nw, dtype=torch.uint8, device=dev)
        oa = torch.empty(na, dtype=torch.float32, device=dev)
        ow = torch.empty(nw, dtype=torch.float32, device=dev)
        ws = torch.zeros(ebs.QUANT_WORKSPACE_BYTES // 4, dtype=torch.int32, device=dev)
        cand = [1, 2, 3, 4, 5]
        r = torch.zeros(5, dtype=torch.float32, device=dev)

        def timed(f, reps=10):
            f()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record(stream)
            for _ in range(reps):
                f()
            ev[1].record(stream)
            torch.cuda.synchronize()
            return ev[0].elapsed_time(ev[1]) * 1e3 / reps

        t_qa = timed(lambda: ebs.ebs_quantize_activations(xa, na, 6.0, 4, lva, stream))
        t_aa = timed(lambda: ebs.ebs_aggregate_activations(xa, na, 6.0, cand, r, None, 1.0, oa, ws, stream))
        t_qw = timed(lambda: ebs.ebs_quantize_weights(xw, nw, 4, lvw, ws, stream))
        t_aw = timed(lambda: ebs.ebs_aggregate_weights(xw, nw, cand, r, None, 1.0, ow, ws, stream))
        quant = {
            "activation_elements": na, "weight_elements": nw,
            "quantize_activations": {"us": round(t_qa, 2), "bound": "hbm", "achieved_gbs": round(5 * na / t_qa / 1e3, 1),
                                     "frac": round(5 * na / t_qa / 1e3 / HBM_PEAK_GBS, 4)},
            "aggregate_activations_5_candidates": {"us": round(t_aa, 2), "bound": "hbm", "achieved_gbs": round(8 * na / t_aa / 1e3, 1),
                                                   "frac": round(8 * na / t_aa / 1e3 / HBM_PEAK_GBS, 4)},
            "quantize_weights": {"us": round(t_qw, 2), "gelem_per_s": round(nw / t_qw / 1e3, 2),
                                 "note": "double-precision tanh per element + max reduction; offline per step"},
            "aggregate_weights_5_candidates": {"us": round(t_aw, 2), "gelem_per_s": round(nw / t_aw / 1e3, 2)},
        }

    # ---- whole stacks through the fused re-quantising call (signed weights, per-channel affine map): the 18
    #      ResNet-20-shaped layers of config 2 and the 16 ResNet-18-shaped 3x3 layers, eagerly and as a HIP graph
    chain_out = None
    if not args.no_chain:
        def time_chain(chain, label):
            L0, k0 = chain["layers"][0]["layer"], chain["layers"][0]["k_a"]
            a0 = torch.from_numpy(chain["a0"]).to(dev)
            packed = [torch.empty(ebs.ebs_packed_activations_bytes(L0.N, L0.H, L0.W, L0.C, k0) // 4, dtype=torch.int32, device=dev)]
            pws, scs, ofs = [], [], []
            for sdef in chain["layers"]:
                L = sdef["layer"]
                pw = torch.empty(ebs.ebs_packed_weights_bytes(L.K, L.C, L.R, L.S, sdef["k_w"]) // 4, dtype=torch.int32, device=dev)
                ebs.ebs_pack_weights(torch.from_numpy(sdef["q"]).to(dev), L.K, L.C, L.R, L.S, sdef["k_w"], pw)
                pws.append(pw)
                scs.append(torch.from_numpy(sdef["scale"]).to(dev))
                ofs.append(torch.from_numpy(sdef["offset"]).to(dev))
                packed.append(torch.empty(ebs.ebs_packed_activations_bytes(L.N, L.OH, L.OW, L.K, sdef["k_next"]) // 4,
                                          dtype=torch.int32, device=dev))

            def run_chain(st):
                ebs.ebs_pack_activations(a0, L0.N, L0.H, L0.W, L0.C, k0, packed[0], st)
                for i, sdef in enumerate(chain["layers"]):
                    L = sdef["layer"]
                    ebs.ebs_mixed_conv2d_requant(packed[i], pws[i], L.N, L.C, L.H, L.W, L.K, L.R, L.S, L.stride, L.pad,
                                                 sdef["k_w"], sdef["k_a"], scs[i], ofs[i], True, sdef["alpha"], sdef["k_next"],
                                                 packed[i + 1], st, signed_weights=True)

            def timed_us(f, reps=20):
                for _ in range(3):
                    f()
                torch.cuda.synchronize()
                e0c, e1c = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0c.record(stream)
                for _ in range(reps):
                    f()
                e1c.record(stream)
                torch.cuda.synchronize()
                return e0c.elapsed_time(e1c) * 1e3 / reps

            t_eager = timed_us(lambda: run_chain(stream))
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            with torch.cuda.graph(graph, stream=side):
                run_chain(torch.cuda.current_stream())
            torch.cuda.synchronize()
            t_graph = timed_us(graph.replay)
            ops = sum(2 * sdef["layer"].int_macs * sdef["k_w"] * sdef["k_a"] for sdef in chain["layers"])
            best = min(t_eager, t_graph)
            return {"workload": label, "layers": len(chain["layers"]), "batch": L0.N,
                    "bitwidths": [[sdef["k_w"], sdef["k_a"]] for sdef in chain["layers"]],
                    "eager_us": round(t_eager, 1), "graph_us": round(t_graph, 1),
                    "binary_tops": round(ops / best / 1e6, 1), "frac_of_alu_roof": round(ops / best / 1e6 / PEAK_BINARY_TOPS, 4),
                    "images_per_s": round(L0.N / (best * 1e-6), 0)}

        chain_out = {
            "resnet20": time_chain(wl.resnet20_chain(N=128), "configs[1] ResNet-20-shaped stack (CIFAR sizes), bitwidths from {1..5}"),
            "resnet18": time_chain(wl.resnet18_chain(N=64), "configs[2] ResNet-18-shaped 3x3 stack (ImageNet sizes), bitwidths from {1..4}"),
        }

    traffic, note = read_traffic(args.workload)
    roofline["traffic"] = traffic
    roofline["traffic_source"] = note

    out = {
        "metric": "effective binary TOP/s and latency per mixed-precision conv layer; % of int roofline",
        "metric_detail": "value = effective binary TOP/s of pack_activations + conv over all cases of the workload; "
                         "latency per layer = roofline.avg_launch_us; % of the integer roofline = roofline.frac",
        "value": round(value, 2), "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bit-planes, int32 accumulate, fp32 epilogue", "data": "synthetic",
        "config": {"workload": f"configs[{cfg - 1}] {args.workload}: {len(cases)} (layer, k_w, k_a) cases, "
                               f"N={cases[0].layer.N}", "cases": len(cases), "variant": args.variant},
        "conv_only_tops": round(achieved, 2),
        "wall_s": round(wall, 3),
        "roofline": roofline, "pack_roofline": pack_roof,
    }
    if mfma is not None:
        out["mfma_i8_comparison"] = mfma
    if requant is not None:
        out["requant_epilogue"] = requant
    if two_stage is not None:
        out["two_stage_comparison"] = two_stage
    if quant is not None:
        out["quantizers"] = quant
    if chain_out is not None:
        out["chained_stacks"] = chain_out
    clocks = gpu_clocks()
    if clocks:
        out["clocks"] = clocks
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cases)
    cases_out = args.cases_out
    if cases_out:
        with open(cases_out, "w") as f:
            json.dump(table, f, indent=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
