#!/usr/bin/env python3
"""Benchmark of the qwZ/qgZ kernel path on one MI355X.

A "step" is one simulated training step of one GPU's share of a 40-layer,
hidden-12288 GPT-style model under ZeRO++ with X = 8 GPUs per node and Y = 48
nodes (Sec. 3 of the paper; the collectives themselves are not part of the step):

  forward,  per layer:  qwz_dequantize of the gathered int8 weights (bf16 out)
  backward, per layer:  qwz_dequantize again, then for the layer's fp16 gradient
                        qgz_reorder (fused reorder + int4 quantize),
                        qgz_intra_reduce (8 peers -> int4),
                        qgz_inter_reduce (48 nodes -> fp32 average),
                        and qwz_quantize of the rank's own updated weight shard.

Inputs are seeded synthetic tensors resident in HBM before the timed region.
Prints ONE JSON line; `value` is algorithmic bytes per second over the whole step.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
ALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9   # plain (unpacked) vector-ALU lane-operations per second
METRIC = "effective HBM GB/s (and % of peak) per qwZ/qgZ kernel at 1 MI355X"
KERNEL_SOURCE = os.path.join(ROOT, "paper_2306_10209_amd", "csrc", "zpp_gfx950.hip")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=40)
    ap.add_argument("--hidden", type=int, default=12288)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-schedules", action="store_true",
                    help="skip the timings of the Sec. 4.1 launch schedules (pipeline stages, weight prefetch)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the per-kernel timings at the shapes of the other configurations")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replays of the step")
    ap.add_argument("--cpu-sample-div", type=int, default=1,
                    help="the CPU oracle is timed on 1/div of one layer")
    return ap.parse_args()


class Bytes:
    """Algorithmic bytes each operation must move (codes + fp32 scales + payload)."""

    @staticmethod
    def quantize(n, B, bits, in_bytes=2):
        return n * in_bytes + n * bits // 8 + 4 * (n // B)

    @staticmethod
    def dequantize(n, B, bits, out_bytes=2):
        return n * bits // 8 + 4 * (n // B) + n * out_bytes

    @staticmethod
    def intra(m, B, bits, X):
        return (X + 1) * (m * bits // 8 + 4 * (m // B))

    @staticmethod
    def inter(m, B, bits, Y):
        return Y * (m * bits // 8 + 4 * (m // B)) + 4 * m


def profile_figures(name, kernel, elements):
    """Per-launch figures of `kernel` from a committed rocprofv3 counter summary under profiles/.
    They are measurements of an earlier run, so they are handed out only with their source
    attached and only if the summary says it was taken from this very kernel source (sha256 of
    the .hip file) at this problem size; otherwise the reason is returned instead."""
    path = os.path.join(ROOT, "profiles", name)
    src = {"file": f"profiles/{name}"}
    if not os.path.exists(path):
        return None, dict(src, refused="summary not present")
    want_hash = hashlib.sha256(open(KERNEL_SOURCE, "rb").read()).hexdigest()
    facts, rows = {}, {}
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == "SOURCE":
            facts.update(p.split("=", 1) for p in parts[1:] if "=" in p)
        if len(parts) >= 3 and parts[0] in ("TRAFFIC", "VALU", "TRACE"):
            rows[parts[1]] = dict(p.split("=", 1) for p in parts[2:] if "=" in p)
    if facts.get("sha256") != want_hash:
        return None, dict(src, refused="summary was taken from another version of the kernel source")
    row = rows.get(kernel)
    if row is None:
        return None, dict(src, refused=f"no row for {kernel}")
    if int(row.get("elements", -1)) != elements:
        return None, dict(src, refused="summary was taken at another problem size")
    return row, dict(src, kernel=row.get("kernel"), grid_threads=int(row.get("grid_threads", 0)), elements=elements)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the P ranks of the method are simulated as buffers on it; "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2306_10209_amd import binding as zpp, diagnostics, workloads

    zpp.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    X, Y, W = 8, 48, 384
    WB, WBITS = 2048, 8           # weights: int8, block 2048
    GB_, GBITS = 512, 4           # gradients: int4, block 512
    n_L = workloads.layer_numel(args.hidden)
    assert n_L % (X * Y * GB_) == 0 and (n_L // W) % WB == 0
    m = n_L // X                  # intra-node stage output elements
    L = n_L // W                  # inter-node stage output elements = own partition
    layers = args.layers

    # ---------------- setup (untimed): resident inputs ----------------
    t0 = time.time()
    w = workloads.weights(n_L, device=dev, tensor_id=1)
    wcodes, wscales = zpp.qwz_quantize(w, WB, WBITS)
    torch.cuda.synchronize()
    wout = w                       # reuse the 3.6 GB buffer as the dequantize output
    own = workloads.weights(L, device=dev, tensor_id=2)
    own_codes = torch.empty(L, dtype=torch.uint8, device=dev)
    own_scales = torch.empty(L // WB, dtype=torch.float32, device=dev)
    grad = workloads.gradients(n_L, device=dev, tensor_id=3, tail_std=0.0)
    gcodes = torch.empty(n_L // 2, dtype=torch.uint8, device=dev)
    gscales = torch.empty(n_L // GB_, dtype=torch.float32, device=dev)
    # peers' contributions to the intra-node stage (2 sets), already encoded
    peer_sets = []
    for s in range(2):
        peers = []
        for k in range(X - 1):
            g = workloads.gradients(m, device=dev, tensor_id=100 + s * 16 + k, tail_std=0.0)
            peers.append(zpp.qwz_quantize(g, GB_, GBITS))
            torch.cuda.synchronize()
            del g
        peer_sets.append(peers)
    icodes = torch.empty(m // 2, dtype=torch.uint8, device=dev)
    iscales = torch.empty(m // GB_, dtype=torch.float32, device=dev)
    # other nodes' contributions to the inter-node stage (8 sets, so they do not stay in cache)
    node_sets = []
    for s in range(8):
        g = workloads.gradients((Y - 1) * L, device=dev, tensor_id=200 + s, tail_std=0.0)
        c, sc = zpp.qwz_quantize(g, GB_, GBITS)
        torch.cuda.synchronize()
        del g
        node_sets.append(([c[i * L // 2:(i + 1) * L // 2] for i in range(Y - 1)],
                          [sc[i * L // GB_:(i + 1) * L // GB_] for i in range(Y - 1)]))
    gout = torch.empty(L, dtype=torch.float32, device=dev)
    # pointer tables of the two simulated all-to-alls: this GPU's own piece first, then the others'
    intra_tables = [zpp.PeerTable([gcodes[:m // 2]] + [p[0] for p in peers], [gscales[:m // GB_]] + [p[1] for p in peers])
                    for peers in peer_sets]
    inter_tables = [zpp.PeerTable([icodes[:L // 2]] + nc, [iscales[:L // GB_]] + ns) for nc, ns in node_sets]
    setup_s = time.time() - t0

    bytes_per = {
        "qwz_dequantize": Bytes.dequantize(n_L, WB, WBITS),
        "qwz_quantize": Bytes.quantize(L, WB, WBITS),
        "qgz_reorder": Bytes.quantize(n_L, GB_, GBITS),
        "qgz_intra_reduce": Bytes.intra(m, GB_, GBITS, X),
        "qgz_inter_reduce": Bytes.inter(L, GB_, GBITS, Y),
    }
    elements_per = {"qwz_dequantize": n_L, "qwz_quantize": L, "qgz_reorder": n_L, "qgz_intra_reduce": m,
                    "qgz_inter_reduce": L}
    calls_per_step = {"qwz_dequantize": 2 * layers, "qwz_quantize": layers, "qgz_reorder": layers,
                      "qgz_intra_reduce": layers, "qgz_inter_reduce": layers}
    step_bytes = sum(bytes_per[k] * calls_per_step[k] for k in bytes_per)

    launch = {
        "qwz_dequantize": lambda l: zpp.qwz_dequantize(wcodes, wscales, n_L, WB, WBITS, out=wout),
        "qgz_reorder": lambda l: zpp.qgz_reorder(grad, X, Y, 1, GB_, GBITS, codes=gcodes, scales=gscales),
        "qgz_intra_reduce": lambda l: zpp.qgz_intra_reduce(intra_tables[l % 2], None, m, GB_, GBITS, codes_out=icodes,
                                                           scales_out=iscales),
        "qgz_inter_reduce": lambda l: zpp.qgz_inter_reduce(inter_tables[l % 8], None, L, GB_, GBITS, float(W), out=gout),
        "qwz_quantize": lambda l: zpp.qwz_quantize(own, WB, WBITS, codes=own_codes, scales=own_scales),
    }

    events = {k: [] for k in bytes_per}
    DOM = "qwz_dequantize"
    counter = [0]
    last = [None]

    def timed(name, l, record):
        """record = "sparse": every fourth launch of the dominant kernel sits between two HIP events of
        its own (an event costs a few microseconds of queue time, and the timed region should pay
        as little of that as possible).  record = "all": one event after every launch; a kernel's
        time runs from the event after the launch before it to the event after its own, the
        accounting rocprofv3's kernel trace uses for back-to-back launches on one queue."""
        counter[0] += 1
        if record == "sparse" and name == DOM and counter[0] % 4 == 0:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            launch[name](l)
            b.record()
            events[name].append((a, b))
        elif record == "all":
            launch[name](l)
            b = torch.cuda.Event(enable_timing=True)
            b.record()
            events[name].append((last[0], b))
            last[0] = b
        else:
            launch[name](l)

    def step(record):
        if record == "all":
            last[0] = torch.cuda.Event(enable_timing=True)
            last[0].record()
        for l in range(layers):                                   # forward
            timed("qwz_dequantize", l, record)
        for l in reversed(range(layers)):                         # backward
            for name in ("qwz_dequantize", "qgz_reorder", "qgz_intra_reduce", "qgz_inter_reduce", "qwz_quantize"):
                timed(name, l, record)

    for _ in range(args.warmup):
        step(None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step("sparse")
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    ms_per_step = elapsed * 1e3 / args.steps
    value = step_bytes / (elapsed / args.steps) / 1e9
    dom_ms = [a.elapsed_time(b) for a, b in events[DOM]]
    dom_avg = sum(dom_ms) / len(dom_ms)
    dom_launches = len(dom_ms)

    # per-kernel table: two more steps with every launch bracketed (outside the timed region)
    events = {k: [] for k in bytes_per}
    for _ in range(2):
        step("all")
    torch.cuda.synchronize()
    kernels = {}
    for k, ev in events.items():
        ms = [a.elapsed_time(b) for a, b in ev]
        avg = sum(ms) / len(ms)
        gbs = bytes_per[k] / (avg * 1e-3) / 1e9
        kernels[k] = {"bytes": bytes_per[k], "avg_ms": round(avg, 5), "min_ms": round(min(ms), 5),
                      "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                      "launches": len(ms),
                      "protocol": "inside the step, one HIP event after every launch; from the event before to the event after"}
        # vector-ALU instructions per launch from a committed rocprofv3 --pmc SQ_INSTS_VALU summary: one
        # wave64 instruction is 64 lane-operations; the chip retires 256 CUs x 4 SIMDs x 16 lanes x
        # 2.4 GHz = 39.3e12 of them per second at its peak clock
        row, source = profile_figures("bench_step_valu.txt", k, elements_per[k])
        if row is not None:
            alu = int(row["valu_insts"]) * 64 / (avg * 1e-3)
            kernels[k]["frac_of_alu_peak"] = round(alu / ALU_PEAK_LANE_OPS, 4)
            kernels[k]["bound"] = "alu" if alu / ALU_PEAK_LANE_OPS > gbs / HBM_PEAK_GBS else "hbm"
            kernels[k]["valu_insts_per_launch"] = int(row["valu_insts"])
            kernels[k]["valu_source"] = source
        else:
            kernels[k]["valu_source"] = source
        # the same kernel's duration in the committed rocprofv3 kernel trace of this benchmark (dispatch
        # time stamps, no event between the launches); an earlier run, hence with its source
        row, source = profile_figures("bench_step_kernel_stats.txt", k, elements_per[k])
        if row is not None:
            us = float(row["avg_us"])
            kernels[k]["kernel_trace"] = dict(source, avg_us=us, calls=int(row["calls"]),
                                              frac_of_hbm_peak=round(bytes_per[k] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4))
        else:
            kernels[k]["kernel_trace"] = source

    # the same step captured once into a HIP graph (kernel nodes only) and replayed
    graph = None
    if not args.no_graph:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream(device=dev)
        side.wait_stream(torch.cuda.current_stream(dev))
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                step(None)
        torch.cuda.current_stream(dev).wait_stream(side)
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        g_el = time.perf_counter() - t2
        graph = {"graph_ms_per_step": round(g_el * 1e3 / args.steps, 3),
                 "graph_GBps": round(step_bytes / (g_el / args.steps) / 1e9, 1),
                 "eager_ms_per_step": round(ms_per_step, 3), "kernel_nodes": sum(calls_per_step.values()),
                 "note": "the eager step is `value`; the step is not bound by launch rate"}
        del g

    # measured copy ceiling: 2 GiB read + 2 GiB written per launch
    src = grad.view(torch.uint8)[: 1 << 31]
    dst = wout.view(torch.uint8)[: 1 << 31]
    for _ in range(2):
        diagnostics.stream_copy(dst, src)
    ce = []
    for _ in range(5):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        diagnostics.stream_copy(dst, src)
        b.record()
        ce.append((a, b))
    torch.cuda.synchronize()
    copy_ms = min(a.elapsed_time(b) for a, b in ce)
    copy_gbs = 2 * (1 << 31) / (copy_ms * 1e-3) / 1e9

    dom = DOM
    # HBM bytes per launch from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary
    row, traffic_source = profile_figures("bench_step_hbm_traffic.txt", dom, elements_per[dom])
    traffic = int(row["bytes_per_launch"]) if row is not None else None
    dom_gbs = bytes_per[dom] / (dom_avg * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": traffic_source,
                "algorithmic_bytes_per_launch": bytes_per[dom], "avg_launch_ms": round(dom_avg, 5),
                "launches_timed": dom_launches, "copy_ceiling_GBps": round(copy_gbs, 1)}

    runner = Runner(torch, diagnostics, dev)
    # each kernel of the step alone, at the step's shapes and operands, in batches of back-to-back launches
    step_shapes = {}
    it = [0]
    for name in bytes_per:
        def one(name=name):
            it[0] += 1
            launch[name](it[0])
        step_shapes[name] = runner.run(bytes_per[name], one, batch=10 if bytes_per[name] < 2e9 else 4)

    schedules = None
    if not args.no_schedules:
        schedules = schedule_timings(torch, zpp, dev, n_L, X, Y, W, GB_, GBITS, WB, WBITS, grad, peer_sets[0],
                                     node_sets[0], own, wcodes, wscales, wout)
    del w, wout, grad, gcodes, gscales, peer_sets, node_sets, wcodes, src, dst, intra_tables, inter_tables, launch
    torch.cuda.empty_cache()
    per_config = None if args.no_configs else per_config_kernels(torch, zpp, workloads, dev, runner)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(args, n_L, X, Y, W, WB, WBITS, GB_, GBITS)

    out = {
        "metric": METRIC, "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[4]: per-step kernel sequence, one GPU's share of a {layers}-layer "
                               f"hidden-{args.hidden} GPT-style model (bf16 weights int8 block {WB}, fp16 grads "
                               f"int4 block {GB_}, X={X}, Y={Y})",
                   "layers": layers, "hidden": args.hidden, "elements_per_layer": n_L,
                   "step_algorithmic_bytes": step_bytes, "calls_per_step": calls_per_step},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "roofline": roofline, "cpu_baseline": cpu, "graph": graph, "kernels": kernels,
        "kernels_alone_at_step_shapes": step_shapes, "other_configs": per_config,
        "schedules": schedules,
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


class Runner:
    """Timing protocol of everything outside the timed step: HIP events on the launch stream around
    `batch` back-to-back launches, >= 3 warm-up launches, `rounds` batches, median / min / max of the
    per-launch time.  A 1 GiB copy is queued in front of each batch so that the host is ahead of the
    GPU when the first event is reached: short kernels are then timed at the GPU's pace, not the
    host's.  Callers rotate their operands so that inputs do not stay in the 256 MB last-level cache."""

    def __init__(self, torch, diagnostics, dev):
        self.torch, self.diagnostics = torch, diagnostics
        self.blk_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        self.blk_dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)

    def times(self, fn, batch=10, rounds=7, warm=3):
        torch = self.torch
        for _ in range(warm):
            fn()
        ev = []
        for _ in range(rounds):
            self.diagnostics.stream_copy(self.blk_dst, self.blk_src)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(batch):
                fn()
            b.record()
            ev.append((a, b))
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) / batch for a, b in ev)

    def run(self, nbytes, fn, note=None, batch=10, rounds=7, launches=1):
        ms = self.times(fn, batch, rounds)
        med = ms[len(ms) // 2]
        gbs = nbytes / (med * 1e-3) / 1e9
        res = {"bytes": int(nbytes), "median_us": round(med * 1e3, 2), "min_us": round(ms[0] * 1e3, 2),
               "max_us": round(ms[-1] * 1e3, 2), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
               "launches_per_sample": batch * launches, "samples": rounds}
        if note:
            res["note"] = note
        return res


def schedule_timings(torch, zpp, dev, n_L, X, Y, W, GB_, GBITS, WB, WBITS, grad, peers, nodes, own, wcodes, wscales,
                     wout):
    """Sec. 4.1 schedules at the benchmark's layer size: (a) the gradient path of one layer cut
    into S pipeline stages, on one stream and with the two hops on two streams; (b) eight layers
    of the forward weight path with the next layer's shard quantization on a side stream.
    Protocol: all variants of a family are built first and then timed interleaved (variant 1,
    2, ..., variant 1, 2, ...), 3 warm-up rounds, 20 timed rounds; every variant moves several GB
    per run, so between two runs of one variant the last-level cache has been turned over many
    times.  min / median / max in ms."""
    from paper_2306_10209_amd.schedule import QgzPipeline, QwzPrefetch

    def interleaved(variants, warm=3, reps=20):
        for _ in range(warm):
            for fn in variants.values():
                fn()
        ev = {k: [] for k in variants}
        for _ in range(reps):
            for k, fn in variants.items():
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                ev[k].append((a, b))
        torch.cuda.synchronize()
        out = {}
        for k, pairs in ev.items():
            ms = sorted(a.elapsed_time(b) for a, b in pairs)
            out[k] = {"min": round(ms[0], 4), "median": round(ms[len(ms) // 2], 4), "max": round(ms[-1], 4)}
        return out

    res = {"protocol": "variants interleaved, 3 warm-up rounds, 20 timed rounds, HIP events; ms"}
    nc, ns = nodes
    out = torch.empty(n_L // W, dtype=torch.float32, device=dev)
    pipes = {}
    for S in (1, 2, 4):
        for two in (False, True):
            pipe = QgzPipeline(n_L, X, Y, S, GB_, GBITS, device=dev, two_streams=two)
            pipe.bind(0, 0, peers, list(zip(nc, ns)))
            pipes[f"S={S},{'two_streams' if two else 'one_stream'}"] = pipe
    res["qgz_pipeline_ms_per_layer"] = interleaved({k: (lambda p=p: p.run(grad, out, float(W))) for k, p in pipes.items()})
    del pipes
    L = n_L // W
    scheds = {}
    for overlap in (False, True):
        sched = QwzPrefetch(n_L, L, 0, WB, WBITS, device=dev, overlap=overlap)
        for slot in range(2):
            sched.gather_codes[slot].copy_(wcodes)
            sched.gather_scales[slot].copy_(wscales)
        scheds["overlapped" if overlap else "serial"] = sched
    res["qwz_prefetch_ms_8_layers"] = interleaved({k: (lambda s=s: s.run([own] * 8, [wout] * 8)) for k, s in scheds.items()})
    return res


def per_config_kernels(torch, zpp, workloads, dev, runner):
    """Each kernel alone at the shapes of configs[0..3], and the paths for block sizes that are not
    powers of two; protocol: Runner."""
    res = {}

    def run(name, nbytes, fn, note=None, **kw):
        res[name] = runner.run(nbytes, fn, note, **kw)

    # configs[0]: one fp16 4096x256 tensor, int8 block 256 (3 MB: launch-latency bound, cache resident)
    n = 1 << 20
    x = workloads.weights(n, device=dev, tensor_id=30, dtype=torch.float16, outlier_prob=0.0)
    c, s = zpp.qwz_quantize(x, 256, 8)
    note = "3 MB per launch: bounded by launch latency, resident in cache; parity configuration"
    run("cfg0.qwz_quantize", Bytes.quantize(n, 256, 8), lambda: zpp.qwz_quantize(x, 256, 8, codes=c, scales=s), note)
    run("cfg0.qwz_dequantize", Bytes.dequantize(n, 256, 8), lambda: zpp.qwz_dequantize(c, s, n, 256, 8, out=x), note)
    # the same kernels on 1024 such tensors in one launch
    n = 1024 << 20
    x = workloads.weights(n, device=dev, tensor_id=30, dtype=torch.float16, outlier_prob=0.0)
    c, s = zpp.qwz_quantize(x, 256, 8)
    run("cfg0x1024.qwz_quantize", Bytes.quantize(n, 256, 8), lambda: zpp.qwz_quantize(x, 256, 8, codes=c, scales=s))
    run("cfg0x1024.qwz_dequantize", Bytes.dequantize(n, 256, 8), lambda: zpp.qwz_dequantize(c, s, n, 256, 8, out=x))
    del x, c, s

    # configs[1]: one layer, hidden 8192, bf16, P = 8 shards per matrix, int8 block 2048
    P, B = 8, 2048
    shapes = workloads.gpt_layer_shapes(8192)
    n_total = sum(r * c_ for _, r, c_ in shapes)
    w = workloads.weights(n_total, device=dev, tensor_id=10)
    codes = torch.empty(n_total, dtype=torch.uint8, device=dev)
    scales = torch.empty(n_total // B, dtype=torch.float32, device=dev)
    shards, off = [], 0          # (offset, length, simulated rank)
    for _, r, c_ in shapes:
        sh = r * c_ // P
        for rank in range(P):
            shards.append((off + rank * sh, sh, rank))
        off += r * c_

    def quantize_shard(lo, sh, stream=None):
        zpp.qwz_quantize(w[lo:lo + sh], B, 8, codes=codes[lo:lo + sh], scales=scales[lo // B:(lo + sh) // B], stream=stream)

    def quantize_layer():
        for lo, sh, _ in shards:
            quantize_shard(lo, sh)

    nb = Bytes.quantize(n_total, B, 8)
    run("cfg1.qwz_quantize_32_shards", nb, quantize_layer,
        "32 launches (8 rank shards x 4 matrices) on one stream, written at their offsets of the gather buffer",
        batch=2, launches=32)
    # The 8 simulated ranks are 8 independent processes in the method, so their launches carry no
    # order among each other.  One GPU stands in for all of them here: the launches of different
    # ranks go to 4 streams (the hardware queues a process has), rank r on stream r % 4, each
    # rank's four shards in order.  This is the recorded protocol for configs[1].
    streams = [torch.cuda.Stream(device=dev) for _ in range(4)]

    def quantize_layer_rank_streams():
        main = torch.cuda.current_stream(dev)
        for st in streams:
            st.wait_stream(main)
        for lo, sh, rank in shards:
            quantize_shard(lo, sh, streams[rank % 4])
        for st in streams:
            main.wait_stream(st)

    run("cfg1.qwz_quantize_32_shards_rank_streams", nb, quantize_layer_rank_streams,
        "recorded protocol for configs[1]: the same 32 launches, simulated rank r on stream r % 4 "
        "(ranks are independent processes in the method), fork and join through events", batch=2, launches=32)
    # both sequences captured into HIP graphs (kernel nodes only) and replayed
    cap = torch.cuda.Stream(device=dev)
    for key, fn in (("cfg1.qwz_quantize_32_shards_graph", quantize_layer),
                    ("cfg1.qwz_quantize_32_shards_rank_streams_graph", quantize_layer_rank_streams)):
        g = torch.cuda.CUDAGraph()
        cap.wait_stream(torch.cuda.current_stream(dev))
        with torch.cuda.stream(cap):
            with torch.cuda.graph(g, stream=cap):
                fn()
        torch.cuda.current_stream(dev).wait_stream(cap)
        run(key, nb, g.replay, "the sequence above captured once into a HIP graph and replayed", batch=2, launches=32)
        del g
    run("cfg1.qwz_dequantize_layer", Bytes.dequantize(n_total, B, 8),
        lambda: zpp.qwz_dequantize(codes, scales, n_total, B, 8, out=w), batch=4)
    del w, codes, scales

    # configs[2]: 8 ranks x 2^28 fp16 heavy-tailed gradients, X = 8, Y = 64, int4 block 512
    X, Y, B = 8, 64, 512
    n = 1 << 28
    m = n // X
    grads = [workloads.gradients(n, device=dev, tensor_id=40 + r) for r in range(X)]
    first = [zpp.qgz_reorder(g, X, Y, 1, B, 4) for g in grads]
    it = [0]

    def reorder_one():
        r = it[0] % X
        it[0] += 1
        zpp.qgz_reorder(grads[r], X, Y, 1, B, 4, codes=first[r][0], scales=first[r][1])

    run("cfg2.qgz_reorder_per_rank", Bytes.quantize(n, B, 4), reorder_one)
    co = torch.empty(m // 2, dtype=torch.uint8, device=dev)
    so = torch.empty(m // B, dtype=torch.float32, device=dev)
    cb, sb = m // 2, m // B

    tables = [zpp.PeerTable([f[0][j * cb:(j + 1) * cb] for f in first], [f[1][j * sb:(j + 1) * sb] for f in first])
              for j in range(X)]

    def intra_one():
        j = it[0] % X
        it[0] += 1
        zpp.qgz_intra_reduce(tables[j], None, m, B, 4, codes_out=co, scales_out=so)

    run("cfg2.qgz_intra_reduce_per_rank", Bytes.intra(m, B, 4, X), intra_one)

    # the paths that parity tests cover for other block sizes, at the same sizes: a block that is not a
    # power of two (1536 = 3 x 512), the int4 intra-node stage with the largest block (4096), and the
    # inter-node stage with a block that is not a whole number of 16-lane rows (96)
    GBk = 1536
    ng = n - n % (X * Y * GBk)
    gq = grads[0][:ng]
    qc = torch.empty(ng // 2, dtype=torch.uint8, device=dev)
    qs = torch.empty(ng // GBk, dtype=torch.float32, device=dev)
    note = "block 1536: the path for blocks that are not powers of two"
    run("generic.qgz_reorder_block1536", Bytes.quantize(ng, GBk, 4), lambda: zpp.qgz_reorder(gq, X, Y, 1, GBk, 4, codes=qc, scales=qs), note)
    gy = torch.empty(ng, dtype=torch.float16, device=dev)
    run("generic.qwz_dequantize_block1536", Bytes.dequantize(ng, GBk, 4), lambda: zpp.qwz_dequantize(qc, qs, ng, GBk, 4, out=gy), note)
    del gy
    mg = m - m % GBk
    for blk, key in ((GBk, "generic.qgz_intra_reduce_block1536"), (4096, "generic.qgz_intra_reduce_block4096")):
        mm = m - m % blk
        enc = [zpp.qwz_quantize(grads[k][:mm], blk, 4) for k in range(X)]
        tb = zpp.PeerTable([e[0] for e in enc], [e[1] for e in enc])
        run(key, Bytes.intra(mm, blk, 4, X),
            lambda: zpp.qgz_intra_reduce(tb, None, mm, blk, 4, codes_out=co, scales_out=so),
            "one wave per block, its sums in registers between the maximum and the encode")
        del enc, tb
    Lg = 4718592                                            # the step's inter-node size, a multiple of 1536
    enc = [zpp.qwz_quantize(grads[k % X][(k // X) * Lg:(k // X + 1) * Lg], GBk, 4) for k in range(48)]
    tb = zpp.PeerTable([e[0] for e in enc], [e[1] for e in enc])
    og = torch.empty(Lg, dtype=torch.float32, device=dev)
    run("generic.qgz_inter_reduce_block1536", Bytes.inter(Lg, GBk, 4, 48),
        lambda: zpp.qgz_inter_reduce(tb, None, Lg, GBk, 4, 384.0, out=og),
        "12 rows of 16 lanes per block: the kernel of the power-of-two blocks, block index by a prepared division")
    del enc, tb
    enc = [zpp.qwz_quantize(grads[k % X][(k // X) * Lg:(k // X + 1) * Lg], 96, 4) for k in range(48)]
    tb = zpp.PeerTable([e[0] for e in enc], [e[1] for e in enc])
    run("generic.qgz_inter_reduce_block96", Bytes.inter(Lg, 96, 4, 48),
        lambda: zpp.qgz_inter_reduce(tb, None, Lg, 96, 4, 384.0, out=og), "every lane fetches its own scales")
    del enc, tb, og, gq, qc, qs

    # the variants the same entry points take by argument, at the same sizes: the gradient path with int8
    # codes, the one-hop reduction (the second-hop kernel over all ranks at once: 64 of them here, the most
    # one call takes), and the weight path with int4 codes and with fp32 weights
    g8 = [zpp.qgz_reorder(g, X, Y, 1, B, 8) for g in grads[:2]]
    run("variants.qgz_reorder_int8", Bytes.quantize(n, B, 8),
        lambda: zpp.qgz_reorder(grads[0], X, Y, 1, B, 8, codes=g8[0][0], scales=g8[0][1]))
    co8 = torch.empty(m, dtype=torch.uint8, device=dev)
    tb = zpp.PeerTable([g8[k % 2][0][(k // 2) * m:(k // 2 + 1) * m] for k in range(X)],
                       [g8[k % 2][1][(k // 2) * sb:(k // 2 + 1) * sb] for k in range(X)])
    run("variants.qgz_intra_reduce_int8", Bytes.intra(m, B, 8, X),
        lambda: zpp.qgz_intra_reduce(tb, None, m, B, 8, codes_out=co8, scales_out=so),
        "int8 blocks of 512 and more take the wave-per-block kernel")
    og = torch.empty(Lg, dtype=torch.float32, device=dev)
    tb = zpp.PeerTable([g8[k % 2][0][(k // 2) * Lg:(k // 2 + 1) * Lg] for k in range(48)],
                       [g8[k % 2][1][(k // 2) * (Lg // B):(k // 2 + 1) * (Lg // B)] for k in range(48)])
    run("variants.qgz_inter_reduce_int8", Bytes.inter(Lg, B, 8, 48),
        lambda: zpp.qgz_inter_reduce(tb, None, Lg, B, 8, 384.0, out=og))
    del g8, co8, tb
    tb = zpp.PeerTable([first[k % X][0][(k // X) * (Lg // 2):(k // X + 1) * (Lg // 2)] for k in range(64)],
                       [first[k % X][1][(k // X) * (Lg // B):(k // X + 1) * (Lg // B)] for k in range(64)])
    run("variants.qgz_inter_reduce_one_hop_64_ranks", Bytes.inter(Lg, B, 4, 64),
        lambda: zpp.qgz_inter_reduce(tb, None, Lg, B, 4, 64.0, out=og), "Sec. 3.3.1: every rank's slice reduced in one hop")
    del tb, og, grads, first, co, so, tables
    wn = 1 << 28
    wb = workloads.weights(wn, device=dev, tensor_id=12)
    c4, s4 = zpp.qwz_quantize(wb, 2048, 4)
    run("variants.qwz_quantize_int4", Bytes.quantize(wn, 2048, 4), lambda: zpp.qwz_quantize(wb, 2048, 4, codes=c4, scales=s4))
    run("variants.qwz_dequantize_int4", Bytes.dequantize(wn, 2048, 4), lambda: zpp.qwz_dequantize(c4, s4, wn, 2048, 4, out=wb))
    del wb, c4, s4
    wf = workloads.weights(wn, device=dev, tensor_id=13, dtype=torch.float32)
    c8, s8 = zpp.qwz_quantize(wf, 2048, 8)
    run("variants.qwz_quantize_fp32_weights", Bytes.quantize(wn, 2048, 8, in_bytes=4),
        lambda: zpp.qwz_quantize(wf, 2048, 8, codes=c8, scales=s8))
    run("variants.qwz_dequantize_to_fp32", Bytes.dequantize(wn, 2048, 8, out_bytes=4),
        lambda: zpp.qwz_dequantize(c8, s8, wn, 2048, 8, out=wf))
    del wf, c8, s8

    # configs[3]: 48 node chunks of 46,875,136 elements (46,875,000 padded to the block), int4 block 512.
    # The chunks sit one after the other in one receive buffer for the codes and one for the scales, as
    # an all-to-all leaves them (48 separate allocations measured 5 % slower: more pages per wave).
    Y, L = 48, 46875136
    rc = torch.empty(Y * L // 2, dtype=torch.uint8, device=dev)
    rs = torch.empty(Y * L // B, dtype=torch.float32, device=dev)
    for i in range(Y):
        g = workloads.gradients(L, device=dev, tensor_id=60 + i, tail_std=0.0)
        zpp.qwz_quantize(g, B, 4, codes=rc[i * L // 2:(i + 1) * L // 2], scales=rs[i * L // B:(i + 1) * L // B])
        del g
    out = torch.empty(L, dtype=torch.float32, device=dev)
    table = zpp.PeerTable([rc[i * L // 2:(i + 1) * L // 2] for i in range(Y)], [rs[i * L // B:(i + 1) * L // B] for i in range(Y)])
    run("cfg3.qgz_inter_reduce", Bytes.inter(L, B, 4, Y),
        lambda: zpp.qgz_inter_reduce(table, None, L, B, 4, 384.0, out=out), batch=4)
    return res


def cpu_baseline(args, n_L, X, Y, W, WB, WBITS, GB_, GBITS):
    """The CPU oracle, as it stands, on 1/div of one layer pushed through the same
    six calls a layer costs in a step (2 dequantize, reorder, intra, inter, quantize):
    on all host threads (best of 3, outputs allocated and touched beforehand), and on
    1/16 of that sample with one thread (whose outputs must be the bytes the threaded
    run gives for the same sample)."""
    import numpy as np
    import torch
    import oracle
    from paper_2306_10209_amd import workloads

    gen = "cuda:0" if torch.cuda.is_available() else "cpu"     # drawing the numbers is not part of the baseline

    def prepare(n):
        assert n % (X * Y * GB_) == 0 and (n // W) % WB == 0
        m, L = n // X, n // W
        w = workloads.as_bits(workloads.weights(n, device=gen, tensor_id=1))
        wc, ws = oracle.qwz_quantize(w, oracle.BF16, WB, WBITS)
        g = workloads.as_bits(workloads.gradients(n, device=gen, tensor_id=3, tail_std=0.0))
        peers = [oracle.qwz_quantize(workloads.as_bits(workloads.gradients(m, device=gen, tensor_id=100 + k, tail_std=0.0)),
                                     oracle.F16, GB_, GBITS) for k in range(X - 1)]
        nodes = [oracle.qwz_quantize(workloads.as_bits(workloads.gradients(L, device=gen, tensor_id=200 + i, tail_std=0.0)),
                                     oracle.F16, GB_, GBITS) for i in range(Y - 1)]
        own = workloads.as_bits(workloads.weights(L, device=gen, tensor_id=2))
        outs = {"y": np.zeros(n, np.uint16), "gc": np.zeros(n // 2, np.uint8), "gs": np.zeros(n // GB_, np.float32),
                "ic": np.zeros(m // 2, np.uint8), "is": np.zeros(m // GB_, np.float32), "o": np.zeros(L, np.float32),
                "qc": np.zeros(L, np.uint8), "qs": np.zeros(L // WB, np.float32)}
        return n, wc, ws, g, peers, nodes, own, outs

    def six(inp):
        n, wc, ws, g, peers, nodes, own, o = inp
        m, L = n // X, n // W
        t0 = time.perf_counter()
        oracle.qwz_dequantize(wc, ws, n, WB, WBITS, oracle.BF16, out=o["y"])
        oracle.qwz_dequantize(wc, ws, n, WB, WBITS, oracle.BF16, out=o["y"])
        oracle.qgz_reorder(g, oracle.F16, X, Y, 1, GB_, GBITS, codes=o["gc"], scales=o["gs"])
        oracle.qgz_intra_reduce([o["gc"][:m // 2]] + [p[0] for p in peers], [o["gs"][:m // GB_]] + [p[1] for p in peers],
                                m, GB_, GBITS, codes=o["ic"], scales=o["is"])
        oracle.qgz_inter_reduce([o["ic"][:L // 2]] + [c for c, _ in nodes], [o["is"][:L // GB_]] + [s for _, s in nodes],
                                L, GB_, GBITS, float(W), out=o["o"])
        oracle.qwz_quantize(own, oracle.BF16, WB, WBITS, codes=o["qc"], scales=o["qs"])
        dt = time.perf_counter() - t0
        return dt, six_bytes(n), [v.copy() for v in o.values()]

    def six_bytes(n):
        m, L = n // X, n // W
        return (2 * Bytes.dequantize(n, WB, WBITS) + Bytes.quantize(n, GB_, GBITS) + Bytes.intra(m, GB_, GBITS, X)
                + Bytes.inter(L, GB_, GBITS, Y) + Bytes.quantize(L, WB, WBITS))

    div = args.cpu_sample_div
    threads = oracle.set_threads(0)
    inp = prepare(n_L // div)
    runs = [six(inp)[0] for _ in range(3)]
    dt = min(runs)
    nbytes = six_bytes(n_L // div)
    res = {"value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
           "sample": f"1/{div} of one layer ({n_L // div} elements) through the six calls a layer costs per step "
                     f"(= 1/{div * args.layers} of a step); best of 3 runs of {dt:.1f} s "
                     f"({', '.join(f'{r:.2f}' for r in runs)} s), outputs allocated beforehand",
           "seconds": round(dt, 2)}
    del inp
    small = prepare(n_L // (16 * div))
    _, _, threaded = six(small)
    oracle.set_threads(1)
    dt1, nbytes1, single = six(small)
    oracle.set_threads(threads)
    res["single_thread"] = {"value": round(nbytes1 / dt1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                            "sample": f"1/{16 * div} of one layer ({n_L // (16 * div)} elements), {dt1:.1f} s",
                            "same_bytes_as_threaded": all(np.array_equal(a.view(np.uint8), b.view(np.uint8))
                                                          for a, b in zip(threaded, single))}
    return res


if __name__ == "__main__":
    main()
