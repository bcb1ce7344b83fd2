#!/usr/bin/env python3
"""Benchmark of the Adacc hot path on one MI355X: compress + decompress of saved bf16
activations (Section 3.2) through libadacc, next to the CPU oracle timed on the host.

A step = one compression and one decompression of the workload (every row of the hot-path
table: load, statistics, outlier mask, ordered compaction, scale, quantise, pack, and on the
way back unpack, dequantise, outlier patch, store).  Inputs are generated once and are
resident in HBM before the timed region.  Several buffer sets are rotated and a step
decompresses a blob that was compressed in another step, so that neither call reads its input
from the 256 MB Infinity Cache.

The headline workload is C5, the largest configuration that fits one GPU: the saved tensors of
32 LLaMA-7B-shaped layers (20 GiB of bf16), compressed by one batched call and restored by one
batched call.  The other configurations, the layer-specific schemes (outlier channels, dropout
mask, channel-wise Q/K/V) and the stream ceilings of the part follow as short runs in the same
JSON line, each with a roofline block of its own.

Prints ONE JSON line.  value = bytes of bf16 activations compressed plus bytes restored,
per second (GB/s, 1e9), whole job.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published peak HBM3E bandwidth

WORKLOAD_TEXT = {
    "c1": "c1: single activation [4096,1024] bf16, int8 per-row absmax, outliers |x|>6*row_std",
    "c2": "c2: GPT-1.3B-shaped [16x2048,2048] bf16, int4 group-128 absmax, top-2 outliers per 2048-row",
    "c3": "c3: MLP GELU output [8x2048,16384] bf16, int8 group-64, outliers at 8*group_std",
    "c4": "c4: attention softmax [4,32,2048,2048] bf16, asymmetric int8 per row, outliers > 0.05",
    "c5": "c5: LLaMA-7B-shaped layer set, 32 layers x 5 tensors at batch 2 x seq 4096, batched launch",
    # second readings of two configurations (same tensors, another method)
    "c2b": "c2 read as top-1 of every 128-group: [16x2048,2048] bf16, int4 group-128, top-1 per 128",
    "c4b": "c4 with symmetric codes: [4,32,2048,2048] bf16, symmetric int8 per row, outliers > 0.05",
    # the paper's own formats (Section 3.2: FP16 activations to INT4): c2's tensor and method in binary16
    "c2h": "c2 in binary16 (FP16 -> INT4): [16x2048,2048] float16, int4 group-128 absmax, top-2 outliers per 2048-row",
}
# name -> (configuration whose tensor it takes, method or None for that configuration's own, 16-bit format: 0 bf16, 1 binary16)
SECOND_READINGS = {
    "c2b": ("c2", dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=128, thresh=0.0, topk=1), 0),
    "c4b": ("c4", dict(bits=8, quant_group=2048, asym=0, outlier_mode="abs", stat_group=0, thresh=0.05, topk=0), 0),
    "c2h": ("c2", None, 1),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (0 = enough to exceed 1 GiB)")
    ap.add_argument("--no-extras", action="store_true", help="skip the short runs of the other workloads and schemes")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--cpu-seconds", type=float, default=16.0, help="about this much CPU time for the oracle")
    ap.add_argument("--only-channelwise", action="store_true",
                    help="run only the channel-wise (Q/K/V) quantisation measurement and print its JSON")
    ap.add_argument("--only-mask", action="store_true",
                    help="run only the dropout-mask (byte <-> bit) measurement and print its JSON")
    ap.add_argument("--only-channel", action="store_true",
                    help="run only the outlier-channel (Z-score) measurement and print its JSON")
    ap.add_argument("--only-streams", action="store_true",
                    help="run only the read / write / copy / 2R:1W stream probes and print their JSON")
    return ap.parse_args()


def measured_traffic():
    """HBM bytes per call from profiles/hbm_traffic_pmc.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
    this file, scaled by the copy kernel).  Lines of the form `traffic <workload> <compress|decompress> <bytes>`."""
    out = {}
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")) as f:
            for line in f:
                m = re.match(r"^traffic\s+(\S+)\s+(compress|decompress)\s+(\d+)\s*$", line)
                if m:
                    out[(m.group(1), m.group(2))] = int(m.group(3))
    except OSError:
        pass
    return out


class Workload:
    """Device buffers of one workload: `sets` rotating copies of (inputs, blobs, outputs)."""

    def __init__(self, name, sets):
        import torch
        import workloads
        import paper_2508_00806_amd as adacc
        self.name = name
        self.adacc = adacc
        if name == "c5":
            specs = [(f"L{layer}.{tname}", x.shape[-1], md, x) for layer, tname, x, md in workloads.c5("cuda")]
        else:
            base, md, fmt = SECOND_READINGS.get(name, (name, None, 0))
            x = workloads.make(base, "cuda")
            if fmt == 1:
                x = x.to(torch.float16)
            specs = [(name, x.shape[-1], md or workloads.METHODS[base], x)]
        self.mds = [s[2] for s in specs]
        self.numels = [s[3].numel() for s in specs]
        self.methods = [adacc.method_from_dict(md, workloads.outlier_capacity(md, n, h),
                                               dtype=adacc.DTYPE_F16 if x.dtype == torch.float16 else adacc.DTYPE_BF16)
                        for (_, h, md, x), n in zip(specs, self.numels)]
        self.layouts = [adacc.layout_of(m, n) for m, n in zip(self.methods, self.numels)]
        self.batched = len(specs) > 1
        in_bytes = sum(2 * n for n, md in zip(self.numels, self.mds) if md is not None)
        if sets <= 0:  # at least 1 GiB of inputs in rotation (the Infinity Cache holds 256 MB), at most 64 sets
            sets = max(2, min(64, -(-(1 << 30) // max(in_bytes, 1))))
            sets += sets % 2
        if name == "c5":
            sets = 2  # 20 GiB per set: far beyond any cache already
        self.sets = sets
        self.src, self.blob, self.dst = [], [], []
        for s in range(sets):
            self.src.append([sp[3].view(-1) if s == 0 else sp[3].view(-1).clone() for sp in specs])
            self.blob.append([None if md is None else adacc.alloc_blob(m, n)[0]
                              for m, n, md in zip(self.methods, self.numels, self.mds)])
            self.dst.append([None if md is None else torch.empty(n, dtype=sp[3].dtype, device="cuda")
                             for n, md, sp in zip(self.numels, self.mds, specs)])
        if self.batched:
            wsb = adacc.batch_workspace_bytes(self.methods, self.numels)
        else:
            wsb = adacc.workspace_bytes(self.methods[0], self.numels[0])
        self.ws = adacc.alloc_workspace(max(wsb, 512))
        if self.batched:  # the argument arrays of the batch calls, marshalled once per buffer set
            self.cargs = [adacc.prepare_compress_batch(self.methods, self.src[s], self.blob[s]) for s in range(sets)]
            self.dargs = [adacc.prepare_decompress_batch(self.methods, self.blob[s], self.dst[s]) for s in range(sets)]
        self.act_bytes = in_bytes
        self.n_out = None

    def compress(self, s):
        a = self.adacc
        if self.batched:
            a.compress_batch(self.methods, self.src[s], self.blob[s], self.ws, prepared=self.cargs[s])
        else:
            a.compress(self.methods[0], self.src[s][0], self.blob[s][0], self.ws)

    def decompress(self, s):
        a = self.adacc
        if self.batched:
            a.decompress_batch(self.methods, self.blob[s], self.dst[s], self.ws, prepared=self.dargs[s])
        else:
            a.decompress(self.methods[0], self.blob[s][0], self.dst[s][0])

    def algorithmic_bytes(self):
        """Per direction: bf16 tensor once + codes + scales/offsets + outliers produced + tile offsets."""
        import workloads
        if self.n_out is None:
            self.n_out = [0 if md is None else self.adacc.read_status(b, L)[0]
                          for md, b, L in zip(self.mds, self.blob[0], self.layouts)]
        return sum(workloads.algorithmic_bytes(md, n, k, L.n_tiles)
                   for md, n, k, L in zip(self.mds, self.numels, self.n_out, self.layouts))

    def check_status(self):
        """Every blob of every buffer set: no overflow of the outlier stream, and the same count in all sets."""
        for s in range(self.sets):
            for i, (md, b, L) in enumerate(zip(self.mds, self.blob[s], self.layouts)):
                if md is None:
                    continue
                st = self.adacc.read_status(b, L)
                if st[1] or st[2]:
                    raise RuntimeError(f"{self.name}: set {s} tensor {i}: compression reported overflow: {st}")
                if s and st[0] != self.adacc.read_status(self.blob[0][i], L)[0]:
                    raise RuntimeError(f"{self.name}: set {s} tensor {i}: outlier count differs between buffer sets")


def time_steps(w, steps, warmup):
    """Returns (ms per step, ms per compress call, ms per decompress call, wall ms per step).  Events are
    recorded on the stream the library launches on (torch's current stream), inside the timed region."""
    import torch
    half = w.sets // 2
    for s in range(w.sets):       # every blob exists before a decompress reads it
        w.compress(s)
    for i in range(warmup):
        w.compress(i % w.sets)
        w.decompress((i + half) % w.sets)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i][0].record()
        w.compress(i % w.sets)
        ev[i][1].record()
        w.decompress((i + half) % w.sets)
        ev[i][2].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    total_ms = ev[0][0].elapsed_time(ev[-1][2])
    c_all = sorted(e[0].elapsed_time(e[1]) for e in ev)
    d_all = sorted(e[1].elapsed_time(e[2]) for e in ev)
    spread = {"compress": {"ms_median": c_all[len(c_all) // 2], "ms_min": c_all[0]},
              "decompress": {"ms_median": d_all[len(d_all) // 2], "ms_min": d_all[0]}}
    return total_ms / steps, sum(c_all) / steps, sum(d_all) / steps, wall_ms / steps, spread


def direction_block(alg, ms, act_bytes, traffic):
    gbps = alg / (ms * 1e-3) / 1e9
    return {"ms": ms, "activation_GBps": act_bytes / (ms * 1e-3) / 1e9, "hbm_GBps": gbps,
            "frac_of_peak": gbps / HBM_PEAK_GBPS, "algorithmic_bytes": alg, "traffic": traffic}


def roofline_block(res):
    """The slower of the two calls of a workload against the HBM peak."""
    dom = "compress" if res["compress"]["ms"] >= res["decompress"]["ms"] else "decompress"
    r = res[dom]
    return {"bound": "hbm", "kernel": f"{res['workload']} {dom} call", "achieved": r["hbm_GBps"], "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": r["frac_of_peak"], "traffic": r["traffic"],
            "algorithmic_bytes_per_launch": r["algorithmic_bytes"], "ms_per_launch": r["ms"]}


def run_workload(name, steps, warmup, sets, cold=True):
    import torch
    w = Workload(name, sets if cold else 1)
    if not cold:
        w.sets = 1
    ms, c_ms, d_ms, wall_ms, spread = time_steps(w, steps, warmup)
    w.check_status()
    alg = w.algorithmic_bytes()
    traffic = measured_traffic()
    res = {
        "workload": name,
        "description": WORKLOAD_TEXT[name],
        "ms_per_step": ms,
        "wall_ms_per_step": wall_ms,
        "activation_GBps": 2.0 * w.act_bytes / (ms * 1e-3) / 1e9,
        "compress": direction_block(alg, c_ms, w.act_bytes, traffic.get((name, "compress"))),
        "decompress": direction_block(alg, d_ms, w.act_bytes, traffic.get((name, "decompress"))),
        "roundtrip_hbm_frac_of_peak": 2.0 * alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "activation_bytes": w.act_bytes,
        "n_outliers": int(sum(w.n_out)),
        "tensors": len(w.methods),
        "buffer_sets": w.sets,
        "cache_state": "cold: rotating buffer sets, inputs come from HBM" if cold else "warm: one buffer set, 8 MB stays in the caches",
    }
    res["compress"].update(spread["compress"])
    res["decompress"].update(spread["decompress"])
    res["roofline"] = roofline_block(res)
    del w
    torch.cuda.empty_cache()
    return res


def run_graph_replay(name, replays=6):
    """The same calls replayed from captured HIP graphs (one graph holds the compressions of all buffer sets,
    another the decompressions): what a launch-bound caller gets for small tensors."""
    import torch
    w = Workload(name, 0)
    half = w.sets // 2
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # every blob exists, and everything has run once, before the capture
        for s in range(w.sets):
            w.compress(s)
        for s in range(w.sets):
            w.decompress((s + half) % w.sets)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g_c, g_d = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_c):
        for s in range(w.sets):
            w.compress(s)
    with torch.cuda.graph(g_d):
        for s in range(w.sets):
            w.decompress((s + half) % w.sets)
    torch.cuda.synchronize()
    g_c.replay(); g_d.replay()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(replays):
        g_c.replay()
    ev[1].record()
    for _ in range(replays):
        g_d.replay()
    ev[2].record()
    torch.cuda.synchronize()
    calls = replays * w.sets
    c_ms, d_ms = ev[0].elapsed_time(ev[1]) / calls, ev[1].elapsed_time(ev[2]) / calls
    w.check_status()
    alg = w.algorithmic_bytes()
    res = {
        "workload": f"{name} (graph replay)",
        "description": WORKLOAD_TEXT[name] + "; the calls of all buffer sets captured in two HIP graphs and replayed",
        "ms_per_step": c_ms + d_ms,
        "activation_GBps": 2.0 * w.act_bytes / ((c_ms + d_ms) * 1e-3) / 1e9,
        "compress": direction_block(alg, c_ms, w.act_bytes, None),
        "decompress": direction_block(alg, d_ms, w.act_bytes, None),
        "buffer_sets": w.sets,
        "cache_state": "cold: rotating buffer sets, inputs come from HBM",
    }
    res["roofline"] = roofline_block(res)
    del w, g_c, g_d
    torch.cuda.empty_cache()
    return res


def stream_ceilings():
    """What a kernel that only moves bytes reaches on this part, in the access shape of the library's
    tensor kernels, for four mixes of reads and writes at 1 GiB per operand (GB/s of bytes moved)."""
    import torch
    import paper_2508_00806_amd as adacc
    n = 1 << 30
    a = [torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(2)]
    b = [torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(2)]
    d = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(2)]
    out = {}
    for key, mix, moved in (("read", adacc.STREAM_READ, 1), ("write", adacc.STREAM_WRITE, 1),
                            ("copy_1r1w", adacc.STREAM_COPY, 2), ("2r1w", adacc.STREAM_READ2_WRITE, 3)):
        for i in range(3):
            adacc.hbm_stream(mix, d[i % 2], a[i % 2], b[i % 2], n)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record()
        for i in range(reps):
            adacc.hbm_stream(mix, d[i % 2], a[i % 2], b[i % 2], n)
        e1.record()
        torch.cuda.synchronize()
        gbps = moved * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        out[key] = {"GBps": gbps, "frac_of_peak": gbps / HBM_PEAK_GBPS}
    del a, b, d
    torch.cuda.empty_cache()
    return out


def bits_of(t):
    """bf16 torch tensor (any device) -> numpy uint16 bit patterns, for the oracle."""
    import numpy as np
    import torch
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)


def host_description():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    usable = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
    return {"cpu_model": model, "os_cpu_count": os.cpu_count(), "usable_cores": usable}


def cpu_baseline(name, seconds):
    """The oracle as it stands on a bounded sample of the same workload: on one thread, and on all host
    cores (row blocks of the sample handed to a pool of threads; the oracle's C code runs outside the
    interpreter lock, and every group lies inside a row, so the blocks are independent)."""
    from concurrent.futures import ThreadPoolExecutor
    import numpy as np
    import torch
    import workloads
    import oracle
    host = host_description()
    cores = max(1, min(int(os.environ.get("OMP_NUM_THREADS", host["usable_cores"])), host["usable_cores"]))
    if name == "c5":
        rows = 2048
        parts = [(workloads.c5_tensor(t, "cpu", rows=rows), md) for t, _h, md in workloads.C5_LAYER if md is not None]
        sample = f"first {rows} rows of each of the 4 compressed tensors of layer 0"
    else:
        base, md2, fmt = SECOND_READINGS.get(name, (name, None, 0))
        rows = {"c1": 4096, "c2": 4096, "c3": 512, "c4": 4096}[base]
        x = workloads.make(base, "cpu", rows=rows)
        if fmt == 1:
            x = x.to(torch.float16)
        parts = [(x, md2 or workloads.METHODS[base])]
        sample = f"{rows} rows ({x.numel()} elements) of the workload, same generator"
    work = []  # (method, bits of a block of whole rows)
    total = 0
    for x, md in parts:
        b = bits_of(x).reshape(x.shape[0], -1)
        total += b.size
        om = oracle.method_from_dict(md, 0, 1 if x.dtype == torch.float16 else 0)
        step = max(1, b.shape[0] // (4 * cores))
        step += (-step) % max(1, -(-md["stat_group"] // b.shape[1]))  # whole statistics groups per block
        for r0 in range(0, b.shape[0], step):
            work.append((om, np.ascontiguousarray(b[r0:r0 + step]).reshape(-1)))

    def one(item):
        c = oracle.compress(item[0], item[1])
        oracle.decompress(c)

    def timed(threads):
        reps, t0 = 0, time.perf_counter()
        with ThreadPoolExecutor(max_workers=threads) as pool:
            while True:
                list(pool.map(one, work))
                reps += 1
                el = time.perf_counter() - t0
                if el >= seconds / 2 or reps >= 50:
                    break
        return 4.0 * total * reps / el / 1e9, reps, el

    v1, r1, e1 = timed(1)
    vn, rn, en = timed(cores)
    return {"value": vn, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{sample}; compress+decompress of the sample {rn}x in {en:.1f} s on {cores} threads",
            "single_thread": {"value": v1, "unit": "GB/s", "cores": 1,
                              "sample": f"the same sample {r1}x in {e1:.1f} s on one thread"},
            "host": host}


def two_pass_block(alg, ms, n, kernels):
    gbps = alg / (ms * 1e-3) / 1e9
    return {"ms": ms, "kernels": kernels, "algorithmic_bytes": alg, "hbm_GBps": gbps,
            "frac_of_peak": gbps / HBM_PEAK_GBPS, "activation_GBps": 2.0 * n / (ms * 1e-3) / 1e9}


def run_channel_mode(steps=30, warmup=4, cpu_rows=1024):
    """The paper's own selection rule (Section 3.2, Eq. 1) on a [16384,16384] activation (512 MiB, so that
    the second read of the tensor comes from HBM, not from the Infinity Cache): outlier channels by
    Z-score > 3 kept whole, the rest int4 in groups of 128.  Compression reads the tensor twice (channel
    sums, then extraction + quantisation): algorithmic bytes 4N + outputs; decompression 2N + inputs."""
    import torch
    import workloads
    import oracle
    import paper_2508_00806_amd as adacc
    tokens, hidden = 16384, 16384
    x = workloads.c2("cuda", rows=tokens, hidden=hidden)
    n = tokens * hidden
    m = adacc.ChannelMethod(bits=4, quant_group=128, z_thresh=3.0, max_channels=256)
    sets = 3
    xs = [x if i == 0 else x.clone() for i in range(sets)]
    L = adacc.channel_layout_of(m, tokens, hidden)
    blobs = [adacc.alloc_channel_blob(m, tokens, hidden)[0] for _ in range(sets)]
    dsts = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(sets)]
    ws = adacc.alloc_channel_workspace(tokens, hidden)
    for i in range(sets):
        adacc.channel_compress(m, xs[i], tokens, hidden, blobs[i], ws)
    for i in range(warmup):
        adacc.channel_compress(m, xs[i % sets], tokens, hidden, blobs[i % sets], ws)
        adacc.channel_decompress(m, blobs[(i + 1) % sets], tokens, hidden, dsts[(i + 1) % sets])
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    for i in range(steps):
        ev[i][0].record()
        adacc.channel_compress(m, xs[i % sets], tokens, hidden, blobs[i % sets], ws)
        ev[i][1].record()
        adacc.channel_decompress(m, blobs[(i + 1) % sets], tokens, hidden, dsts[(i + 1) % sets])
        ev[i][2].record()
    torch.cuda.synchronize()
    c_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    d_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    st = adacc.channel_read_status(blobs[0], L)
    if st[1]:
        raise RuntimeError(f"more outlier channels than the blob holds: {st}")
    outputs = n // 2 + 4 * (n // 128) + 2 * tokens * st[0] + 4 * st[0]
    alg_c, alg_d = 4 * n + outputs, 2 * n + outputs
    # the oracle on the first rows of the same tensor, single thread
    xb = bits_of(x[:cpu_rows].cpu())
    om = oracle.Method(bits=4, quant_group=128)
    t0 = time.perf_counter()
    oc = oracle.channel_compress(om, xb, cpu_rows, hidden, 3.0, cap=256)
    oracle.channel_decompress(oc)
    el = time.perf_counter() - t0
    del xs, blobs, dsts, x
    torch.cuda.empty_cache()
    res = {
        "workload": f"outlier channels by Z-score>3 on a [{tokens},{hidden}] bf16 activation (0.5 % heavy-tailed channels), int4 group-128",
        "n_outlier_channels": st[0],
        "compress": two_pass_block(alg_c, c_ms, n, 4),
        "decompress": two_pass_block(alg_d, d_ms, n, 1),
        "cpu_oracle": {"value": 4.0 * cpu_rows * hidden / el / 1e9, "unit": "GB/s", "cores": 1,
                       "sample": f"first {cpu_rows} rows, compress+decompress once in {el:.2f} s"},
    }
    res["roofline"] = {"bound": "hbm", "kernel": "channel compress call (4 kernels)", "achieved": res["compress"]["hbm_GBps"],
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": res["compress"]["frac_of_peak"], "traffic": None}
    return res


def run_channelwise(steps=30, warmup=4, cpu_rows=1024):
    """Channel-wise symmetric int4 quantisation (Section 3.2, the Query / Key / Value scheme) of a
    [16384,16384] tensor (512 MiB: the second read comes from HBM).  Compression reads the tensor twice
    (channel maxima, then quantisation): algorithmic bytes 4N + N/2 + 4*hidden; decompression 2N + N/2 +
    4*hidden."""
    import torch
    import workloads
    import oracle
    import paper_2508_00806_amd as adacc
    tokens, hidden = 16384, 16384
    x = workloads.c2("cuda", rows=tokens, hidden=hidden)
    n = tokens * hidden
    sets = 3
    xs = [x if i == 0 else x.clone() for i in range(sets)]
    bufs = [adacc.alloc_channelwise(4, tokens, hidden) for _ in range(sets)]
    dsts = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(sets)]
    ws = bufs[0][2]

    def comp(i):
        adacc.channelwise_compress(4, xs[i % sets], tokens, hidden, bufs[i % sets][0], ws)

    def dec(i):
        adacc.channelwise_decompress(4, bufs[i % sets][0], tokens, hidden, dsts[i % sets])
    for i in range(sets + warmup):
        comp(i)
        dec(i)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    for i in range(steps):
        ev[i][0].record()
        comp(i)
        ev[i][1].record()
        dec(i + 1)
        ev[i][2].record()
    torch.cuda.synchronize()
    c_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    d_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    outputs = n // 2 + 4 * hidden
    alg_c, alg_d = 4 * n + outputs, 2 * n + outputs
    xb = bits_of(x[:cpu_rows].cpu())
    t0 = time.perf_counter()
    _, packed, scale = oracle.channelwise_compress(4, xb, cpu_rows, hidden)
    oracle.channelwise_decompress(4, packed, scale, cpu_rows, hidden)
    el = time.perf_counter() - t0
    del xs, bufs, dsts, x
    torch.cuda.empty_cache()
    res = {
        "workload": f"channel-wise symmetric int4 (Q/K/V scheme) on a [{tokens},{hidden}] bf16 tensor",
        "compress": two_pass_block(alg_c, c_ms, n, 3),
        "decompress": two_pass_block(alg_d, d_ms, n, 1),
        "cpu_oracle": {"value": 4.0 * cpu_rows * hidden / el / 1e9, "unit": "GB/s", "cores": 1,
                       "sample": f"first {cpu_rows} rows, compress+decompress once in {el:.2f} s"},
    }
    res["roofline"] = {"bound": "hbm", "kernel": "channel-wise compress call (3 kernels)", "achieved": res["compress"]["hbm_GBps"],
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": res["compress"]["frac_of_peak"], "traffic": None}
    return res


def run_mask(steps=30, warmup=3):
    """Dropout mask of the attention layer of C4 ([4,32,2048,2048] bytes, keep probability 0.9):
    byte format -> bit format and back (Section 3.2).  Algorithmic bytes per direction: n + n/8."""
    import torch
    import oracle
    import paper_2508_00806_amd as adacc
    n = 4 * 32 * 2048 * 2048
    sets = 3
    g = torch.Generator(device="cuda").manual_seed(77)
    masks = [(torch.rand(n, device="cuda", generator=g) < 0.9).to(torch.uint8) for _ in range(sets)]
    bits = [torch.empty(adacc.mask_packed_bytes(n), dtype=torch.uint8, device="cuda") for _ in range(sets)]
    backs = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(sets)]
    for i in range(sets + warmup):
        adacc.mask_pack(masks[i % sets], bits[i % sets])
        adacc.mask_unpack(bits[i % sets], backs[i % sets])
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    for i in range(steps):
        ev[i][0].record()
        adacc.mask_pack(masks[i % sets], bits[i % sets])
        ev[i][1].record()
        adacc.mask_unpack(bits[(i + 1) % sets], backs[(i + 1) % sets])
        ev[i][2].record()
    torch.cuda.synchronize()
    p_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    u_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    if not torch.equal(backs[0], masks[0]):
        raise RuntimeError("mask round trip is not lossless")
    alg = n + n // 8
    sample = masks[0][:1 << 24].cpu().numpy()
    t0 = time.perf_counter()
    oracle.mask_unpack(oracle.mask_pack(sample), sample.size)
    el = time.perf_counter() - t0
    del masks, bits, backs
    torch.cuda.empty_cache()
    res = {
        "workload": "dropout mask [4,32,2048,2048] bytes <-> bits, keep probability 0.9",
        "pack": {"ms": p_ms, "algorithmic_bytes": alg, "hbm_GBps": alg / (p_ms * 1e-3) / 1e9,
                 "frac_of_peak": alg / (p_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "unpack": {"ms": u_ms, "algorithmic_bytes": alg, "hbm_GBps": alg / (u_ms * 1e-3) / 1e9,
                   "frac_of_peak": alg / (u_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "cpu_oracle": {"value": 2.0 * sample.size / el / 1e9, "unit": "GB/s of mask bytes", "cores": 1,
                       "sample": f"first {sample.size} elements, pack+unpack once in {el:.2f} s"},
    }
    slow = "pack" if p_ms >= u_ms else "unpack"
    res["roofline"] = {"bound": "hbm", "kernel": f"mask_{slow}_kernel", "achieved": res[slow]["hbm_GBps"], "peak": HBM_PEAK_GBPS,
                       "unit": "GB/s", "frac": res[slow]["frac_of_peak"], "traffic": None}
    return res


def run_fallback(steps=5):
    """Group sizes outside the fast kernels' shapes (a whole 11008-wide row as one statistics group, groups
    that are no powers of two) on an [8192, 11008] bf16 tensor: the fallback kernels, for the record."""
    import torch
    import workloads
    import paper_2508_00806_amd as adacc
    x = workloads.c5_tensor("mlp_up", "cuda", rows=8192, seed=1).view(-1)
    n = x.numel()
    out = []
    for name, md in (
            ("TOPK-8 of every 11008-row, int4 g128", dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=11008, thresh=0.0, topk=8)),
            ("STD 4 sigma of every 11008-row, int8 per row", dict(bits=8, quant_group=11008, asym=0, outlier_mode="std", stat_group=11008, thresh=4.0, topk=0)),
            ("no outliers, int8 g96", dict(bits=8, quant_group=96, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0))):
        m = adacc.method_from_dict(md, max(4096, n // 64))
        blob, L = adacc.alloc_blob(m, n)
        ws = adacc.alloc_workspace(max(512, adacc.workspace_bytes(m, n)))
        dst = torch.empty(n, dtype=torch.bfloat16, device="cuda")
        adacc.compress(m, x, blob, ws)
        adacc.decompress(m, blob, dst)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        for _ in range(steps):
            adacc.compress(m, x, blob, ws)
        e[1].record()
        for _ in range(steps):
            adacc.decompress(m, blob, dst)
        e[2].record()
        torch.cuda.synchronize()
        c_ms, d_ms = e[0].elapsed_time(e[1]) / steps, e[1].elapsed_time(e[2]) / steps
        st = adacc.read_status(blob, L)
        if st[1]:
            raise RuntimeError(f"fallback workload {name}: overflow {st}")
        out.append({"workload": name, "compress_ms": c_ms, "decompress_ms": d_ms, "n_outliers": st[0],
                    "compress_activation_GBps": 2.0 * n / (c_ms * 1e-3) / 1e9,
                    "decompress_activation_GBps": 2.0 * n / (d_ms * 1e-3) / 1e9})
    del x
    torch.cuda.empty_cache()
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print(f"bench.py: this build measures one GPU (compression is rank-local, no collective is on the "
              f"path); --gpus {a.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    import paper_2508_00806_amd as adacc
    adacc.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    if a.only_channelwise:
        print(json.dumps({"channelwise_qkv": run_channelwise()}))
        return
    if a.only_mask:
        print(json.dumps({"dropout_mask": run_mask()}))
        return
    if a.only_channel:
        print(json.dumps({"channel_zscore": run_channel_mode()}))
        return
    if a.only_streams:
        print(json.dumps({"stream_ceilings": stream_ceilings()}))
        return
    main_res = run_workload(a.workload, a.steps, a.warmup, a.sets)
    extras, channel, mask, channelwise, ceilings, fallback = [], None, None, None, None, None
    if not a.no_extras:
        ceilings = stream_ceilings()
        for name in sorted(WORKLOAD_TEXT):
            if name == a.workload:
                continue
            k = 10 if name == "c5" else 50
            extras.append(run_workload(name, k, 5, a.sets))
            if name == "c1":  # 8 MB: also with everything in the caches
                warm = run_workload(name, k, 5, 1, cold=False)
                warm["workload"] = "c1 (warm)"
                extras.append(warm)
            if name in ("c1", "c2"):  # small tensors, bound by launches: also replayed from a graph
                extras.append(run_graph_replay(name))
        channel = run_channel_mode()
        mask = run_mask()
        channelwise = run_channelwise()
        fallback = run_fallback()
    cpu = None if a.no_cpu else cpu_baseline(a.workload, a.cpu_seconds)
    if cpu:  # the same metric on both sides: bytes compressed plus bytes restored per second
        cpu["gpu_over_cpu"] = {"all_cores": main_res["activation_GBps"] / cpu["value"],
                               "single_thread": main_res["activation_GBps"] / cpu["single_thread"]["value"]}
    props = torch.cuda.get_device_properties(0)

    roof = dict(main_res["roofline"])
    roof["stream_ceilings"] = ceilings
    out = {
        "metric": "compress+decompress GB/s of bf16 activations; fraction of MI355X HBM peak",
        "value": main_res["activation_GBps"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[a.workload], "device": f"{props.name} ({getattr(props, 'gcnArchName', '?')}, "
                                                                      f"{props.multi_processor_count} CUs, {props.total_memory >> 30} GiB)",
                   "buffer_sets": main_res["buffer_sets"],
                   "tensors": main_res["tensors"], "n_outliers": main_res["n_outliers"],
                   "storage": ("binary16 in and out; int4 codes, binary32 scales, (int32, binary16) outliers in between"
                               if SECOND_READINGS.get(a.workload, (0, 0, 0))[2] == 1 else
                               "bf16 in and out; int8 / int4 codes, binary32 scales, (int32, bf16) outliers in between")},
        "hbm_frac_of_peak_roundtrip": main_res["roundtrip_hbm_frac_of_peak"],
        "compress": main_res["compress"],
        "decompress": main_res["decompress"],
        "roofline": roof,
        "cpu_baseline": cpu,
        "other_workloads": extras,
        "channel_zscore": channel,
        "dropout_mask": mask,
        "channelwise_qkv": channelwise,
        "fallback_group_sizes": fallback,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
