#!/usr/bin/env python3
"""Benchmark of the Adacc hot path on one MI355X: compress + decompress of saved bf16
activations (Section 3.2) through libadacc, next to the CPU oracle timed on the host.

A step = one compression and one decompression of the workload (every row of the hot-path
table: load, statistics, outlier mask, ordered compaction, scale, quantise, pack, and on the
way back unpack, dequantise, outlier patch, store).  Inputs are generated once and are
resident in HBM before the timed region.  Several buffer sets are rotated and a step
decompresses a blob that was compressed two steps earlier, so that neither kernel reads
its input from the 256 MB Infinity Cache.

Prints ONE JSON line.  value = bytes of bf16 activations compressed plus bytes restored,
per second (GB/s, 1e9), whole job.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBPS = 8000.0  # MI355X published peak HBM3E bandwidth

WORKLOAD_TEXT = {
    "c1": "c1: single activation [4096,1024] bf16, int8 per-row absmax, outliers |x|>6*row_std",
    "c2": "c2: GPT-1.3B-shaped [16x2048,2048] bf16, int4 group-128 absmax, top-2 outliers per 2048-row",
    "c3": "c3: MLP GELU output [8x2048,16384] bf16, int8 group-64, outliers at 8*group_std",
    "c4": "c4: attention softmax [4,32,2048,2048] bf16, asymmetric int8 per row, outliers > 0.05",
    "c5": "c5: LLaMA-7B-shaped layer set, 32 layers x 5 tensors at batch 2 x seq 4096, batched launch",
}

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by the plain copy kernel: FETCH_SIZE x 2.000, WRITE_SIZE x 1.000); copied
# from profiles/hbm_traffic_pmc.txt.
MEASURED_TRAFFIC_BYTES = {
    "c2": {"compress": 172618445, "decompress": 173085286},
    "c3": {"compress": 824715571, "decompress": 826351923},
    "c4": {"compress": 1622748877, "decompress": 1652543386},
    "c5": {"compress": 23084046336, "decompress": 23150024499},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--sets", type=int, default=0, help="rotating buffer sets (0 = enough to exceed 1 GiB)")
    ap.add_argument("--no-extras", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--only-channelwise", action="store_true",
                    help="run only the channel-wise (Q/K/V) quantisation measurement and print its JSON")
    ap.add_argument("--only-mask", action="store_true",
                    help="run only the dropout-mask (byte <-> bit) measurement and print its JSON")
    ap.add_argument("--only-channel", action="store_true",
                    help="run only the outlier-channel (Z-score) measurement and print its JSON")
    return ap.parse_args()


class Workload:
    """Device buffers of one workload: `sets` rotating copies of (inputs, blobs, outputs)."""

    def __init__(self, name, sets):
        import torch
        import workloads
        import paper_2508_00806_amd as adacc
        from helpers import adacc_method
        self.name = name
        self.adacc = adacc
        if name == "c5":
            specs = [(f"L{layer}.{tname}", hidden, md, x) for layer, tname, x, md in workloads.c5("cuda")
                     for hidden in [x.shape[-1]]]
        else:
            x = workloads.make(name, "cuda")
            specs = [(name, x.shape[-1], workloads.METHODS[name], x)]
        self.mds = [s[2] for s in specs]
        self.numels = [s[3].numel() for s in specs]
        self.methods = [adacc_method(md, workloads.outlier_capacity(md, n, h))
                        for (_, h, md, _), n in zip(specs, self.numels)]
        self.layouts = [adacc.layout_of(m, n) for m, n in zip(self.methods, self.numels)]
        self.batched = len(specs) > 1
        in_bytes = sum(2 * n for n, md in zip(self.numels, self.mds) if md is not None)
        if sets <= 0:
            sets = max(2, min(8, -(-(1 << 30) // max(in_bytes, 1))))
            sets += sets % 2
        if name == "c5":
            sets = 2  # 20 GiB per set: far beyond any cache already
        self.sets = sets
        self.src, self.blob, self.dst = [], [], []
        for s in range(sets):
            self.src.append([sp[3].view(-1) if s == 0 else sp[3].view(-1).clone() for sp in specs])
            self.blob.append([None if md is None else adacc.alloc_blob(m, n)[0]
                              for m, n, md in zip(self.methods, self.numels, self.mds)])
            self.dst.append([None if md is None else torch.empty(n, dtype=torch.bfloat16, device="cuda")
                             for n, md in zip(self.numels, self.mds)])
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
        for md, b, L in zip(self.mds, self.blob[0], self.layouts):
            if md is None:
                continue
            st = self.adacc.read_status(b, L)
            if st[1] or st[2]:
                raise RuntimeError(f"compression reported overflow/abort: {st}")


def time_steps(w, steps, warmup):
    """Returns (ms per step, ms per compress launch, ms per decompress launch), all measured with
    events on the stream the kernels run on, inside the same timed region."""
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
    c_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    d_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    return total_ms / steps, c_ms, d_ms, wall_ms / steps


def copy_ceiling():
    """GB/s (read + written bytes) of the library's copy kernel on 1 GiB, with the streaming accesses
    the tensor streams use when ADACC_COPY_STREAM=1 is set by the caller (see main)."""
    import torch
    import paper_2508_00806_amd as adacc
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    b = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(2)]
    for i in range(3):
        adacc.hbm_copy(b[i % 2], a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for i in range(reps):
        adacc.hbm_copy(b[i % 2], a)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def cpu_baseline(name, seconds):
    """The oracle as it stands, single thread, on a bounded sample of the same workload."""
    import workloads
    import oracle
    from helpers import bits_of, oracle_method
    if name == "c5":
        tname, hidden, md = workloads.C5_LAYER[0]
        x = workloads.c5_tensor(tname, "cpu", rows=2048)
        sample = f"first 2048 rows of tensor {tname} of layer 0"
    else:
        rows = {"c1": 4096, "c2": 4096, "c3": 512, "c4": 4096}[name]
        x = workloads.make(name, "cpu", rows=rows)
        md = workloads.METHODS[name]
        sample = f"{rows} rows ({x.numel()} elements) of the workload, same generator"
    b = bits_of(x)
    om = oracle_method(md)
    reps, t0 = 0, time.perf_counter()
    while True:
        c = oracle.compress(om, b)
        oracle.decompress(c)
        reps += 1
        el = time.perf_counter() - t0
        if el >= seconds or reps >= 200:
            break
    gbps = 4.0 * b.size * reps / el / 1e9
    return {"value": gbps, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{sample}; compress+decompress repeated {reps}x in {el:.1f} s"}


def run_channel_mode(steps=50, warmup=5, cpu_rows=2048):
    """The paper's own selection rule (Section 3.2, Eq. 1) on the C2-shaped activation: outlier
    channels by Z-score > 3 kept whole, the rest int4 in groups of 128.  Compression reads the
    tensor twice (channel sums, then extraction + quantisation): algorithmic bytes 4N + outputs;
    decompression 2N + inputs.  Three rotating buffer sets, as for the main workload."""
    import torch
    import workloads
    import oracle
    import paper_2508_00806_amd as adacc
    from helpers import bits_of
    x = workloads.make("c2", "cuda")
    tokens, hidden = x.shape
    n = tokens * hidden
    m = adacc.ChannelMethod(bits=4, quant_group=128, z_thresh=3.0, max_channels=64)
    sets = 4
    xs = [x if i == 0 else x.clone() for i in range(sets)]
    L = adacc.channel_layout_of(m, tokens, hidden)
    blobs = [adacc.alloc_channel_blob(m, tokens, hidden)[0] for _ in range(sets)]
    dsts = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(sets)]
    ws = adacc.alloc_channel_workspace(tokens, hidden)
    for i in range(sets):
        adacc.channel_compress(m, xs[i], tokens, hidden, blobs[i], ws)
    for i in range(warmup):
        adacc.channel_compress(m, xs[i % sets], tokens, hidden, blobs[i % sets], ws)
        adacc.channel_decompress(m, blobs[(i + 2) % sets], tokens, hidden, dsts[(i + 2) % sets])
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    for i in range(steps):
        ev[i][0].record()
        adacc.channel_compress(m, xs[i % sets], tokens, hidden, blobs[i % sets], ws)
        ev[i][1].record()
        adacc.channel_decompress(m, blobs[(i + 2) % sets], tokens, hidden, dsts[(i + 2) % sets])
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
    oc = oracle.channel_compress(om, xb, cpu_rows, hidden, 3.0, cap=64)
    oracle.channel_decompress(oc)
    el = time.perf_counter() - t0
    del xs, blobs, dsts
    torch.cuda.empty_cache()
    return {
        "workload": f"outlier channels by Z-score>3 on the c2 tensor [{tokens},{hidden}] bf16, int4 group-128",
        "n_outlier_channels": st[0],
        "compress": {"ms": c_ms, "kernels": 4, "algorithmic_bytes": alg_c, "hbm_GBps": alg_c / (c_ms * 1e-3) / 1e9,
                     "frac_of_peak": alg_c / (c_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "activation_GBps": 2.0 * n / (c_ms * 1e-3) / 1e9},
        "decompress": {"ms": d_ms, "kernels": 1, "algorithmic_bytes": alg_d, "hbm_GBps": alg_d / (d_ms * 1e-3) / 1e9,
                       "frac_of_peak": alg_d / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                       "activation_GBps": 2.0 * n / (d_ms * 1e-3) / 1e9},
        "cpu_oracle": {"value": 4.0 * cpu_rows * hidden / el / 1e9, "unit": "GB/s", "cores": 1,
                       "sample": f"first {cpu_rows} rows, compress+decompress once in {el:.2f} s"},
    }


def run_channelwise(steps=50, warmup=5, cpu_rows=2048):
    """Channel-wise symmetric int4 quantisation (Section 3.2, the Query / Key / Value scheme) of the
    C2-shaped tensor.  Compression reads the tensor twice (channel maxima, then quantisation):
    algorithmic bytes 4N + N/2 + 4*hidden; decompression 2N + N/2 + 4*hidden."""
    import torch
    import workloads
    import oracle
    import paper_2508_00806_amd as adacc
    from helpers import bits_of
    x = workloads.make("c2", "cuda")
    tokens, hidden = x.shape
    n = tokens * hidden
    sets = 4
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
        dec(i + 2)
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
    del xs, bufs, dsts
    torch.cuda.empty_cache()
    return {
        "workload": f"channel-wise symmetric int4 (Q/K/V scheme) on the c2 tensor [{tokens},{hidden}] bf16",
        "compress": {"ms": c_ms, "kernels": 3, "algorithmic_bytes": alg_c, "hbm_GBps": alg_c / (c_ms * 1e-3) / 1e9,
                     "frac_of_peak": alg_c / (c_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "activation_GBps": 2.0 * n / (c_ms * 1e-3) / 1e9},
        "decompress": {"ms": d_ms, "kernels": 1, "algorithmic_bytes": alg_d, "hbm_GBps": alg_d / (d_ms * 1e-3) / 1e9,
                       "frac_of_peak": alg_d / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                       "activation_GBps": 2.0 * n / (d_ms * 1e-3) / 1e9},
        "cpu_oracle": {"value": 4.0 * cpu_rows * hidden / el / 1e9, "unit": "GB/s", "cores": 1,
                       "sample": f"first {cpu_rows} rows, compress+decompress once in {el:.2f} s"},
    }


def run_mask(steps=30, warmup=3):
    """Dropout mask of the attention layer of C4 ([4,32,2048,2048] bytes, keep probability 0.9):
    byte format -> bit format and back (Section 3.2).  Algorithmic bytes per direction: n + n/8."""
    import torch
    import numpy as np
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
    return {
        "workload": "dropout mask [4,32,2048,2048] bytes <-> bits, keep probability 0.9",
        "pack": {"ms": p_ms, "algorithmic_bytes": alg, "hbm_GBps": alg / (p_ms * 1e-3) / 1e9,
                 "frac_of_peak": alg / (p_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "unpack": {"ms": u_ms, "algorithmic_bytes": alg, "hbm_GBps": alg / (u_ms * 1e-3) / 1e9,
                   "frac_of_peak": alg / (u_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "cpu_oracle": {"value": 2.0 * sample.size / el / 1e9, "unit": "GB/s of mask bytes", "cores": 1,
                       "sample": f"first {sample.size} elements, pack+unpack once in {el:.2f} s"},
    }


def run_workload(name, steps, warmup, sets):
    import torch
    w = Workload(name, sets)
    ms, c_ms, d_ms, wall_ms = time_steps(w, steps, warmup)
    w.check_status()
    alg = w.algorithmic_bytes()
    res = {
        "workload": name,
        "ms_per_step": ms,
        "wall_ms_per_step": wall_ms,
        "activation_GBps": 2.0 * w.act_bytes / (ms * 1e-3) / 1e9,
        "compress": {"ms": c_ms, "activation_GBps": w.act_bytes / (c_ms * 1e-3) / 1e9,
                     "hbm_GBps": alg / (c_ms * 1e-3) / 1e9, "frac_of_peak": alg / (c_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "decompress": {"ms": d_ms, "activation_GBps": w.act_bytes / (d_ms * 1e-3) / 1e9,
                       "hbm_GBps": alg / (d_ms * 1e-3) / 1e9, "frac_of_peak": alg / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "roundtrip_hbm_frac_of_peak": 2.0 * alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_direction": alg,
        "activation_bytes": w.act_bytes,
        "n_outliers": int(sum(w.n_out)),
        "tensors": len(w.methods),
        "buffer_sets": w.sets,
    }
    del w
    torch.cuda.empty_cache()
    return res


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
    main_res = run_workload(a.workload, a.steps, a.warmup, a.sets)
    ceiling = copy_ceiling()
    os.environ["ADACC_COPY_STREAM"] = "1"
    ceiling_stream = copy_ceiling()
    os.environ.pop("ADACC_COPY_STREAM")
    extras = []
    if not a.no_extras:
        for name in sorted(WORKLOAD_TEXT):
            if name == a.workload:
                continue
            k = 10 if name == "c5" else 50
            extras.append(run_workload(name, k, 5, a.sets))
    channel = None if a.no_extras else run_channel_mode()
    mask = None if a.no_extras else run_mask()
    channelwise = None if a.no_extras else run_channelwise()
    cpu = None if a.no_cpu else cpu_baseline(a.workload, a.cpu_seconds)

    dom = "compress" if main_res["compress"]["ms"] >= main_res["decompress"]["ms"] else "decompress"
    roof = {
        "bound": "hbm",
        "kernel": dom,
        "achieved": main_res[dom]["hbm_GBps"],
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": main_res[dom]["frac_of_peak"],
        "traffic": MEASURED_TRAFFIC_BYTES.get(a.workload, {}).get(dom),
        "algorithmic_bytes_per_launch": main_res["algorithmic_bytes_per_direction"],
        "ms_per_launch": main_res[dom]["ms"],
        "copy_kernel_GBps": ceiling,
        "copy_kernel_streaming_GBps": ceiling_stream,
    }
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
        "config": {"workload": WORKLOAD_TEXT[a.workload], "buffer_sets": main_res["buffer_sets"],
                   "tensors": main_res["tensors"], "n_outliers": main_res["n_outliers"]},
        "hbm_frac_of_peak_roundtrip": main_res["roundtrip_hbm_frac_of_peak"],
        "compress": main_res["compress"],
        "decompress": main_res["decompress"],
        "roofline": roof,
        "cpu_baseline": cpu,
        "other_workloads": extras,
        "channel_zscore": channel,
        "dropout_mask": mask,
        "channelwise_qkv": channelwise,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
