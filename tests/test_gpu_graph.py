"""The library's calls inside a captured HIP graph (launch-bound callers replay a graph instead of launching
kernel by kernel): every call only enqueues kernels on the stream it is given - no allocation, no memset node,
no host round trip - so a compression and a decompression can be captured and replayed.  Each replay, with
other inputs, is compared with the same calls made eagerly (blob sections and output bit for bit); eager work
and synchronisations lie between the replays."""
import numpy as np
import pytest
import torch

import paper_2508_00806_amd as adacc
from helpers import adacc_method, from_bits

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


def inputs(seed, n):
    g = np.random.default_rng(seed)
    x = g.standard_normal(n).astype(np.float32)
    x[g.choice(n, n // 100, replace=False)] *= 25.0
    return torch.from_numpy(x).to(torch.bfloat16)


@pytest.mark.parametrize("md", [
    dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=3.0, topk=0),
    dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=2048, thresh=0.0, topk=2),
    dict(bits=8, quant_group=256, asym=1, outlier_mode="abs", stat_group=0, thresh=20.0, topk=0),
    dict(bits=4, quant_group=128, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0),
    # the fallback kernels (dynamic LDS, a second launch for what the first could not place)
    dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=11008, thresh=0.0, topk=3),
    dict(bits=8, quant_group=24, asym=1, outlier_mode="std", stat_group=4080, thresh=2.5, topk=0),
], ids=["std", "topk", "abs", "none", "fallback-topk", "fallback-std"])
def test_compress_and_decompress_replayed_from_a_graph(md):
    n = 2048 * 333 + 640
    m = adacc_method(md, n // 8)
    src = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    dst = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    blob, L = adacc.alloc_blob(m, n)
    ws = adacc.alloc_workspace(max(512, adacc.workspace_bytes(m, n))) if md["outlier_mode"] != "none" else None
    # eager twins with buffers of their own
    e_dst = torch.empty_like(dst)
    e_blob, _ = adacc.alloc_blob(m, n)
    e_ws = adacc.alloc_workspace(max(512, adacc.workspace_bytes(m, n))) if ws is not None else None

    src.copy_(inputs(1, n))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on the capture stream's side, as torch asks for
        adacc.compress(m, src, blob, ws)
        adacc.decompress(m, blob, dst)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        adacc.compress(m, src, blob, ws)
        adacc.decompress(m, blob, dst)
    torch.cuda.synchronize()

    for rep in range(4):
        log(f"[graph] {md['outlier_mode']} replay {rep}")
        x = inputs(10 + rep, n)
        if rep == 2 and md["outlier_mode"] == "topk":
            x[5:2048:200] = float("inf")  # more values that are not finite than k in the first group: the placement runs
        src.copy_(x)
        blob.fill_(0x5A)
        dst.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        adacc.compress(m, src, e_blob, e_ws)
        adacc.decompress(m, e_blob, e_dst)
        torch.cuda.synchronize()
        st, e_st = adacc.read_status(blob, L), adacc.read_status(e_blob, L)
        assert st == e_st and st[1] == 0, (st, e_st)
        got = adacc.blob_sections(blob, L, m, n)
        want = adacc.blob_sections(e_blob, L, m, n)
        for k in want:
            a, b = got[k], want[k]
            if k in ("idx", "val"):
                a, b = a[:st[0]], b[:st[0]]
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep}: section {k} differs from the eager call"
        assert torch.equal(dst.view(torch.int16), e_dst.view(torch.int16)), f"replay {rep}: output differs"


def test_batch_calls_replayed_from_a_graph():
    """adacc_compress_batch / adacc_decompress_batch: the tables travel as kernel arguments of upload kernels, so
    the batch calls can be captured as well.  Four tensors of different methods and sizes, one retained (NOOP),
    one through the fallback kernels; every replay against single eager calls."""
    mds = [dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=3.0, topk=0),
           dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=2048, thresh=0.0, topk=2),
           None,
           dict(bits=8, quant_group=96, asym=1, outlier_mode="abs", stat_group=0, thresh=15.0, topk=0)]
    ns = [2048 * 40, 2048 * 75, 4096, 96 * 500 + 8]
    methods = [adacc.NOOP if md is None else adacc_method(md, n // 8) for md, n in zip(mds, ns)]
    srcs = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for n in ns]
    dsts = [None if md is None else torch.empty(n, dtype=torch.bfloat16, device="cuda") for md, n in zip(mds, ns)]
    blobs, layouts = [], []
    for md, m, n in zip(mds, methods, ns):
        if md is None:
            blobs.append(None); layouts.append(None)
        else:
            b, L = adacc.alloc_blob(m, n)
            blobs.append(b); layouts.append(L)
    ws = adacc.alloc_workspace(adacc.batch_workspace_bytes(methods, ns))
    cargs = adacc.prepare_compress_batch(methods, srcs, blobs)
    dargs = adacc.prepare_decompress_batch(methods, blobs, dsts)
    for i, n in enumerate(ns):
        srcs[i].copy_(inputs(100 + i, n))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        adacc.compress_batch(methods, srcs, blobs, ws, prepared=cargs)
        adacc.decompress_batch(methods, blobs, dsts, ws, prepared=dargs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        adacc.compress_batch(methods, srcs, blobs, ws, prepared=cargs)
        adacc.decompress_batch(methods, blobs, dsts, ws, prepared=dargs)
    torch.cuda.synchronize()
    for rep in range(3):
        log(f"[graph] batch replay {rep}")
        for i, n in enumerate(ns):
            srcs[i].copy_(inputs(200 + 10 * rep + i, n))
            if blobs[i] is not None:
                blobs[i].fill_(0x33)
                dsts[i].fill_(-3.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (md, m, n) in enumerate(zip(mds, methods, ns)):
            if md is None:
                continue
            e_blob, L = adacc.alloc_blob(m, n)
            e_ws = adacc.alloc_workspace(max(512, adacc.workspace_bytes(m, n)))
            e_dst = torch.empty(n, dtype=torch.bfloat16, device="cuda")
            adacc.compress(m, srcs[i], e_blob, e_ws)
            adacc.decompress(m, e_blob, e_dst)
            torch.cuda.synchronize()
            st = adacc.read_status(blobs[i], layouts[i])
            assert st == adacc.read_status(e_blob, L) and st[1] == 0
            got, want = adacc.blob_sections(blobs[i], layouts[i], m, n), adacc.blob_sections(e_blob, L, m, n)
            for k in want:
                a, b = got[k], want[k]
                if k in ("idx", "val"):
                    a, b = a[:st[0]], b[:st[0]]
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep} tensor {i}: section {k}"
            assert torch.equal(dsts[i].view(torch.int16), e_dst.view(torch.int16)), f"replay {rep} tensor {i}: output"
