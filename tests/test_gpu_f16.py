"""GPU parity for binary16 (FP16) tensors, the format the paper compresses (Section 3.2, "compressed
from FP16 to INT4"): the same entry points with adacc_method.dtype = ADACC_DTYPE_F16, against the
oracle run with the same format.  Same bar as for bf16: every section of the blob bit-exact,
binary32 reconstruction bit-equal, binary16 reconstruction equal."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_00806_amd as adacc
import workloads
from helpers import (adacc_method, assert_bf16_matches, assert_f32_matches, bits_of, compare_blob_with_oracle, from_bits,
                     oracle_method, run_channel_parity, run_parity)
from test_gpu_channelwise import run as run_channelwise
from test_gpu_parity import SWEEP

pytestmark = pytest.mark.gpu
F16 = torch.float16


def log(msg):
    print(msg, flush=True)


def random_f16_bits(seed, n, heavy=True, edge=True, scale=1.0):
    g = np.random.default_rng(seed)
    x = g.standard_normal(n) * scale
    if heavy:
        x[g.choice(n, max(1, n // 64), replace=False)] *= 30.0
    with np.errstate(over="ignore"):  # what does not fit becomes infinite: part of the test
        b = x.astype(np.float16).view(np.uint16).copy()
    if edge and n >= 64:
        # signed zeros, subnormals (smallest and largest), ties in magnitude, the largest finite values
        b[1], b[2], b[3], b[4] = 0x8000, 0x0001, 0x8001, 0x03FF
        b[5] = b[9] = 0x4A10
        b[11] = 0xCA10
        b[n - 1], b[n - 2] = 0x7BFF, 0xFBFF
    return b


def f16(bits):
    return from_bits(bits, dtype=F16)


@pytest.mark.parametrize("mode", ["none", "abs", "std", "topk"])
def test_method_sweep_binary16(mode):
    for rule in (0, 1):
        for bits, asym, gq, gs in SWEEP:
            groups = 13 if gs <= 1024 else 5   # short last tile for most sizes
            n = gs * groups
            x = f16(random_f16_bits(2000 * bits + 10 * gq + gs + asym, n))
            md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode=mode, stat_group=gs,
                      thresh={"abs": 2.5, "std": 3.0}.get(mode, 0.0), topk=3 if mode == "topk" else 0)
            log(f"[f16] sweep mode={mode} rule={rule} bits={bits} asym={asym} gq={gq} gs={gs} n={n}")
            run_parity(x, md, rule=rule)


def test_small_and_large_magnitudes_binary16():
    """Tensors that live among the subnormals (below 6.1e-5) and near the end of the range (65504):
    scales far from 1, reconstructions that round to subnormals or reach the largest finite value."""
    for label, scale in (("tiny", 3e-6), ("large", 1500.0)):
        b = random_f16_bits(61, 4096 * 3 + 1024, scale=scale)
        for mode in ("none", "std", "topk"):
            for bits, asym in ((4, 0), (8, 1)):
                md = dict(bits=bits, quant_group=128, asym=asym, outlier_mode=mode, stat_group=1024,
                          thresh=3.0 if mode == "std" else 0.0, topk=2 if mode == "topk" else 0)
                log(f"[f16] {label} mode={mode} bits={bits} asym={asym}")
                for rule in (0, 1):
                    run_parity(f16(b), md, rule=rule)


def test_degenerate_inputs_binary16():
    z = np.zeros(4096, dtype=np.uint16)
    const = np.full(4096, 0x3A00, dtype=np.uint16)   # 0.75
    tiny = np.zeros(4096, dtype=np.uint16)
    tiny[0], tiny[1], tiny[100] = 0x0001, 0x8001, 0x0400
    huge = np.full(4096, 0x7BFF, dtype=np.uint16)
    huge[::2] = 0xFBFF
    nonfin = random_f16_bits(5, 4096)
    # +Inf, -Inf, a quiet NaN, a signalling NaN, the all-ones pattern
    nonfin[7], nonfin[300], nonfin[2049], nonfin[3000], nonfin[4000] = 0x7C00, 0xFC00, 0x7E00, 0x7D01, 0xFFFF
    for label, b in (("zeros", z), ("const", const), ("tiny", tiny), ("huge", huge), ("nonfinite", nonfin)):
        for mode in ("none", "abs", "std", "topk"):
            for asym in (0, 1):
                if label == "nonfinite" and mode == "none":
                    continue
                md = dict(bits=8, quant_group=64, asym=asym, outlier_mode=mode, stat_group=256,
                          thresh={"abs": 1.0, "std": 4.0}.get(mode, 0.0), topk=2 if mode == "topk" else 0)
                log(f"[f16] degenerate {label} mode={mode} asym={asym}")
                run_parity(f16(b), md)
    md = dict(bits=4, quant_group=64, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0)
    run_parity(f16(nonfin), md)


def test_topk_selection_corner_cases_binary16():
    rng = np.random.default_rng(98)
    big = 0x5240  # 50.0
    for gs in (512, 2048, 4096):
        for k in (1, 4, 9):
            b = rng.normal(0.0, 1.0, size=gs * 7).astype(np.float16).view(np.uint16).copy()
            g = lambda i: slice(i * gs, (i + 1) * gs)
            b[g(0)][8:8 + k + 1] = [big + i for i in range(k + 1)]      # the largest share a lane
            pos = np.sort(rng.choice(gs, size=k + 2, replace=False))
            b[g(1)][pos] = big                                          # a tie at the k-th place
            b[g(1)][pos[::2]] |= 0x8000
            b[g(2)] = 0x3C00                                            # constant
            b[g(3)] = 0
            b[g(3)][5] = 0x8000
            b[g(4)][[3, 200, 300, 301]] = [0x7C00, 0xFE01, big, big + 1]  # Inf, NaN and large values
            b[g(5)][rng.choice(gs, size=k + 3, replace=False)] = 0xFC00   # more that are not finite than k
            for bits, gq, asym in ((4, 128, 0), (8, gs, 1)):
                md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode="topk", stat_group=gs, thresh=0.0, topk=k)
                log(f"[f16] topk corner cases gs={gs} k={k} bits={bits} gq={gq} asym={asym}")
                run_parity(f16(b), md)


@pytest.mark.parametrize("name,rows", [("c1", 67), ("c2", 37), ("c3", 5), ("c4", 2048)])
def test_config_reduced_binary16(name, rows):
    x = workloads.make(name, "cpu", rows=rows).to(F16)
    md = workloads.METHODS[name]
    cap = workloads.outlier_capacity(md, x.numel(), x.shape[-1])
    oc, *_ = run_parity(x, md, cap=cap)
    log(f"[f16] {name}: numel={x.numel()} n_out={oc.n_out}")


def test_many_tiles_and_dense_outliers_binary16():
    """Placement across blocks of tiles, and tiles with more outliers than a slot holds."""
    b = random_f16_bits(31, 2048 * 700 + 512)
    md = dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=2.5, topk=0)
    run_parity(f16(b), md)
    md = dict(bits=4, quant_group=128, asym=1, outlier_mode="abs", stat_group=0, thresh=0.3, topk=0)  # most elements
    run_parity(f16(random_f16_bits(32, 2048 * 9)), md)
    md = dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=4096, thresh=0.0, topk=4)
    run_parity(f16(random_f16_bits(33, 4096 * 300)), md)


def test_batch_of_both_formats():
    """One batch call over bf16 and binary16 tensors of several methods, a retained one among them."""
    rows = 12
    table = []
    for t, (tname, hidden, md) in enumerate(workloads.C5_LAYER):
        x = workloads.c5_tensor(tname, "cpu", rows=rows, seed=5100 + t)
        table.append((hidden, md, x))
        table.append((hidden, md, x.to(F16)))
    table.append((2048, workloads.C4_METHOD, workloads.c4("cpu", rows=2048)[:64].contiguous().to(F16)))
    methods, srcs, blobs, layouts, ocs = [], [], [], [], []
    for hidden, md, x in table:
        n = x.numel()
        if md is None:
            methods.append(adacc.NOOP); srcs.append(x.cuda()); blobs.append(None); layouts.append(None); ocs.append(None)
            continue
        fmt = 1 if x.dtype == F16 else 0
        cap = workloads.outlier_capacity(md, n, hidden)
        m = adacc_method(md, cap, fmt=fmt)
        oc = oracle.compress(oracle_method(md, fmt=fmt), bits_of(x), cap=cap)
        assert oc.n_out <= cap
        oc._full_idx = oc.out_idx.astype(np.int64)
        blob, L = adacc.alloc_blob(m, n)
        methods.append(m); srcs.append(x.contiguous().view(-1).cuda()); blobs.append(blob); layouts.append(L); ocs.append(oc)
    ws = adacc.alloc_workspace(adacc.batch_workspace_bytes(methods, [s.numel() for s in srcs]))
    for rep in range(2):
        log(f"[f16] mixed batch compress rep={rep} tensors={len(methods)}")
        adacc.compress_batch(methods, srcs, blobs, ws)
        torch.cuda.synchronize()
        for (hidden, md, x), m, blob, L, oc in zip(table, methods, blobs, layouts, ocs):
            if md is not None:
                compare_blob_with_oracle(blob, L, m, x.numel(), oc)
    for kind in ("own", "f32"):
        dsts = [None if b is None else torch.empty(s.numel(), dtype=s.dtype if kind == "own" else torch.float32, device="cuda")
                for s, b in zip(srcs, blobs)]
        log(f"[f16] mixed batch decompress {kind}")
        adacc.decompress_batch(methods, blobs, dsts, ws)
        torch.cuda.synchronize()
        for d, oc, m in zip(dsts, ocs, methods):
            if d is None:
                continue
            of32, o16 = oracle.decompress(oc)
            if kind == "f32":
                assert_f32_matches(d.cpu().numpy(), of32)
            else:
                assert_bf16_matches(bits_of(d), o16, m.dtype)


@pytest.mark.parametrize("bits,asym", [(4, 0), (8, 1)])
def test_outlier_channels_binary16(bits, asym):
    """Eq. 1 on a binary16 activation with heavy-tailed channels; one of them holds Inf and a NaN, whose
    patterns (a signalling one among them) come back bit for bit."""
    x = workloads.c2("cpu", rows=300).to(F16)
    oc, st = run_channel_parity(x, bits, 128, asym)
    assert oc.n_ch > 0
    log(f"[f16] channels bits={bits} asym={asym}: {oc.n_ch} outlier channels")
    xb = bits_of(x).reshape(300, -1).copy()
    xb[17, 40], xb[18, 40], xb[19, 40] = 0x7C00, 0x7D01, 0xFE00
    oc, st = run_channel_parity(from_bits(xb.reshape(-1), dtype=F16).view(300, -1), bits, 128, asym)
    assert 40 in [int(c) for c in oc.ch_idx]


def test_channelwise_binary16():
    g = torch.Generator().manual_seed(77)
    for tokens, hidden, bits, rule in ((300, 2048, 4, 0), (37, 11008, 8, 1), (70, 8, 4, 1)):
        x = (torch.randn(tokens, hidden, generator=g) * torch.exp(torch.randn(hidden, generator=g) * 1.5)).to(F16)
        xb = bits_of(x).copy()
        xb[3], xb[hidden + 5] = 0x7C00, 0x7E00   # not finite: counts as zero
        log(f"[f16] channelwise tokens={tokens} hidden={hidden} bits={bits} rule={rule}")
        run_channelwise(from_bits(xb, dtype=F16).view(tokens, hidden), bits, rule)
