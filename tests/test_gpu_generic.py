"""GPU parity for group sizes outside the fast kernels' shapes (Section 3.2 groups the flat activation;
nothing makes the groups powers of two): quantisation groups of any multiple of 8, statistics groups of any
multiple of those up to 16384 - a whole 11008-wide row as one STD / TOPK group.  These run in fallback
kernels (a workgroup per segment, octets in registers, one word per octet in LDS); the bar is the same as everywhere: every section
of the blob and both reconstructions against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_00806_amd as adacc
import workloads
from helpers import (adacc_method, assert_bf16_matches, assert_f32_matches, bits_of, compare_blob_with_oracle, from_bits,
                     oracle_method, run_parity)
from test_gpu_f16 import random_f16_bits
from test_gpu_parity import random_bits

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


def tensor(seed, n, fmt):
    if fmt == 1:
        return from_bits(random_f16_bits(seed, n), dtype=torch.float16)
    return from_bits(random_bits(seed, n))


# (quantisation group, statistics group, elements)
SHAPES = [(24, 24, 24 * 700 + 5), (24, 96, 96 * 200), (40, 4000, 4000 * 3 + 17), (1000, 1000, 1000 * 9 + 999),
          (344, 11008, 11008 * 3), (11008, 11008, 11008 * 2 + 300), (8192, 8192, 8192 * 3), (128, 11008, 11008 * 5 + 64),
          (4096, 16384, 16384 * 2 + 4097), (48, 48, 40)]


@pytest.mark.parametrize("mode", ["none", "abs", "std", "topk"])
def test_group_sizes_of_every_kind(mode):
    for gq, gs, n in SHAPES:
        for bits, asym, rule, fmt in ((4, 0, 0, 0), (8, 1, 1, 0), (4, 1, 0, 1), (8, 0, 0, 1)):
            md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode=mode, stat_group=gs,
                      thresh={"abs": 2.5, "std": 2.5}.get(mode, 0.0), topk=5 if mode == "topk" else 0)
            log(f"[generic] mode={mode} gq={gq} gs={gs} n={n} bits={bits} asym={asym} rule={rule} fmt={fmt}")
            run_parity(tensor(n % 1000 + bits + asym, n, fmt), md, rule=rule)


def test_whole_rows_of_a_llama_mlp_activation_as_groups():
    """An [rows, 11008] activation with the row as the statistics group, the shape the configurations'
    per-row rules ask for on the MLP tensors: STD over the row and TOPK of the row."""
    x = workloads.c5_tensor("mlp_up", "cpu", rows=48, seed=77)
    for md in (dict(bits=8, quant_group=11008, asym=0, outlier_mode="std", stat_group=11008, thresh=4.0, topk=0),
               dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=11008, thresh=0.0, topk=11)):
        log(f"[generic] mlp_up rows as groups: {md['outlier_mode']}")
        oc, *_ = run_parity(x, md)
        if md["outlier_mode"] == "topk":
            assert oc.n_out == 11 * 48


def test_topk_of_a_row_for_every_number_of_outliers_kept():
    """TOPK over a segment-wide group finds its threshold through lists whose length depends on k (up to 8, up to 16,
    up to 32 keys per wavefront): k = 1 .. 32 on rows with many equal magnitudes, and on rows shorter than k octets."""
    b = random_bits(23, 11008 * 3 + 100)
    b[::7] = (b[::7] & 0x8000) | 0x4120          # every seventh value has the same magnitude, either sign
    b[11008:11008 + 40] = 0x7F7F                 # forty times the largest finite magnitude at the start of the second row
    for k in (1, 2, 7, 8, 9, 15, 16, 17, 31, 32):
        for n, gs in ((11008 * 3 + 100, 11008), (4104 * 2 + 9, 4104)):
            md = dict(bits=4, quant_group=8, asym=0, outlier_mode="topk", stat_group=gs, thresh=0.0, topk=k)
            log(f"[generic] topk k={k} n={n} gs={gs}")
            oc, *_ = run_parity(from_bits(b[:n]), md)
            assert oc.n_out == k * (n // gs) + min(k, n % gs)


def test_values_that_are_not_finite_and_degenerate_groups():
    n = 1000 * 6
    b = random_bits(3, n)
    b[5], b[1500], b[1501], b[5999] = 0x7F80, 0xFFC1, 0xFF80, 0x7FFF
    b[2000:3000] = 0x3F80          # a constant group
    b[3000:4000] = 0               # an all-zero group
    b[3007] = 0x8000
    for mode, kw in (("none", {}), ("abs", dict(thresh=3.0)), ("std", dict(thresh=3.0)), ("topk", dict(topk=2))):
        for asym in (0, 1):
            md = dict(bits=8, quant_group=200, asym=asym, outlier_mode=mode, stat_group=1000, thresh=0.0, topk=0)
            md.update(kw)
            log(f"[generic] not finite / degenerate mode={mode} asym={asym}")
            run_parity(from_bits(b), md)


def test_capacity_and_many_segments():
    """More segments than one placement block holds (block sums), and a capacity that ends inside a segment."""
    n = 4080 * 2100 + 77
    x = tensor(9, n, 0)
    md = dict(bits=8, quant_group=24, asym=0, outlier_mode="abs", stat_group=0, thresh=2.0, topk=0)
    log("[generic] many segments")
    oc, blob, L, m = run_parity(x, md)
    assert L.n_tiles == 2101 and oc.n_out > 10000
    oc2, blob, L, m = run_parity(x, md, cap=oc.n_out // 2, decompress=False)
    assert adacc.read_status(blob, L)[:2] == (oc.n_out, 1)


def test_batch_with_both_kinds_of_kernels():
    table = []
    for i, (n, md) in enumerate([
            (11008 * 7, dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=11008, thresh=0.0, topk=4)),
            (2048 * 5, dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=2048, thresh=0.0, topk=2)),
            (24 * 333 + 7, dict(bits=8, quant_group=24, asym=1, outlier_mode="std", stat_group=72, thresh=2.0, topk=0)),
            (64 * 70, dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=2.0, topk=0)),
            (1000, dict(bits=8, quant_group=40, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0))]):
        for fmt in (0, 1):
            table.append((n, md, tensor(60 + i, n, fmt), fmt))
    methods, srcs, blobs, layouts, ocs = [], [], [], [], []
    for n, md, x, fmt in table:
        oc = oracle.compress(oracle_method(md, fmt=fmt), bits_of(x))
        oc._full_idx = oc.out_idx.astype(np.int64)
        m = adacc_method(md, max(oc.n_out, 1), fmt=fmt)
        blob, L = adacc.alloc_blob(m, n)
        methods.append(m); srcs.append(x.cuda()); blobs.append(blob); layouts.append(L); ocs.append(oc)
    ws = adacc.alloc_workspace(adacc.batch_workspace_bytes(methods, [s.numel() for s in srcs]))
    for rep in range(2):
        log(f"[generic] batch compress rep={rep}")
        adacc.compress_batch(methods, srcs, blobs, ws)
        torch.cuda.synchronize()
        for (n, md, x, fmt), m, blob, L, oc in zip(table, methods, blobs, layouts, ocs):
            compare_blob_with_oracle(blob, L, m, n, oc)
    for kind in ("own", "f32"):
        dsts = [torch.empty(s.numel(), dtype=s.dtype if kind == "own" else torch.float32, device="cuda") for s in srcs]
        log(f"[generic] batch decompress {kind}")
        adacc.decompress_batch(methods, blobs, dsts, ws)
        torch.cuda.synchronize()
        for d, oc, m in zip(dsts, ocs, methods):
            of32, o16 = oracle.decompress(oc)
            if kind == "f32":
                assert_f32_matches(d.cpu().numpy(), of32)
            else:
                assert_bf16_matches(bits_of(d), o16, m.dtype)


def test_segments_through_the_slots_and_segments_selected_again():
    """ABS / STD: a segment's outliers travel through its slot of the workspace (32 records) or, when it has more,
    are written by the second launch; thresholds that give segments of both kinds side by side, none at all,
    and only crowded ones."""
    g = torch.Generator().manual_seed(41)
    n = 4080 * 300 + 1000
    x = torch.randn(n, generator=g).to(torch.bfloat16)
    for gq, gs in ((24, 4080), (120, 120), (11008, 11008)):
        for mode, th in (("abs", 2.7), ("abs", 3.6), ("abs", 1.0), ("std", 2.7), ("std", 3.5)):
            md = dict(bits=8, quant_group=gq, asym=0, outlier_mode=mode, stat_group=gs if mode == "std" else 0,
                      thresh=th, topk=0)
            log(f"[generic] slots and second launch gq={gq} gs={gs} mode={mode} thresh={th}")
            oc, blob, L, m = run_parity(x, md)
            per_seg = np.bincount(oc.out_idx // L.tile_elems, minlength=L.n_tiles)
            log(f"          outliers per segment: min {per_seg.min()} max {per_seg.max()}")
    # both kinds in one tensor for certain: quiet segments and crowded ones in turn
    y = x.clone()
    seg = 4080
    for s in range(0, n // seg, 3):
        y[s * seg:(s + 1) * seg] *= 0.2
    md = dict(bits=4, quant_group=24, asym=1, outlier_mode="abs", stat_group=0, thresh=2.2, topk=0)
    oc, blob, L, m = run_parity(y, md)
    per_seg = np.bincount(oc.out_idx // L.tile_elems, minlength=L.n_tiles)
    assert per_seg.min() <= 32 < per_seg.max()
    # a capacity that ends inside the slots' part and inside a crowded segment
    for cap in (oc.n_out // 3, oc.n_out - 5):
        run_parity(y, md, cap=cap, decompress=False)


def test_topk_groups_with_more_values_that_are_not_finite_than_k():
    """TOPK in the fallback kernels writes at offsets known in advance; a group with another count than k sends
    the tensor through the placement and the second launch."""
    for gq, gs, n in ((128, 11008, 11008 * 9 + 40), (24, 96, 96 * 500 + 24), (1000, 1000, 1000 * 40)):
        b = random_bits(17, n)
        b[(b & 0x7FFF) >= 0x7F80] = 0x3F80
        clean = b.copy()
        md = dict(bits=4, quant_group=gq, asym=0, outlier_mode="topk", stat_group=gs, thresh=0.0, topk=3)
        log(f"[generic] topk regular gq={gq} gs={gs}")
        oc, *_ = run_parity(from_bits(clean), md)
        assert oc.n_out == 3 * (n // gs) + min(3, n % gs)
        # five values that are not finite in one group in the middle, four in the last (short) group
        g0 = (n // gs // 2) * gs
        b[g0 + 1], b[g0 + 2], b[g0 + 9], b[g0 + gs - 1], b[g0 + gs // 2] = 0x7F80, 0xFF80, 0x7FC0, 0xFFFF, 0x7F81
        b[n - 1], b[n - 2], b[n - 3], b[n - 4] = 0x7F80, 0x7F80, 0xFF80, 0x7FFF
        log(f"[generic] topk irregular gq={gq} gs={gs}")
        oc2, blob, L, m = run_parity(from_bits(b), md)
        assert oc2.n_out > oc.n_out
        # the same workspace for irregular and regular tensors in turn: the flag of an earlier call must not count
        ws = adacc.alloc_workspace(adacc.workspace_bytes(m, n))
        for bits_now, full in ((b, oc2), (clean, oc), (b, oc2), (clean, oc)):
            want = oracle.compress(oracle_method(md), bits_now, cap=m.max_outliers)
            want._full_idx = full.out_idx.astype(np.int64)
            blob, L = adacc.alloc_blob(m, n)
            adacc.compress(m, from_bits(bits_now).cuda(), blob, ws)
            torch.cuda.synchronize()
            compare_blob_with_oracle(blob, L, m, n, want)


@pytest.mark.parametrize("mode", ["none", "abs", "std", "topk"])
def test_tensors_shorter_than_an_octet_and_last_groups_shorter_than_k(mode):
    for gq, gs, n in ((24, 24, 3), (24, 96, 8), (8, 16, 9), (128, 11008, 11008 * 2 + 3), (24, 96, 96 * 10 + 2),
                      (16384, 16384, 16384 + 1), (8, 16384, 16384 * 2 - 7)):
        for bits, asym in ((4, 0), (8, 1)):
            md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode=mode, stat_group=gs,
                      thresh={"abs": 1.5, "std": 1.5}.get(mode, 0.0), topk=5 if mode == "topk" else 0)
            log(f"[generic] short ends mode={mode} gq={gq} gs={gs} n={n} bits={bits} asym={asym}")
            run_parity(tensor(n % 1000 + 3, n, 0), md)


def test_the_largest_sizes_through_the_fallback_kernels():
    """More than 2^32 elements without outliers (64-bit element, code and group offsets in the fallback kernels too),
    and nearly 2^31 elements with outliers (32-bit signed indices; 195 000 rows of 11008 as STD and as TOPK groups:
    segments through 762 placement blocks).  Oracle on segments sampled over the whole range."""
    from test_gpu_parity import check_sampled
    n = (1 << 32) + 24 * 1000 + 8
    log(f"[generic] {n} elements without outliers, int8 in groups of 24")
    x = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(99)
    step = 1 << 28
    for i0 in range(0, n, step):
        x[i0:i0 + step].normal_(0.0, 1.5, generator=g)
    dst = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    md = dict(bits=8, quant_group=24, asym=1, outlier_mode="none", stat_group=0, thresh=0.0, topk=0)
    m = adacc_method(md, 0)
    blob, L = adacc.alloc_blob(m, n)
    adacc.compress(m, x, blob, None)
    adacc.decompress(m, blob, dst)
    torch.cuda.synchronize()
    assert L.tile_elems == 4080 and L.n_tiles == (n + 4079) // 4080
    check_sampled("fallback beyond 2^32", x, md, m, blob, L, dst, 24, 3)
    lo = (L.n_tiles - 1) * 4080  # the last, short segment and its short last group
    oc = oracle.compress(oracle_method(md), bits_of(x[lo:]))
    sec = adacc.blob_sections(blob, L, m, n)
    assert np.array_equal(sec["codes"][lo:].cpu().numpy(), oc.packed)
    assert np.array_equal(sec["scales"][lo // 24:].cpu().numpy().view(np.uint32), oc.scale.view(np.uint32))
    assert np.array_equal(sec["zp"][lo // 24:].cpu().numpy().view(np.uint32), oc.zp.view(np.uint32))
    assert np.array_equal(bits_of(dst[lo:]), oracle.decompress(oc)[1])
    del blob
    torch.cuda.empty_cache()

    rows = 195000
    n2 = rows * 11008
    assert n2 < (1 << 31)
    x2, dst2 = x[:n2], dst[:n2]
    x2[n2 - 3] = 900.0  # an outlier whose index is close to 2^31
    for md, cap in ((dict(bits=8, quant_group=11008, asym=0, outlier_mode="std", stat_group=11008, thresh=4.0, topk=0), n2 // 4096),
                    (dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=11008, thresh=0.0, topk=4), 4 * rows)):
        log(f"[generic] {n2} elements, {md['outlier_mode']} over rows of 11008")
        m = adacc_method(md, cap)
        blob, L = adacc.alloc_blob(m, n2)
        ws = adacc.alloc_workspace(adacc.workspace_bytes(m, n2))
        adacc.compress(m, x2, blob, ws)
        adacc.decompress(m, blob, dst2)
        torch.cuda.synchronize()
        assert L.tile_elems == 11008 and L.n_tiles == rows
        st = check_sampled("fallback longest with outliers", x2, md, m, blob, L, dst2, 24, 8)
        sec = adacc.blob_sections(blob, L, m, n2)
        assert st[1] == 0 and (n2 - 3) in sec["idx"][st[0] - 4:st[0]].cpu().tolist()
        if md["outlier_mode"] == "topk":
            assert st[0] == 4 * rows
        # the last row against the oracle on that slice (check_sampled leaves the last tile out)
        lo = n2 - 11008
        oc = oracle.compress(oracle_method(md), bits_of(x2[lo:]))
        p0 = int(sec["tile_ptr"][rows - 1])
        assert st[0] - p0 == oc.n_out
        assert np.array_equal(sec["idx"][p0:st[0]].cpu().numpy().astype(np.int64), oc.out_idx.astype(np.int64) + lo)
        assert np.array_equal(bits_of(dst2[lo:]), oracle.decompress(oc)[1])
        del blob, ws
        torch.cuda.empty_cache()
    del x, dst, x2, dst2
    torch.cuda.empty_cache()
