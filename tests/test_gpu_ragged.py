"""GPU parity for tensors whose length the group sizes do not divide (Section 3.2: a tensor of any shape
is one flat array cut into groups from its start): the last quantisation group and the last statistics
group are short.  Same bar as everywhere: every section of the blob and both reconstructions against
the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_00806_amd as adacc
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


# (quant group, statistics group, number of whole statistics groups before the short one)
SHAPES = [(8, 8, 300), (64, 64, 45), (128, 512, 9), (128, 2048, 3), (128, 2048, 4), (2048, 2048, 1), (128, 4096, 2),
          (4096, 4096, 3), (512, 4096, 0), (64, 64, 0)]


def lengths(gq, gs, whole):
    """Ends of every kind: one element, an odd count, whole quantisation groups only, one element short of
    a whole statistics group."""
    rests = sorted({1, 7, 8, gq - 1, gq, gq + 3, gs // 2 + 5, gs - 1} - {0, gs})
    return [whole * gs + r for r in rests if r < gs]


@pytest.mark.parametrize("mode", ["none", "abs", "std", "topk"])
@pytest.mark.parametrize("fmt", [0, 1])
def test_short_last_groups(mode, fmt):
    for gq, gs, whole in SHAPES:
        for n in lengths(gq, gs, whole):
            for bits, asym, rule in ((4, 0, 0), (8, 1, 1), (4, 1, 0), (8, 0, 0)):
                md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode=mode, stat_group=gs,
                          thresh={"abs": 2.5, "std": 2.0}.get(mode, 0.0), topk=3 if mode == "topk" else 0)
                log(f"[ragged] mode={mode} fmt={fmt} gq={gq} gs={gs} n={n} bits={bits} asym={asym} rule={rule}")
                run_parity(tensor(n + bits + asym, n, fmt), md, rule=rule)


def test_tail_with_values_that_are_not_finite_and_more_largest_values_than_elements():
    n = 2048 * 2 + 5
    b = random_bits(8, n)
    b[n - 1], b[n - 3] = 0x7F80, 0xFFC1
    for mode, kw in (("topk", dict(topk=8)), ("std", dict(thresh=3.0)), ("abs", dict(thresh=100.0)), ("none", {})):
        md = dict(bits=4, quant_group=128, asym=0, outlier_mode=mode, stat_group=2048, thresh=0.0, topk=0)
        md.update(kw)
        log(f"[ragged] not finite in the tail, mode={mode}")
        oc, *_ = run_parity(from_bits(b), md)
        if mode == "topk":  # the tail has 5 elements and k = 8: all of it is kept
            assert [int(i) for i in oc.out_idx if i >= 4096] == list(range(4096, n))


def test_outlier_capacity_reached_in_the_tail():
    n = 2048 + 300
    x = tensor(77, n, 0)
    md = dict(bits=8, quant_group=64, asym=0, outlier_mode="abs", stat_group=0, thresh=0.5, topk=0)
    full = oracle.compress(oracle_method(md), bits_of(x))
    in_main = int((full.out_idx < 2048).sum())
    assert full.n_out > in_main + 10
    log(f"[ragged] capacity ends inside the tail: {in_main} + {full.n_out - in_main}")
    oc, blob, L, m = run_parity(x, md, cap=in_main + 5, decompress=False)
    assert adacc.read_status(blob, L)[:2] == (full.n_out, 1)


def test_batch_with_short_last_groups():
    table = []
    for i, (n, md) in enumerate([
            (2048 * 5 + 77, dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=2048, thresh=0.0, topk=2)),
            (4096 * 3, dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=4096, thresh=0.0, topk=4)),
            (64 * 70 + 1, dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=2.0, topk=0)),
            (100, dict(bits=8, quant_group=128, asym=1, outlier_mode="none", stat_group=0, thresh=0.0, topk=0)),
            (4096 * 2 + 4095, dict(bits=8, quant_group=4096, asym=1, outlier_mode="abs", stat_group=0, thresh=2.0, topk=0))]):
        for fmt in (0, 1):
            table.append((n, md, tensor(40 + i, n, fmt), fmt))
    methods, srcs, blobs, layouts, ocs = [], [], [], [], []
    for n, md, x, fmt in table:
        oc = oracle.compress(oracle_method(md, fmt=fmt), bits_of(x))
        oc._full_idx = oc.out_idx.astype(np.int64)
        m = adacc_method(md, max(oc.n_out, 1), fmt=fmt)
        blob, L = adacc.alloc_blob(m, n)
        methods.append(m); srcs.append(x.cuda()); blobs.append(blob); layouts.append(L); ocs.append(oc)
    ws = adacc.alloc_workspace(adacc.batch_workspace_bytes(methods, [s.numel() for s in srcs]))
    for rep in range(2):
        log(f"[ragged] batch compress rep={rep}")
        adacc.compress_batch(methods, srcs, blobs, ws)
        torch.cuda.synchronize()
        for (n, md, x, fmt), m, blob, L, oc in zip(table, methods, blobs, layouts, ocs):
            compare_blob_with_oracle(blob, L, m, n, oc)
    for kind in ("own", "f32"):
        dsts = [torch.empty(s.numel(), dtype=s.dtype if kind == "own" else torch.float32, device="cuda") for s in srcs]
        log(f"[ragged] batch decompress {kind}")
        adacc.decompress_batch(methods, blobs, dsts, ws)
        torch.cuda.synchronize()
        for d, oc, m in zip(dsts, ocs, methods):
            of32, o16 = oracle.decompress(oc)
            if kind == "f32":
                assert_f32_matches(d.cpu().numpy(), of32)
            else:
                assert_bf16_matches(bits_of(d), o16, m.dtype)
