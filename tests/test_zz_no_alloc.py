"""adacc_compress_noalloc (the entry point for callers that cannot allocate: its scan state lives in a
device array of the library) against adacc_compress, through the C ABI: the two must produce the
same blob, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2508_00806_amd as adacc
import workloads
from helpers import adacc_method

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


def used_sections(blob, L, m, numel):
    sec = adacc.blob_sections(blob, L, m, numel)
    st = sec["status"].cpu().numpy().view(np.uint32)
    n = min(int(st[0]), m.max_outliers)
    out = {"codes": sec["codes"], "scales": sec["scales"].view(torch.int32), "status": sec["status"][:3]}
    if m.asym:
        out["zp"] = sec["zp"].view(torch.int32)
    if m.outlier_mode != adacc.OUTLIER_NONE:
        out.update(tile_ptr=sec["tile_ptr"], idx=sec["idx"][:n], val=sec["val"][:n])
    return {k: v.clone() for k, v in out.items()}, st


CASES = [
    ("c1", 300, 120),   # std outliers, 8-bit, whole-row groups
    ("c2", 301, 64),    # top-k, 4-bit
    ("c4", 4096, 2048),  # abs outliers, asymmetric
]


@pytest.mark.parametrize("name,rows_a,rows_b", CASES)
def test_noalloc_matches_compress_twice_in_a_row(name, rows_a, rows_b):
    md = workloads.METHODS[name]
    for rows in (rows_a, rows_b):  # the second call is smaller and finds the first call's words in the array
        log(f"[noalloc] {name} rows={rows}")
        x = workloads.make(name, "cuda", rows=rows).view(-1)
        numel = x.numel()
        m = adacc_method(md, workloads.outlier_capacity(md, numel, workloads.SHAPES[name][1]))
        blob_a, L = adacc.alloc_blob(m, numel)
        blob_b, _ = adacc.alloc_blob(m, numel)
        blob_a.fill_(0x5A)
        blob_b.fill_(0xA5)
        ws = adacc.alloc_workspace(adacc.workspace_bytes(m, numel))
        adacc.compress(m, x, blob_a, ws)
        adacc.compress_noalloc(m, x, blob_b)
        torch.cuda.synchronize()
        a, st_a = used_sections(blob_a, L, m, numel)
        b, st_b = used_sections(blob_b, L, m, numel)
        assert st_a[1] == 0 and st_a[2] == 0 and st_a[0] > 0
        for k in a:
            assert torch.equal(a[k], b[k]), f"{name} rows={rows}: section {k} differs"
        # and the blob decompresses to the same tensor
        da = torch.empty(numel, dtype=torch.bfloat16, device="cuda")
        db = torch.empty(numel, dtype=torch.bfloat16, device="cuda")
        adacc.decompress(m, blob_a, da)
        adacc.decompress(m, blob_b, db)
        torch.cuda.synchronize()
        assert torch.equal(da.view(torch.int16), db.view(torch.int16))


def test_noalloc_without_outliers():
    log("[noalloc] none")
    md = dict(bits=8, quant_group=128, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0)
    x = workloads.c2("cuda", rows=33).view(-1)
    m = adacc_method(md, 0)
    blob_a, L = adacc.alloc_blob(m, x.numel())
    blob_b, _ = adacc.alloc_blob(m, x.numel())
    adacc.compress(m, x, blob_a)
    adacc.compress_noalloc(m, x, blob_b)
    torch.cuda.synchronize()
    a, _ = used_sections(blob_a, L, m, x.numel())
    b, _ = used_sections(blob_b, L, m, x.numel())
    for k in a:
        assert torch.equal(a[k], b[k]), k
