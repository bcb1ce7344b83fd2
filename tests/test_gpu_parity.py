"""GPU parity: libadacc (through the C ABI) against the CPU oracle, element by element.
Bar: bit-exact packed codes, scales, offsets, outlier indices / values / counts / tile
offsets; decompressed binary32 within 1e-6 absolute of the oracle (checked bit-equal as
well); decompressed bf16 equal to the oracle's bf16."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_00806_amd as adacc
import workloads
from helpers import (adacc_method, assert_bf16_matches, assert_f32_matches, bits_of, compare_blob_with_oracle, from_bits, gpu_compress, oracle_method,
                     run_parity)

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


def random_bits(seed, n, heavy=True, edge=True):
    g = np.random.default_rng(seed)
    x = g.standard_normal(n).astype(np.float32)
    if heavy:
        k = max(1, n // 64)
        x[g.choice(n, k, replace=False)] *= 30.0
    t = torch.from_numpy(x).to(torch.bfloat16)
    b = bits_of(t).copy()
    if edge and n >= 64:
        # ties in magnitude, signed zeros, denormals, the largest finite values
        b[1] = 0x8000
        b[2] = 0x0001
        b[3] = 0x8001
        b[5] = b[9] = 0x4110
        b[11] = 0xC110
        b[n - 1] = 0x7F7F
        b[n - 2] = 0xFF7F
    return b


# ------------------------------------------------------------------ the five configurations, reduced
@pytest.mark.parametrize("name,rows", [("c1", 67), ("c2", 37), ("c3", 5), ("c4", 2048)])
def test_config_reduced(name, rows):
    log(f"[parity] config {name} rows={rows}")
    x = workloads.make(name, "cpu", rows=rows)
    md = workloads.METHODS[name]
    cap = workloads.outlier_capacity(md, x.numel(), x.shape[-1])
    oc, *_ = run_parity(x, md, cap=cap)
    log(f"[parity] {name}: numel={x.numel()} n_out={oc.n_out} cap={cap}")
    if name == "c2":
        assert oc.n_out == 2 * rows
    if name == "c4":
        assert 0 < oc.n_out <= cap


def test_config5_layer_reduced():
    for t, (tname, hidden, md) in enumerate(workloads.C5_LAYER):
        if md is None:
            continue
        log(f"[parity] c5 {tname}")
        x = workloads.c5_tensor(tname, "cpu", rows=24, seed=5000 + t)
        cap = workloads.outlier_capacity(md, x.numel(), hidden)
        run_parity(x, md, cap=cap)


# ------------------------------------------------------------------ the whole method space on small tensors
SWEEP = []
for bits in (4, 8):
    for asym in (0, 1):
        for gq, gs in ((8, 8), (16, 64), (64, 64), (128, 512), (512, 512), (128, 1024), (1024, 1024), (256, 2048),
                       (2048, 2048), (128, 4096), (4096, 4096)):
            SWEEP.append((bits, asym, gq, gs))


@pytest.mark.parametrize("mode", ["none", "abs", "std", "topk"])
@pytest.mark.parametrize("rule", [0, 1])
def test_method_sweep(mode, rule):
    for bits, asym, gq, gs in SWEEP:
        groups = 13 if gs <= 1024 else 5   # ragged last tile for most sizes
        n = gs * groups
        x = from_bits(random_bits(1000 * bits + 10 * gq + gs + asym, n))
        md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode=mode, stat_group=gs,
                  thresh={"abs": 2.5, "std": 3.0}.get(mode, 0.0), topk=3 if mode == "topk" else 0)
        log(f"[parity] sweep mode={mode} rule={rule} bits={bits} asym={asym} gq={gq} gs={gs} n={n}")
        run_parity(x, md, rule=rule)


# ------------------------------------------------------------------ edge cases
def test_degenerate_inputs():
    z = np.zeros(4096, dtype=np.uint16)
    const = bits_of(torch.full((4096,), 0.75, dtype=torch.bfloat16))
    tiny = np.zeros(4096, dtype=np.uint16)
    tiny[0], tiny[1], tiny[100] = 0x0001, 0x8001, 0x0080
    huge = np.full(4096, 0x7F7F, dtype=np.uint16)
    huge[::2] = 0xFF7F
    nonfin = random_bits(5, 4096)
    nonfin[7], nonfin[300], nonfin[2049], nonfin[4000] = 0x7F80, 0xFF80, 0x7FC0, 0xFFFF
    for label, b in (("zeros", z), ("const", const), ("tiny", tiny), ("huge", huge), ("nonfinite", nonfin)):
        for mode in ("none", "abs", "std", "topk"):
            for asym in (0, 1):
                if label == "nonfinite" and mode == "none":
                    continue  # nothing is kept aside then: non-finite values are zeroed, covered below
                md = dict(bits=8, quant_group=64, asym=asym, outlier_mode=mode, stat_group=256,
                          thresh={"abs": 1.0, "std": 4.0}.get(mode, 0.0), topk=2 if mode == "topk" else 0)
                log(f"[parity] degenerate {label} mode={mode} asym={asym}")
                run_parity(from_bits(b), md)
    md = dict(bits=4, quant_group=64, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0)
    run_parity(from_bits(nonfin), md)


def topk_corner_case_bits(gs, k, rng):
    """Seven groups: the largest values share a lane, tie at the k-th place, sit in a constant group, or
    come with Inf / NaN, next to groups where the k largest are clear-cut."""
    n_groups = 7
    v = rng.normal(0.0, 1.0, size=gs * n_groups).astype(np.float32)
    b = bits_of(torch.from_numpy(v).to(torch.bfloat16)).copy()
    big = int(bits_of(torch.tensor([50.0], dtype=torch.bfloat16))[0])
    g = lambda i: slice(i * gs, (i + 1) * gs)
    # group 0: the k+1 largest next to each other (one lane holds most of them)
    b[g(0)][8:8 + k + 1] = [big + i for i in range(k + 1)]
    # group 1: k+2 equal maxima spread over the group, negative ones included
    pos = np.sort(rng.choice(gs, size=k + 2, replace=False))
    b[g(1)][pos] = big
    b[g(1)][pos[::2]] |= 0x8000
    # group 2: constant; group 3: all zero with one -0
    b[g(2)] = 0x3F80
    b[g(3)] = 0
    b[g(3)][5] = 0x8000
    # group 4: Inf, NaN and large values together
    b[g(4)][[3, gs // 2, gs // 2 + 9, gs // 2 + 10]] = [0x7F80, 0xFFC1, big, big + 1]
    # group 5: more Inf / NaN than k
    b[g(5)][rng.choice(gs, size=k + 3, replace=False)] = 0xFF80
    # group 6 stays plain random
    return b


def test_topk_selection_corner_cases():
    """TOPK over groups of whole rows."""
    rng = np.random.default_rng(99)
    for gs in (512, 2048, 4096):
        for k in (1, 2, 4, 8, 9):
            b = topk_corner_case_bits(gs, k, rng)
            for bits, gq, asym in ((4, 128, 0), (8, gs, 1)):
                md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode="topk", stat_group=gs, thresh=0.0, topk=k)
                log(f"[parity] topk corner cases gs={gs} k={k} bits={bits} gq={gq} asym={asym}")
                run_parity(from_bits(b), md)


def test_topk_selection_corner_cases_in_groups_inside_a_row():
    """TOPK whose statistics group is the quantisation group and lies inside a 512-element row (the
    row-at-a-time encoder): the same corner cases in groups of 32 .. 512, k up to 32."""
    rng = np.random.default_rng(98)
    for gs in (32, 128, 256, 512):
        for k in (1, 2, 5, 8, 32):  # 32: the most the library takes; for groups of 32 the whole group
            b = topk_corner_case_bits(gs, min(k, 9), rng)
            for bits, asym in ((4, 0), (8, 1), (4, 1)):
                md = dict(bits=bits, quant_group=gs, asym=asym, outlier_mode="topk", stat_group=gs, thresh=0.0, topk=k)
                log(f"[parity] topk in rows gs={gs} k={k} bits={bits} asym={asym}")
                run_parity(from_bits(b), md)
                if k == 1:
                    run_parity(from_bits(b).to(torch.float32).clamp(-6e4, 6e4).to(torch.float16), md)


def test_every_element_an_outlier_and_overflow():
    b = random_bits(77, 2048 * 3 + 512)
    b[(b & 0x7FFF) == 0] = 0x3F80
    md = dict(bits=8, quant_group=64, asym=0, outlier_mode="abs", stat_group=0, thresh=0.0, topk=0)
    log("[parity] all outliers, capacity = numel")
    oc, *_ = run_parity(from_bits(b), md, cap=b.size)
    assert oc.n_out == b.size
    log("[parity] all outliers, capacity 100: overflow flag")
    oc, blob, L, m = run_parity(from_bits(b), md, cap=100, decompress=False)
    st = adacc.read_status(blob, L)
    assert st[0] == b.size and st[1] == 1


def test_empty_and_single_group():
    m = adacc.Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_ABS, thresh=1.0, max_outliers=4)
    blob = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    adacc.compress(m, torch.empty(0, dtype=torch.bfloat16, device="cuda"), blob, None)
    torch.cuda.synchronize()
    assert int(blob.sum()) == 0
    for gq in (8, 64, 4096):
        md = dict(bits=4, quant_group=gq, asym=1, outlier_mode="topk", stat_group=gq, thresh=0.0, topk=1)
        log(f"[parity] single group gq={gq}")
        run_parity(from_bits(random_bits(gq, gq, heavy=False, edge=False)), md)


def test_many_tiles_across_placement_blocks():
    """Enough tiles for ten placement blocks and a ragged last one, every CU busy."""
    n = 2048 * 5000 + 1024
    b = random_bits(123, n)
    md = dict(bits=8, quant_group=128, asym=0, outlier_mode="std", stat_group=1024, thresh=5.0, topk=0)
    log(f"[parity] many tiles n={n}")
    oc, *_ = run_parity(from_bits(b), md)
    assert oc.n_out > 10000
    # sparse outliers: most tiles, and whole placement blocks, are empty
    b2 = bits_of(torch.from_numpy(np.random.default_rng(3).standard_normal(n).astype(np.float32)).to(torch.bfloat16))
    md2 = dict(bits=4, quant_group=64, asym=0, outlier_mode="abs", stat_group=0, thresh=4.6, topk=0)
    oc2, *_ = run_parity(from_bits(b2), md2)
    log(f"[parity] sparse n_out={oc2.n_out}")
    assert 0 < oc2.n_out < 200


def test_dense_outliers_overflow_the_slots():
    """About 5 % outliers: a tile holds around a hundred, more than its slot takes, so the placement
    kernel selects the outliers of (nearly) every tile a second time from the source."""
    n = 2048 * 9001
    rng = np.random.default_rng(4242)
    v = rng.normal(0.0, 1.0, size=n).astype(np.float32)
    x = torch.from_numpy(v).to(torch.bfloat16)
    for mode, thresh, gq, gs, asym in (("abs", 1.96, 64, 0, 0), ("std", 1.96, 2048, 2048, 1)):
        md = dict(bits=8, quant_group=gq, asym=asym, outlier_mode=mode, stat_group=gs, thresh=thresh, topk=0)
        log(f"[parity] dense outliers mode={mode} n={n}")
        oc, *_ = run_parity(x, md)
        assert oc.n_out > n // 25


def test_decompression_with_few_many_and_crowded_outliers_per_tile():
    """The decompression takes up to 64 outliers of a tile, no two in one octet, into the output in registers
    and writes them over the stored piece otherwise: tiles with 1, 63, 64 and 65 outliers in octets of their
    own, with two and with eight in one octet, and tiles of 4096 elements whose outliers lie in one half, in
    both halves (fewer and more than 64 together)."""
    rng = np.random.default_rng(4242)
    small = bits_of(torch.from_numpy(rng.uniform(-0.5, 0.5, size=2048 * 8).astype(np.float32)).to(torch.bfloat16)).copy()
    big = int(bits_of(torch.tensor([8.0], dtype=torch.bfloat16))[0])

    def plant(b, tile, tile_elems, positions):
        for j, p in enumerate(positions):
            b[tile * tile_elems + p] = (big + j % 5) | (0x8000 if j % 3 == 0 else 0)

    b = small.copy()
    octets = rng.permutation(256)
    plant(b, 0, 2048, [int(o) * 8 + int(rng.integers(8)) for o in octets[:1]])
    plant(b, 1, 2048, [int(o) * 8 + int(rng.integers(8)) for o in octets[:63]])
    plant(b, 2, 2048, [int(o) * 8 + int(rng.integers(8)) for o in octets[:64]])
    plant(b, 3, 2048, [int(o) * 8 + int(rng.integers(8)) for o in octets[:65]])
    plant(b, 4, 2048, [800, 803, 17])                 # two in one octet
    plant(b, 5, 2048, list(range(1024, 1032)) + [5])  # a whole octet
    plant(b, 7, 2048, [2047])                         # tile 6 has none
    for bits, gq, asym in ((4, 128, 0), (8, 64, 1)):
        md = dict(bits=bits, quant_group=gq, asym=asym, outlier_mode="abs", stat_group=0, thresh=4.0, topk=0)
        log(f"[parity] outliers per tile bits={bits}")
        oc, _, _, _ = run_parity(from_bits(b), md)
        assert oc.n_out == 1 + 63 + 64 + 65 + 3 + 9 + 1
    # tiles of 4096 elements (statistics over 4096), decompressed in halves
    b = np.tile(small, 2)[:4096 * 4].copy()
    plant(b, 0, 4096, [int(o) * 8 for o in octets[:20]])                                      # first half only
    plant(b, 1, 4096, [int(o) * 8 for o in octets[:30]] + [2048 + int(o) * 8 for o in octets[:30]])  # 60: both halves in registers
    plant(b, 2, 4096, [int(o) * 8 for o in octets[:40]] + [2048 + int(o) * 8 for o in octets[:40]])  # 80: both halves through memory
    plant(b, 3, 4096, [4095])
    md = dict(bits=4, quant_group=128, asym=0, outlier_mode="std", stat_group=4096, thresh=3.0, topk=0)
    log("[parity] outliers per 4096-tile")
    oc, _, _, _ = run_parity(from_bits(b), md)
    assert oc.n_out == 20 + 60 + 80 + 1


@pytest.mark.parametrize("gs,k,gq,bits", [(2048, 2, 128, 4), (4096, 4, 128, 4), (64, 1, 64, 8), (4096, 3, 4096, 8)])
def test_topk_groups_with_more_values_that_are_not_finite_than_k(gs, k, gq, bits):
    """TOPK places its outliers at offsets known in advance (k per group).  A group that holds more
    than k values that are not finite breaks that: every later offset shifts, and the placement
    kernel redoes the stream from the source.  Three placement blocks, irregular groups in the
    first tile, in the middle and in the last tile, then a regular tensor through the same workspace."""
    tile = max(2048, gs)
    n = tile * 1300
    b = random_bits(900 + gs + k, n, heavy=True, edge=False)
    for g0 in (0, (n // gs // 2) * gs, n - gs):
        b[g0 + 1:g0 + gs:max(1, gs // (k + 3))] = 0x7F80  # k + 3 or more infinities in this group
        b[g0 + 5] = 0xFFC0
    md = dict(bits=bits, quant_group=gq, asym=0, outlier_mode="topk", stat_group=gs, thresh=0.0, topk=k)
    log(f"[parity] irregular topk gs={gs} k={k} n={n}")
    oc, blob, L, m = run_parity(from_bits(b), md)
    assert oc.n_out > k * (n // gs)
    ws = adacc.alloc_workspace(adacc.workspace_bytes(m, n))
    regular = random_bits(901 + gs, n, heavy=True, edge=False)  # finite values only
    for bb in (b, regular, b):  # the flag of the first call must not reach the second
        occ = oracle.compress(oracle_method(md), bb)
        occ._full_idx = occ.out_idx.astype(np.int64)
        mm = adacc_method(md, max(occ.n_out, 1))
        blob2, L2, _ = gpu_compress(from_bits(bb, "cuda"), mm, ws=ws)
        torch.cuda.synchronize()
        compare_blob_with_oracle(blob2, L2, mm, n, occ)


def test_deterministic_and_workspace_reuse():
    """One workspace, many calls of different sizes and methods: every blob equals the oracle's,
    and repeated calls give identical bytes."""
    cases = [(2048 * 700 + 64, dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=2.5, topk=0)),
             (4096 * 9, dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=4096, thresh=0.0, topk=4)),
             (2048 * 3, dict(bits=8, quant_group=2048, asym=1, outlier_mode="abs", stat_group=0, thresh=2.0, topk=0)),
             (2048 * 1500, dict(bits=4, quant_group=32, asym=1, outlier_mode="abs", stat_group=0, thresh=3.0, topk=0))]
    ws = adacc.alloc_workspace(max(adacc.workspace_bytes(adacc_method(md, 1), n) for n, md in cases))
    for rep in range(3):
        for i, (n, md) in enumerate(cases):
            b = random_bits(50 + i, n)
            om = oracle_method(md)
            oc = oracle.compress(om, b)
            oc._full_idx = oc.out_idx.astype(np.int64)
            m = adacc_method(md, max(oc.n_out, 1))
            x = from_bits(b, "cuda")
            log(f"[parity] reuse rep={rep} case={i} n={n}")
            blob, L, _ = gpu_compress(x, m, ws=ws)
            torch.cuda.synchronize()
            compare_blob_with_oracle(blob, L, m, n, oc)
            first = blob.clone()
            for _ in range(5):
                blob.zero_()
                adacc.compress(m, x, blob, ws)
            torch.cuda.synchronize()
            used = int(L.status_off) + 16
            sec_a = adacc.blob_sections(first, L, m, n)
            sec_b = adacc.blob_sections(blob, L, m, n)
            for k in ("codes", "scales", "tile_ptr", "status"):
                assert torch.equal(sec_a[k], sec_b[k]), k
            assert torch.equal(sec_a["idx"][:oc.n_out], sec_b["idx"][:oc.n_out])
            assert torch.equal(sec_a["val"][:oc.n_out], sec_b["val"][:oc.n_out])
            assert used <= L.total_bytes


def test_epoch_wrap_clears_the_workspace():
    """The launch counter of a workspace is 30 bits wide: at the wrap the library clears the state
    words and starts over.  Force the wrap from the host and check parity on both sides of it."""
    n = 2048 * 300
    md = dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=256, thresh=3.0, topk=0)
    b = random_bits(31, n)
    oc = oracle.compress(oracle_method(md), b)
    oc._full_idx = oc.out_idx.astype(np.int64)
    m = adacc_method(md, max(oc.n_out, 1))
    x = from_bits(b, "cuda")
    ws = adacc.alloc_workspace(adacc.workspace_bytes(m, n))
    for start in (0x3FFFFFFD, None, None, None):
        if start is not None:
            ws.c.epoch = start
        log(f"[parity] epoch before call = {ws.c.epoch:#x}")
        blob, L, _ = gpu_compress(x, m, ws=ws)
        torch.cuda.synchronize()
        compare_blob_with_oracle(blob, L, m, n, oc)
    assert ws.c.epoch == 2  # 0x3FFFFFFE, 0x3FFFFFFF, then cleared: 1, 2


# ------------------------------------------------------------------ batch
def test_batch_matches_single_calls_and_oracle():
    rows = 12
    table = []
    for layer in range(2):
        for t, (tname, hidden, md) in enumerate(workloads.C5_LAYER):
            x = workloads.c5_tensor(tname, "cpu", rows=rows, seed=5000 + 10 * layer + t)
            table.append((tname, hidden, md, x))
    # an asymmetric + abs entry and a tiny ragged tensor, to mix more variants into one launch
    table.append(("softmax", 2048, workloads.C4_METHOD, workloads.c4("cpu", rows=2048)[:64].contiguous()))
    table.append(("small", 64, dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=2.0, topk=0),
                  from_bits(random_bits(9, 64 * 5)).view(5, 64)))
    # TOPK over the quantisation groups (the row-at-a-time encoder inside the batch kernel): a regular tensor,
    # and one whose first group holds more values that are not finite than k (placed again from the source)
    top1 = dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=128, thresh=0.0, topk=1)
    table.append(("top1", 128, top1, from_bits(random_bits(10, 128 * 70, edge=False)).view(70, 128)))
    irregular = random_bits(11, 128 * 50, edge=False)
    irregular[[3, 40, 77]] = [0x7F80, 0xFF80, 0x7FC0]
    table.append(("top1-irregular", 128, top1, from_bits(irregular).view(50, 128)))
    methods, srcs, blobs, layouts, ocs = [], [], [], [], []
    for tname, hidden, md, x in table:
        n = x.numel()
        if md is None:
            methods.append(adacc.NOOP); srcs.append(x.cuda()); blobs.append(None); layouts.append(None); ocs.append(None)
            continue
        cap = workloads.outlier_capacity(md, n, hidden)
        m = adacc_method(md, cap)
        oc = oracle.compress(oracle_method(md), bits_of(x), cap=cap)
        assert oc.n_out <= cap
        oc._full_idx = oc.out_idx.astype(np.int64)
        blob, L = adacc.alloc_blob(m, n)
        methods.append(m); srcs.append(x.contiguous().view(-1).cuda()); blobs.append(blob); layouts.append(L); ocs.append(oc)
    numels = [s.numel() for s in srcs]
    ws = adacc.alloc_workspace(adacc.batch_workspace_bytes(methods, numels))
    prepared = adacc.prepare_compress_batch(methods, srcs, blobs)  # the argument arrays, marshalled once
    for rep in range(3):
        log(f"[parity] batch compress rep={rep} tensors={len(methods)}")
        for b in blobs:
            if b is not None:
                b.zero_()
        adacc.compress_batch(methods, srcs, blobs, ws, prepared=prepared if rep else None)
        torch.cuda.synchronize()
        for (tname, hidden, md, x), m, blob, L, oc in zip(table, methods, blobs, layouts, ocs):
            if md is None:
                continue
            compare_blob_with_oracle(blob, L, m, x.numel(), oc)
    # decompress: batch, both dtypes, against the oracle
    for dtype in (torch.bfloat16, torch.float32):
        dsts = [None if b is None else torch.empty(s.numel(), dtype=dtype, device="cuda") for s, b in zip(srcs, blobs)]
        log(f"[parity] batch decompress {dtype}")
        adacc.decompress_batch(methods, blobs, dsts, ws, prepared=adacc.prepare_decompress_batch(methods, blobs, dsts))
        torch.cuda.synchronize()
        for d, oc in zip(dsts, ocs):
            if d is None:
                continue
            of32, obf = oracle.decompress(oc)
            if dtype == torch.float32:
                assert_f32_matches(d.cpu().numpy(), of32)
            else:
                assert_bf16_matches(bits_of(d), obf)
    # the retained tensor was not touched
    assert torch.equal(srcs[4].cpu().view(-1), table[4][3].contiguous().view(-1))


# ------------------------------------------------------------------ full-size configurations, sampled
def check_compressed_tiles(name, xf, md, m, blob, L, tiles):
    """The blob of a whole tensor against the oracle on the given tiles (every group lies inside one tile,
    so a tile can be checked alone), plus what holds for the whole outlier stream.  Returns the status."""
    numel = xf.numel()
    st = adacc.read_status(blob, L)
    assert st[1] == 0 and st[2] == 0, (name, st)
    sec = adacc.blob_sections(blob, L, m, numel)
    te = int(L.tile_elems)
    has_out = md["outlier_mode"] != "none"
    if has_out:
        tp = sec["tile_ptr"].cpu().numpy().view(np.uint32).astype(np.int64)
        assert tp[0] == 0 and np.all(np.diff(tp) >= 0) and tp[-1] == st[0], name
        idx = sec["idx"][:st[0]]
        assert bool((idx[1:] > idx[:-1]).all()), f"{name}: outlier stream is not strictly ascending"
    om = oracle_method(md)
    cb, gq = md["bits"], md["quant_group"]
    for t in tiles:
        lo, hi = t * te, min(numel, (t + 1) * te)
        oc = oracle.compress(om, bits_of(xf[lo:hi]))
        got_codes = sec["codes"][lo * cb // 8: hi * cb // 8].cpu().numpy()
        assert np.array_equal(got_codes, oc.packed), (name, t)
        assert np.array_equal(sec["scales"][lo // gq: hi // gq].cpu().numpy().view(np.uint32), oc.scale.view(np.uint32)), (name, t)
        if md["asym"]:
            assert np.array_equal(sec["zp"][lo // gq: hi // gq].cpu().numpy().view(np.uint32), oc.zp.view(np.uint32)), (name, t)
        if has_out:
            p0, p1 = int(tp[t]), int(tp[t + 1])
            assert p1 - p0 == oc.n_out, (name, t, p1 - p0, oc.n_out)
            assert np.array_equal(sec["idx"][p0:p1].cpu().numpy().astype(np.int64), oc.out_idx.astype(np.int64) + lo), (name, t)
            assert np.array_equal(sec["val"][p0:p1].cpu().numpy().view(np.uint16), oc.out_val), (name, t)
    return st


def check_restored_tiles(name, xf, md, m, blob, L, dst, tiles):
    """The bf16 output on the given tiles equals the oracle's reconstruction; every outlier of the whole
    tensor comes back exactly."""
    numel = xf.numel()
    te = int(L.tile_elems)
    om = oracle_method(md)
    for t in tiles:
        lo, hi = t * te, min(numel, (t + 1) * te)
        _, obf = oracle.decompress(oracle.compress(om, bits_of(xf[lo:hi])))
        assert np.array_equal(bits_of(dst[lo:hi]), obf), (name, t)
    n_out = adacc.read_status(blob, L)[0]
    if md["outlier_mode"] != "none" and n_out > 0:
        ii = adacc.blob_sections(blob, L, m, numel)["idx"][:n_out].long()
        assert torch.equal(dst[ii].view(torch.int16), xf[ii].view(torch.int16)), name


def sampled_tiles(g, n_tiles, n_samples):
    return sorted(set([0, n_tiles - 1] + g.integers(0, n_tiles, n_samples).tolist()))


def sampled_full_size(name, x_dev, md, hidden, n_samples=24):
    """Compress the full tensor on the GPU in the launch configuration the bench uses; run the
    oracle on sampled tiles."""
    numel = x_dev.numel()
    m = adacc_method(md, workloads.outlier_capacity(md, numel, hidden))
    xf = x_dev.view(-1)
    blob, L, ws = gpu_compress(xf, m)
    torch.cuda.synchronize()
    tiles = sampled_tiles(np.random.default_rng(2024), L.n_tiles, n_samples)
    st = check_compressed_tiles(name, xf, md, m, blob, L, tiles)
    dst = torch.empty(numel, dtype=torch.bfloat16, device="cuda")
    adacc.decompress(m, blob, dst)
    torch.cuda.synchronize()
    check_restored_tiles(name, xf, md, m, blob, L, dst, tiles)
    return st


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_full_size_sampled(name):
    log(f"[parity] full size {name}")
    x = workloads.make(name, "cuda")
    st = sampled_full_size(name, x, workloads.METHODS[name], x.shape[-1])
    log(f"[parity] full size {name}: n_out={st[0]}")
    if name == "c2":
        assert st[0] == 2 * x.shape[0]
    del x
    torch.cuda.empty_cache()


def c5_batch(layers):
    """The saved tensors of `layers` LLaMA-7B-shaped layers on the GPU with their methods, blobs and layouts,
    seeded as the bench seeds them."""
    names, mds, methods, srcs, blobs, layouts = [], [], [], [], [], []
    for layer, tname, x, md in workloads.c5("cuda", layers=layers):
        n = x.numel()
        m = adacc_method(md, workloads.outlier_capacity(md, n, x.shape[-1]))
        blob, L = (None, None) if md is None else adacc.alloc_blob(m, n)
        names.append(f"L{layer}.{tname}"); mds.append(md); methods.append(m); srcs.append(x.view(-1))
        blobs.append(blob); layouts.append(L)
    return names, mds, methods, srcs, blobs, layouts


def run_c5_batch(layers, n_samples):
    """Batched compression and decompression in the configuration the bench times (argument arrays
    prepared once, one workspace for the whole set); the oracle on sampled tiles of every tensor; then
    every tensor again through the single-tensor decompression, last tensor first, as a backward pass
    would ask for them."""
    names, mds, methods, srcs, blobs, layouts = c5_batch(layers)
    numels = [x.numel() for x in srcs]
    ws = adacc.alloc_workspace(adacc.batch_workspace_bytes(methods, numels))
    dsts = [None if md is None else torch.empty(n, dtype=torch.bfloat16, device="cuda") for md, n in zip(mds, numels)]
    cargs = adacc.prepare_compress_batch(methods, srcs, blobs)
    dargs = adacc.prepare_decompress_batch(methods, blobs, dsts)
    log(f"[parity] c5 x{layers} layers: batch compress of {len(srcs)} tensors")
    adacc.compress_batch(methods, srcs, blobs, ws, prepared=cargs)
    torch.cuda.synchronize()
    log(f"[parity] c5 x{layers} layers: batch decompress")
    adacc.decompress_batch(methods, blobs, dsts, ws, prepared=dargs)
    torch.cuda.synchronize()
    g = np.random.default_rng(7)
    total_out = 0
    for name, md, m, x, blob, L, dst in zip(names, mds, methods, srcs, blobs, layouts, dsts):
        if md is None:
            continue
        tiles = sampled_tiles(g, L.n_tiles, n_samples)
        st = check_compressed_tiles(name, x, md, m, blob, L, tiles)
        if md["outlier_mode"] == "topk":
            assert st[0] == md["topk"] * (x.numel() // md["stat_group"]), name
        total_out += st[0]
        check_restored_tiles(name, x, md, m, blob, L, dst, tiles)
    log(f"[parity] c5 x{layers} layers: {total_out} outliers; single-tensor decompress in reverse order")
    scratch = torch.empty(max(numels), dtype=torch.bfloat16, device="cuda")
    for i in reversed(range(len(srcs))):
        if mds[i] is None:
            continue
        out = scratch[:numels[i]]
        adacc.decompress(methods[i], blobs[i], out)
        assert torch.equal(out.view(torch.int16), dsts[i].view(torch.int16)), names[i]
    del srcs, blobs, dsts, scratch, ws
    torch.cuda.empty_cache()


def test_full_size_c5_one_layer_batch_sampled():
    """One LLaMA-7B-shaped layer at its real shape through the batch entry points."""
    run_c5_batch(1, 8)


def test_full_size_c5_all_layers_batch_sampled():
    """The whole C5 layer set (32 layers, 160 tensors, 20 GiB of bf16) exactly as the bench launches it."""
    run_c5_batch(workloads.C5_LAYERS, 4)


# ------------------------------------------------------------------ the largest sizes the library takes
def check_sampled(name, xf, md, m, blob, L, dst, n_samples, seed):
    tiles = sampled_tiles(np.random.default_rng(seed), L.n_tiles, n_samples)
    st = check_compressed_tiles(name, xf, md, m, blob, L, tiles[:-1])  # the last tile may be short: checked by its own slice
    check_restored_tiles(name, xf, md, m, blob, L, dst, tiles[:-1])
    return st


def test_offsets_beyond_32_bits():
    """Without outliers a tensor may have more than 2^32 elements (element offsets, code offsets and
    group numbers are 64-bit): 2^32 + 6152 bf16 values, int4 in groups of 128 - the length is no multiple of
    the group, so the last 8 elements are a short group.  Oracle on tiles sampled over the whole range and
    on the end of the tensor."""
    n = (1 << 32) + 3 * 2048 + 8
    log(f"[parity] {n} elements without outliers")
    x = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(4242)
    step = 1 << 28
    for i0 in range(0, n, step):
        x[i0:i0 + step].normal_(0.0, 1.5, generator=g)
    md = dict(bits=4, quant_group=128, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0)
    m = adacc_method(md, 0)
    blob, L = adacc.alloc_blob(m, n)
    adacc.compress(m, x, blob, None)
    dst = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    adacc.decompress(m, blob, dst)
    torch.cuda.synchronize()
    assert L.n_tiles == (n + 2047) // 2048
    check_sampled("beyond 2^32", x, md, m, blob, L, dst, 24, 11)
    # the end: the last whole tiles and the short group, against the oracle on that slice
    lo = n - (2048 + 8)
    oc = oracle.compress(oracle_method(md), bits_of(x[lo:]))
    sec = adacc.blob_sections(blob, L, m, n)
    assert np.array_equal(sec["codes"][lo // 2:].cpu().numpy(), oc.packed)
    assert np.array_equal(sec["scales"][lo // 128:].cpu().numpy().view(np.uint32), oc.scale.view(np.uint32))
    assert np.array_equal(bits_of(dst[lo:]), oracle.decompress(oc)[1])
    del x, dst, blob
    torch.cuda.empty_cache()


def test_the_longest_tensor_that_keeps_outliers():
    """Outlier indices are 32-bit signed: 2^31 - 2048 elements is the longest tensor in a mode that keeps
    outliers.  STD in groups of 64 (row encoder, slots, block sums over 4096 blocks) and TOPK over 4096."""
    n = (1 << 31) - 2048
    x = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(777)
    step = 1 << 28
    for i0 in range(0, n, step):
        x[i0:i0 + step].normal_(0.0, 1.0, generator=g)
    x[n - 5] = 1000.0   # an outlier at the very end: its index is close to 2^31
    dst = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    for md, cap in ((dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=3.5, topk=0), n // 256),
                    (dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=4096, thresh=0.0, topk=2), n // 2048 + 8)):
        log(f"[parity] {n} elements, {md['outlier_mode']}")
        m = adacc_method(md, cap)
        blob, L = adacc.alloc_blob(m, n)
        ws = adacc.alloc_workspace(adacc.workspace_bytes(m, n))
        adacc.compress(m, x, blob, ws)
        adacc.decompress(m, blob, dst)
        torch.cuda.synchronize()
        st = check_sampled("longest with outliers", x, md, m, blob, L, dst, 24, 5)
        sec = adacc.blob_sections(blob, L, m, n)
        assert st[1] == 0 and (n - 5) in sec["idx"][st[0] - 2:st[0]].cpu().tolist()
        assert int(bits_of(dst[n - 5:n - 4])[0]) == int(bits_of(x[n - 5:n - 4])[0])
        if md["outlier_mode"] == "topk":
            assert st[0] == 2 * (n // 4096) + 2  # the last tile is half a group short: a tail of 2048 elements
        del blob, ws
        torch.cuda.empty_cache()
    del x, dst
    torch.cuda.empty_cache()
