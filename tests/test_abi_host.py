"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, computes layouts, and rejects bad calls before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2508_00806_amd as adacc
from paper_2508_00806_amd import Method

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(adacc.LIB_PATH):
        from paper_2508_00806_amd.build import build
        build()
    return adacc.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "adacc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adacc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert set(names) == set(adacc.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_struct_sizes_match_the_header(L):
    assert ctypes.sizeof(adacc.CMethod) == 44
    assert ctypes.sizeof(adacc.CLayout) == 72
    assert ctypes.sizeof(adacc.CWorkspace) == 24


def test_layout_closed_form(L):
    m = Method(bits=4, quant_group=128, outlier_mode=adacc.OUTLIER_TOPK, stat_group=2048, topk=2, max_outliers=1000)
    n = 2048 * 37
    lay = adacc.layout_of(m, n)
    assert lay.tile_elems == 2048 and lay.n_tiles == 37
    a = lambda v: (v + 255) // 256 * 256
    assert lay.codes_off == 0
    assert lay.scales_off == a(n // 2)
    assert lay.zp_off == lay.scales_off + a(4 * n // 128)
    assert lay.tile_ptr_off == lay.zp_off
    assert lay.idx_off == lay.tile_ptr_off + a(4 * 38)
    assert lay.val_off == lay.idx_off + a(4000)
    assert lay.status_off == lay.val_off + a(2000)
    assert lay.total_bytes == lay.status_off + 256
    # stat group 4096 -> 4096-element tiles; ragged tail rounds up
    m2 = Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_STD, stat_group=4096, thresh=3.0, max_outliers=8)
    lay2 = adacc.layout_of(m2, 4096 * 3)
    assert lay2.tile_elems == 4096 and lay2.n_tiles == 3
    m3 = Method(bits=8, quant_group=64)
    lay3 = adacc.layout_of(m3, 64 * 33)
    assert lay3.tile_elems == 2048 and lay3.n_tiles == 2 and lay3.tile_ptr_off == lay3.idx_off == lay3.val_off
    # no-op: nothing
    lay0 = adacc.layout_of(adacc.NOOP, 12345)
    assert lay0.total_bytes == 0 and lay0.n_tiles == 0
    # workspace: one count per tile and a flag word; threshold modes add one sum per block of 256 tiles and a slot
    # of 32 (index, value) records of 8 bytes per tile
    assert adacc.workspace_bytes(m, n) == a(4 * 37) + 256
    assert adacc.workspace_bytes(m2, 4096 * 3) == a(4 * 3) + 256 + a(4 * 1) + a(8 * 32 * 3)
    assert adacc.workspace_bytes(m3, 64 * 33) == 0


BAD = [
    Method(bits=5, quant_group=64),
    Method(bits=8, quant_group=44),      # no multiple of 8
    Method(bits=8, quant_group=4),
    Method(bits=8, quant_group=16392),   # beyond the longest segment
    Method(bits=8, quant_group=64, asym=2),
    Method(bits=8, quant_group=64, scale_rule=2),
    Method(bits=8, quant_group=64, outlier_mode=4),
    Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_STD, stat_group=32, thresh=1.0),
    Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_STD, stat_group=16448, thresh=1.0),
    Method(bits=8, quant_group=48, outlier_mode=adacc.OUTLIER_STD, stat_group=100, thresh=1.0),  # no multiple of the quant group
    Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_STD, stat_group=64, thresh=-1.0),
    Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_ABS, thresh=float("nan")),
    Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_TOPK, stat_group=64, topk=0),
    Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_TOPK, stat_group=64, topk=33),
    Method(kind=7, bits=8, quant_group=64),
]


def test_group_sizes_of_the_fallback_kernels(L):
    """Quantisation groups of any multiple of 8 and statistics groups up to 16384: the tile is the largest
    multiple of the larger group up to 4096 (the group itself beyond that); the workspace as for the tile kernels:
    counts and the flag, and for ABS / STD the blocks' sums and a slot of 32 records per segment."""
    a = lambda v: (v + 255) // 256 * 256
    m = Method(bits=8, quant_group=48)
    lay = adacc.layout_of(m, 10000)
    assert lay.tile_elems == 48 * 85 and lay.n_tiles == 3 and lay.scales_off == a(10000)
    assert lay.zp_off - lay.scales_off == a(4 * 209)  # 208 whole groups and one of 16 elements
    row = Method(bits=4, quant_group=128, outlier_mode=adacc.OUTLIER_TOPK, stat_group=11008, topk=8, max_outliers=800)
    lay = adacc.layout_of(row, 11008 * 100)
    assert lay.tile_elems == 11008 and lay.n_tiles == 100
    assert adacc.workspace_bytes(row, 11008 * 100) == a(4 * 100) + 256
    big = Method(bits=8, quant_group=8192, outlier_mode=adacc.OUTLIER_ABS, thresh=1.0, max_outliers=10)
    assert adacc.layout_of(big, 8192 * 5 + 1).tile_elems == 8192 and adacc.layout_of(big, 8192 * 5 + 1).n_tiles == 6
    assert adacc.workspace_bytes(big, 8192 * 5 + 1) == a(4 * 6) + 256 + a(4 * 1) + a(8 * 32 * 6)
    cm = adacc.ChannelMethod(bits=4, quant_group=48, max_channels=4)
    with pytest.raises(adacc.AdaccError):
        adacc.channel_layout_of(cm, 12, 96)  # the channel scheme keeps to powers of two


@pytest.mark.parametrize("m", BAD)
def test_malformed_methods(L, m):
    with pytest.raises(adacc.AdaccError) as e:
        adacc.layout_of(m, 4096)
    assert e.value.code == adacc.EINVAL


def test_numel_rules(L):
    m = Method(bits=8, quant_group=64)
    a = lambda v: (v + 255) // 256 * 256
    lay = adacc.layout_of(m, 100)  # the group does not divide numel: two groups, the second of 36 elements
    assert (lay.scales_off, lay.zp_off - lay.scales_off, lay.n_tiles) == (a(100), a(4 * 2), 1)
    m4 = Method(bits=4, quant_group=128, outlier_mode=adacc.OUTLIER_TOPK, stat_group=2048, topk=2, max_outliers=64)
    lay = adacc.layout_of(m4, 2048 * 3 + 77)  # int4, odd length: the last byte holds one element
    assert lay.scales_off == a((2048 * 3 + 77 + 1) // 2) and lay.n_tiles == 4
    assert lay.idx_off - lay.tile_ptr_off == a(4 * 5)
    assert adacc.compressed_bytes(m4, 2048 * 3 + 77, 7) == (2048 * 3 + 78) // 2 + 4 * 49 + 6 * 7 + 4 * 5
    cm = adacc.ChannelMethod(bits=4, quant_group=128, max_channels=4)
    with pytest.raises(adacc.AdaccError):
        adacc.channel_layout_of(cm, 3, 200)  # with outlier channels the group still has to divide the tensor
    mo = Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_ABS, thresh=1.0, max_outliers=4)
    with pytest.raises(adacc.AdaccError):
        adacc.layout_of(mo, 1 << 31)  # 32-bit indices
    assert adacc.layout_of(m, 1 << 31).n_tiles == (1 << 31) // 2048


def test_errors_are_returned_before_any_device_work(L):
    """Fake device addresses: a call that got past validation would fault, so reaching the
    error code proves the checks come first."""
    m = Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_ABS, thresh=1.0, max_outliers=16)
    n = 4096
    lay = adacc.layout_of(m, n)
    cm = m.c()
    src, blob = 0x10000, 0x20000
    ws = adacc.CWorkspace(0x30000, 4096, 0, 0)
    small = adacc.CWorkspace(0x30000, 8, 0, 0)
    empty = adacc.CWorkspace(None, 4096, 0, 0)
    odd = adacc.CWorkspace(0x30010, 4096, 0, 0)
    w = ctypes.byref(ws)
    f = L.adacc_compress
    assert f(None, src, n, blob, lay.total_bytes, w, None) == adacc.ENULL
    assert f(ctypes.byref(cm), None, n, blob, lay.total_bytes, w, None) == adacc.ENULL
    assert f(ctypes.byref(cm), src, n, None, lay.total_bytes, w, None) == adacc.ENULL
    assert f(ctypes.byref(cm), src, n, blob, lay.total_bytes, None, None) == adacc.ENULL
    assert f(ctypes.byref(cm), src, n, blob, lay.total_bytes, ctypes.byref(empty), None) == adacc.ENULL
    assert f(ctypes.byref(cm), src, n, blob, lay.total_bytes - 1, w, None) == adacc.ESIZE
    assert f(ctypes.byref(cm), src, n, blob, lay.total_bytes, ctypes.byref(small), None) == adacc.ESIZE
    assert f(ctypes.byref(cm), src + 2, n, blob, lay.total_bytes, w, None) == adacc.EALIGN
    assert f(ctypes.byref(cm), src, n, blob + 16, lay.total_bytes, w, None) == adacc.EALIGN
    assert f(ctypes.byref(cm), src, n, blob, lay.total_bytes, ctypes.byref(odd), None) == adacc.EALIGN
    assert f(ctypes.byref(cm), src, 1 << 31, blob, lay.total_bytes, w, None) == adacc.EINVAL  # 32-bit indices
    assert f(ctypes.byref(cm), src, n + 1, blob, lay.total_bytes, w, None) == adacc.ESIZE   # one more group
    assert ws.epoch == 0  # a rejected call does not consume an epoch
    # nothing to do: OK without looking at the pointers
    assert f(ctypes.byref(cm), None, 0, None, 0, None, None) == adacc.OK
    noop = adacc.NOOP.c()
    assert f(ctypes.byref(noop), None, n, None, 0, None, None) == adacc.OK
    g = L.adacc_decompress
    assert g(ctypes.byref(cm), blob, lay.total_bytes, n, None, 0, None) == adacc.ENULL
    assert g(ctypes.byref(cm), blob, lay.total_bytes, n, 0x40000, 2, None) == adacc.EINVAL
    assert g(ctypes.byref(cm), blob, lay.total_bytes - 1, n, 0x40000, 0, None) == adacc.ESIZE
    assert g(ctypes.byref(cm), blob, lay.total_bytes, n, 0x40002, 0, None) == adacc.EALIGN
    assert L.adacc_hbm_copy(0x10000, 0x20000, 24, None) == adacc.EINVAL
    assert L.adacc_workspace_init(None, 0x10000, 4096, None) == adacc.ENULL
    assert L.adacc_workspace_init(w, None, 4096, None) == adacc.ENULL
    assert L.adacc_workspace_init(w, 0x10000, 8, None) == adacc.ESIZE
    assert L.adacc_workspace_init(w, 0x10010, 4096, None) == adacc.EALIGN


def test_batch_validation(L):
    ms = [Method(bits=4, quant_group=128, outlier_mode=adacc.OUTLIER_TOPK, stat_group=4096, topk=4, max_outliers=64),
          adacc.NOOP, Method(bits=8, quant_group=128)]
    numels = [4096 * 5, 999, 128 * 100]
    need = adacc.batch_workspace_bytes(ms, numels)
    a = lambda v: (v + 255) // 256 * 256
    assert need >= adacc.workspace_bytes(ms[0], numels[0]) + 2 * 128 + 2 * a(4 * 3)
    n = 3
    cms = (adacc.CMethod * n)(*[m.c() for m in ms])
    cn = (ctypes.c_uint64 * n)(*numels)
    srcs = (ctypes.c_void_p * n)(0x10000, None, 0x20000)
    blobs = (ctypes.c_void_p * n)(0x100000, None, 0x200000)
    bb = (ctypes.c_uint64 * n)(adacc.layout_of(ms[0], numels[0]).total_bytes, 0,
                               adacc.layout_of(ms[2], numels[2]).total_bytes)
    f = L.adacc_compress_batch
    ws = adacc.CWorkspace(0x300000, need, 0, 0)
    small = adacc.CWorkspace(0x300000, need - 256, 0, 0)
    assert f(n, cms, srcs, cn, blobs, bb, ctypes.byref(small), None) == adacc.ESIZE
    assert f(n, cms, srcs, cn, blobs, bb, None, None) == adacc.ENULL
    bb[2] -= 1
    assert f(n, cms, srcs, cn, blobs, bb, ctypes.byref(ws), None) == adacc.ESIZE
    bb[2] += 1
    srcs[0] = None
    assert f(n, cms, srcs, cn, blobs, bb, ctypes.byref(ws), None) == adacc.ENULL
    assert f(0, None, None, None, None, None, None, None) == adacc.OK
    assert ws.epoch == 0


def test_strerror_and_version(L):
    assert adacc.strerror(0) == "ok"
    assert "align" in adacc.strerror(adacc.EALIGN)
    assert re.match(r"^\d+\.\d+$", adacc.version())


# ----------------------------------------------------------------- outlier channels
def test_channel_layout_closed_form_and_limits(L):
    assert ctypes.sizeof(adacc.CChannelMethod) == 28 and ctypes.sizeof(adacc.CChannelLayout) == 72
    m = adacc.ChannelMethod(bits=4, quant_group=128, asym=1, max_channels=10)
    tokens, hidden = 100, 2048
    n = tokens * hidden
    lay = adacc.channel_layout_of(m, tokens, hidden)
    a = lambda v: (v + 255) // 256 * 256
    assert lay.codes_off == 0 and lay.scales_off == a(n // 2)
    assert lay.zp_off == lay.scales_off + a(4 * n // 128)
    assert lay.ch_mask_off == lay.zp_off + a(4 * n // 128)
    assert lay.ch_base_off == lay.ch_mask_off + a(hidden // 8)
    assert lay.ch_idx_off == lay.ch_base_off + a(4 * hidden // 8)
    assert lay.ch_val_off == lay.ch_idx_off + a(40)
    assert lay.status_off == lay.ch_val_off + a(2 * tokens * 10)
    assert lay.total_bytes == lay.status_off + 256
    # chunk sums (one binary32 per chunk of 64 tokens and channel) + one binary64 per channel
    assert adacc.channel_workspace_bytes(tokens, hidden) == a(4 * 2 * hidden) + a(8 * hidden)
    for bad in (dict(hidden=2044), dict(hidden=0), dict(hidden=65544), dict(tokens=1 << 21),
                dict(m=adacc.ChannelMethod(bits=4, quant_group=4096)), dict(m=adacc.ChannelMethod(bits=5)),
                dict(m=adacc.ChannelMethod(max_channels=0)), dict(m=adacc.ChannelMethod(max_channels=4096)),
                dict(m=adacc.ChannelMethod(z_thresh=float("inf")))):
        args = dict(m=m, tokens=tokens, hidden=hidden)
        args.update(bad)
        with pytest.raises(adacc.AdaccError):
            adacc.channel_layout_of(args["m"], args["tokens"], args["hidden"])
    assert adacc.channel_workspace_bytes(100, 2044) == 0


def test_channel_calls_validate_before_any_device_work(L):
    m = adacc.ChannelMethod(bits=8, quant_group=64, max_channels=4)
    cm = m.c()
    tokens, hidden = 64, 256
    lay = adacc.channel_layout_of(m, tokens, hidden)
    wsb = adacc.channel_workspace_bytes(tokens, hidden)
    src, blob, ws = 0x10000, 0x20000, 0x30000
    f = L.adacc_channel_compress
    r = ctypes.byref(cm)
    assert f(None, src, tokens, hidden, blob, lay.total_bytes, ws, wsb, None) == adacc.ENULL
    assert f(r, None, tokens, hidden, blob, lay.total_bytes, ws, wsb, None) == adacc.ENULL
    assert f(r, src, tokens, hidden, None, lay.total_bytes, ws, wsb, None) == adacc.ENULL
    assert f(r, src, tokens, hidden, blob, lay.total_bytes, None, wsb, None) == adacc.ENULL
    assert f(r, src, tokens, hidden, blob, lay.total_bytes - 1, ws, wsb, None) == adacc.ESIZE
    assert f(r, src, tokens, hidden, blob, lay.total_bytes, ws, wsb - 1, None) == adacc.ESIZE
    assert f(r, src + 2, tokens, hidden, blob, lay.total_bytes, ws, wsb, None) == adacc.EALIGN
    assert f(r, src, tokens, hidden, blob, lay.total_bytes, ws + 16, wsb, None) == adacc.EALIGN
    assert f(r, src, tokens, 250, blob, lay.total_bytes, ws, wsb, None) == adacc.EINVAL
    assert f(r, None, 0, hidden, None, 0, None, 0, None) == adacc.OK
    g = L.adacc_channel_decompress
    assert g(r, blob, lay.total_bytes, tokens, hidden, None, 0, None) == adacc.ENULL
    assert g(r, blob, lay.total_bytes, tokens, hidden, 0x40000, 2, None) == adacc.EINVAL
    assert g(r, blob, lay.total_bytes - 1, tokens, hidden, 0x40000, 0, None) == adacc.ESIZE
    assert g(r, blob, lay.total_bytes, tokens, hidden, 0x40002, 0, None) == adacc.EALIGN


# ----------------------------------------------------------------- dropout mask
def test_mask_calls_validate_before_any_device_work(L):
    assert [L.adacc_mask_packed_bytes(n) for n in (0, 1, 8, 9, 4096)] == [0, 1, 1, 2, 512]
    for f in (L.adacc_mask_pack, L.adacc_mask_unpack):
        assert f(None, 0, None, None) == adacc.OK
        assert f(None, 64, 0x20000, None) == adacc.ENULL
        assert f(0x10000, 64, None, None) == adacc.ENULL
        assert f(0x10008, 64, 0x20000, None) == adacc.EALIGN
        assert f(0x10000, 64, 0x20004, None) == adacc.EALIGN


# ----------------------------------------------------------------- compression rate for the policy maker
def test_compressed_bytes_against_the_oracle_and_the_closed_form(L):
    """The oracle's logical size (pinned to the sizes the paper implies) plus the tile offsets the
    blob also stores; int4 in groups of 128 without outliers is 0.25 + 1/64 of the bf16 bytes."""
    import oracle
    from helpers import oracle_method
    import workloads
    for name in ("c1", "c2", "c3", "c4"):
        md = workloads.METHODS[name]
        n = 2048 * 12
        m = Method(bits=md["bits"], quant_group=md["quant_group"], asym=md["asym"],
                   outlier_mode={"none": 0, "abs": 1, "std": 2, "topk": 3}[md["outlier_mode"]],
                   stat_group=md["stat_group"], thresh=md["thresh"], topk=md["topk"], max_outliers=100)
        lay = adacc.layout_of(m, n)
        for n_out in (0, 7, 100):
            want = oracle.logical_bytes(oracle_method(md), n, n_out) + 4 * (lay.n_tiles + 1)
            assert adacc.compressed_bytes(m, n, n_out) == want
    plain = Method(bits=4, quant_group=128)
    n = 1 << 20
    assert adacc.compressed_bytes(plain, n, 0) == n // 2 + 4 * n // 128
    assert adacc.compressed_bytes(plain, n, 0) / (2 * n) == 0.25 + 1 / 64
    assert adacc.compressed_bytes(adacc.NOOP, n, 0) == 2 * n
    assert adacc.compressed_bytes(Method(bits=5), n, 0) == 0
    # outlier channels: the quantised tensor + per kept channel its index and one bf16 per token
    cm = adacc.ChannelMethod(bits=4, quant_group=128, max_channels=16)
    tokens, hidden = 96, 2048
    for n_ch in (0, 3, 16):
        assert adacc.channel_compressed_bytes(cm, tokens, hidden, n_ch) == \
            adacc.compressed_bytes(plain, tokens * hidden, 0) + n_ch * (2 * tokens + 4)
    asym = adacc.ChannelMethod(bits=8, quant_group=64, asym=1, max_channels=4)
    assert adacc.channel_compressed_bytes(asym, 10, 256, 2) == 2560 + 8 * 40 + 2 * 24
    assert adacc.channel_compressed_bytes(adacc.ChannelMethod(bits=5), tokens, hidden, 0) == 0


# ----------------------------------------------------------------- channel-wise symmetric quantisation
def test_channelwise_layout_and_validation(L):
    assert ctypes.sizeof(adacc.CChannelwiseLayout) == 24
    a = lambda v: (v + 255) // 256 * 256
    lay = adacc.channelwise_layout_of(4, 100, 2048)
    assert (lay.codes_off, lay.scales_off, lay.total_bytes) == (0, a(100 * 2048 // 2), a(100 * 2048 // 2) + a(4 * 2048))
    assert adacc.channelwise_workspace_bytes(100, 2048) == a(2 * 2 * 2048) + a(4 * 2048)
    for bits, tokens, hidden in ((5, 10, 64), (8, 10, 60), (8, 10, 0), (8, 1 << 27, 64), (8, 10, 65544)):
        with pytest.raises(adacc.AdaccError):
            adacc.channelwise_layout_of(bits, tokens, hidden)
    f = L.adacc_channelwise_compress
    src, blob, ws = 0x10000, 0x20000, 0x30000
    tb, wb = lay.total_bytes, adacc.channelwise_workspace_bytes(100, 2048)
    assert f(4, 0, 0, None, 100, 2048, blob, tb, ws, wb, None) == adacc.ENULL
    assert f(4, 0, 0, src, 100, 2048, blob, tb - 1, ws, wb, None) == adacc.ESIZE
    assert f(4, 0, 0, src, 100, 2048, blob, tb, ws, wb - 1, None) == adacc.ESIZE
    assert f(4, 0, 0, src + 8, 100, 2048, blob, tb, ws, wb, None) == adacc.EALIGN
    assert f(4, 2, 1, src, 100, 2048, blob, tb, ws, wb, None) == adacc.EINVAL
    assert f(4, 0, 0, None, 0, 2048, None, 0, None, 0, None) == adacc.OK
    assert f(4, 0, 2, src, 100, 2048, blob, tb, ws, wb, None) == adacc.EINVAL  # no such 16-bit format
    g = L.adacc_channelwise_decompress
    assert g(4, 2, blob, tb, 100, 2048, 0x40000, 0, None) == adacc.EINVAL
    assert g(4, 0, blob, tb, 100, 2048, None, 0, None) == adacc.ENULL
    assert g(4, 0, blob, tb, 100, 2048, 0x40000, 3, None) == adacc.EINVAL
    assert g(4, 0, blob, tb - 1, 100, 2048, 0x40000, 0, None) == adacc.ESIZE
    assert g(4, 0, blob, tb, 100, 2048, 0x40004, 0, None) == adacc.EALIGN


def test_noalloc_limit_is_checked_on_the_host(L):
    """adacc_compress_noalloc refuses what its 24 MiB device array cannot serve, before it looks at any
    pointer (all pointers are NULL here: whatever the outcome, nothing can be launched)."""
    f = L.adacc_compress_noalloc
    m_abs = Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_ABS, thresh=1.0, max_outliers=64)
    m_topk = Method(bits=4, quant_group=128, outlier_mode=adacc.OUTLIER_TOPK, stat_group=2048, topk=2, max_outliers=1 << 20)
    for m, numel, want in ((m_abs, adacc.NOALLOC_MAX_NUMEL, None), (m_abs, 2 * adacc.NOALLOC_MAX_NUMEL, adacc.ELIMIT),
                           (m_topk, 8 * adacc.NOALLOC_MAX_NUMEL, None)):
        assert (adacc.workspace_bytes(m, numel) > (24 << 20)) == (want == adacc.ELIMIT)
        cm = m.c()
        rc = f(ctypes.byref(cm), None, numel, None, 0, None)
        if want is not None:
            assert rc == want and "limit" in adacc.strerror(rc)
        else:
            assert rc in (adacc.ENULL, adacc.EHIP)  # past the limit check: stopped by the NULL pointers (or by the missing device)


def test_group_of_an_octet_by_reciprocal_is_exact():
    """The fallback kernels find the group of octet o as (uint32)(float(o) * r), r = RN(1 / octets per group) moved up
    three units in the last place.  Claimed exact for every o < 2048 and every group of 1 .. 2048 octets: all of them."""
    import numpy as np
    o = np.arange(2048, dtype=np.uint32)
    for opg in range(1, 2049):
        r = np.array([np.float32(1) / np.float32(opg)], dtype=np.float32)
        r = (r.view(np.uint32) + np.uint32(3)).view(np.float32)[0]
        assert np.array_equal((o.astype(np.float32) * r).astype(np.uint32), o // opg), opg
