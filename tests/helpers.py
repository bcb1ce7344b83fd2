"""Glue for the tests: the same method dictionary turned into the oracle's and the
library's descriptor, and the element-by-element comparison of a GPU blob with the oracle."""
import numpy as np
import torch

import oracle
import paper_2508_00806_amd as adacc

MODE_ID = {"none": 0, "abs": 1, "std": 2, "topk": 3}


def fmt_of(t):
    """0 (bf16) or 1 (binary16): the value both the oracle and the library use for the format of t."""
    assert t.dtype in (torch.bfloat16, torch.float16)
    return 1 if t.dtype == torch.float16 else 0


def oracle_method(md, rule=0, fmt=0):
    return oracle.method_from_dict(md, rule, fmt)


def adacc_method(md, cap, rule=0, fmt=0):
    return adacc.method_from_dict(md, cap, rule, fmt)


def bits_of(t):
    """bf16 / float16 torch tensor (any device) -> numpy uint16 bit patterns."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1)


def from_bits(b, device="cpu", dtype=torch.bfloat16):
    return torch.from_numpy(np.ascontiguousarray(b).view(np.int16).copy()).view(dtype).to(device)


def gpu_compress(x_dev, m, ws=None):
    """x_dev: bf16 tensor on the GPU.  Returns (blob, layout, workspace)."""
    numel = x_dev.numel()
    blob, L = adacc.alloc_blob(m, numel)
    if ws is None and m.outlier_mode != adacc.OUTLIER_NONE:
        ws = adacc.alloc_workspace(adacc.workspace_bytes(m, numel))
    adacc.compress(m, x_dev, blob, ws)
    return blob, L, ws


def compare_blob_with_oracle(blob, L, m, numel, oc, check_stream=True):
    """Bit-exact comparison of every used section of a GPU blob with the oracle's result."""
    sec = {k: v.cpu().numpy() for k, v in adacc.blob_sections(blob, L, m, numel).items()}
    assert np.array_equal(sec["codes"], oc.packed), "packed codes differ"
    assert np.array_equal(sec["scales"].view(np.uint32), oc.scale.view(np.uint32)), "scales differ"
    if m.asym:
        assert np.array_equal(sec["zp"].view(np.uint32), oc.zp.view(np.uint32)), "offsets differ"
    st = sec["status"].view(np.uint32)
    assert st[2] == 0, "status word 2 is not zero"
    if m.outlier_mode != adacc.OUTLIER_NONE:
        assert int(st[0]) == oc.n_out, f"outlier count {int(st[0])} != {oc.n_out}"
        assert int(st[1]) == (1 if oc.n_out > m.max_outliers else 0)
        k = min(oc.n_out, m.max_outliers)
        if check_stream:
            assert np.array_equal(sec["idx"][:k], oc.out_idx[:k]), "outlier indices differ"
            assert np.array_equal(sec["val"][:k].view(np.uint16), oc.out_val[:k]), "outlier values differ"
        # tile offsets = number of oracle outliers before each tile boundary
        full = oracle_full_indices(oc)
        bounds = np.arange(L.n_tiles + 1, dtype=np.int64) * L.tile_elems
        want = np.searchsorted(full, bounds, side="left")
        assert np.array_equal(sec["tile_ptr"].view(np.uint32).astype(np.int64), want), "tile offsets differ"
    else:
        assert int(st[0]) == 0 and int(st[1]) == 0
    return sec


def oracle_full_indices(oc):
    """All outlier indices of the oracle result, also past a truncated capacity."""
    if oc.n_out == oc.out_idx.size:
        return oc.out_idx.astype(np.int64)
    return oc._full_idx


def assert_f32_matches(got, want):
    """Within 1e-6 absolute of the oracle's binary32 result (the stated bar) and, stronger, the same
    bits.  Where the oracle itself yields Inf/NaN (a group whose range overflows binary32) only the
    class has to agree: NaN payloads are not part of the format."""
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.all(np.abs(got[fin].astype(np.float64) - want[fin].astype(np.float64)) <= 1e-6), \
        "binary32 reconstruction differs by more than 1e-6"
    ok = ~np.isnan(want)
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok]), "binary32 reconstruction not bit-equal"


def assert_bf16_matches(got_bits, want_bits, fmt=0):
    """16-bit reconstructions, bit for bit; for a NaN only the class has to agree."""
    inf = 0x7C00 if fmt == 1 else 0x7F80
    nan = (want_bits & 0x7FFF) > inf
    assert np.array_equal((got_bits & 0x7FFF) > inf, nan)
    assert np.array_equal(got_bits[~nan], want_bits[~nan]), "16-bit reconstruction differs"


def run_parity(x_cpu_bf16, md, cap=None, rule=0, decompress=True):
    """Compress on the GPU and in the oracle, compare everything, then decompress both ways."""
    x_bits = bits_of(x_cpu_bf16)
    numel = x_bits.size
    fmt = fmt_of(x_cpu_bf16)
    om = oracle_method(md, rule, fmt)
    oc_full = oracle.compress(om, x_bits)
    if cap is None:
        cap = max(oc_full.n_out, 1) if md["outlier_mode"] != "none" else 0
    oc = oracle.compress(om, x_bits, cap=cap)
    oc._full_idx = oc_full.out_idx.astype(np.int64)
    m = adacc_method(md, cap, rule, fmt)
    x_dev = x_cpu_bf16.contiguous().view(-1).cuda()
    blob, L, ws = gpu_compress(x_dev, m)
    torch.cuda.synchronize()
    st = adacc.read_status(blob, L)
    if md["outlier_mode"] != "none":
        assert st[0] == oc.n_out
    compare_blob_with_oracle(blob, L, m, numel, oc)
    if decompress and oc.n_out <= cap:
        of32, obf = oracle.decompress(oc)
        d32 = torch.empty(numel, dtype=torch.float32, device="cuda")
        dbf = torch.empty(numel, dtype=x_cpu_bf16.dtype, device="cuda")
        adacc.decompress(m, blob, d32)
        adacc.decompress(m, blob, dbf)
        torch.cuda.synchronize()
        assert_f32_matches(d32.cpu().numpy(), of32)
        assert_bf16_matches(bits_of(dbf), obf, fmt)
    return oc, blob, L, m


def run_channel_parity(x, bits, gq, asym, z=3.0, cap=None, rule=0):
    """x: bf16 or float16 [tokens, hidden] on the CPU."""
    tokens, hidden = x.shape
    xb = bits_of(x)
    fmt = fmt_of(x)
    om = oracle.Method(bits=bits, quant_group=gq, asym=asym, scale_rule=rule, dtype=fmt)
    S = oracle.channel_scores(xb, tokens, hidden, fmt)
    is_out, mu, sigma = oracle.channel_select(S, z)
    n_ch = int(is_out.sum())
    # The selection is an integer decided by sums.  The oracle's sums are exact; the library adds in
    # binary32 over 64 tokens at a time (relative error of S_h below 64 * 2^-24), so its Z differs by
    # up to about twice that times S / sigma.  The comparison of the channel sets below is complete
    # only if no channel of the input sits that close to the threshold: check it, and name any that do.
    fin = np.isfinite(S)
    if sigma > 0 and fin.any():
        zs = (S[fin] - mu) / sigma
        eps = 4 * 64 * 2.0 ** -24 * float(np.abs(S[fin]).max()) / sigma
        near = np.nonzero(np.abs(zs - z) <= eps)[0]
        assert near.size == 0, f"channels within {eps:.2e} of the Z threshold: {np.nonzero(fin)[0][near]}"
    cap = max(n_ch, 1) if cap is None else cap
    oc = oracle.channel_compress(om, xb, tokens, hidden, z, cap=cap)
    assert oc.n_ch == n_ch
    m = adacc.ChannelMethod(bits=bits, quant_group=gq, asym=asym, scale_rule=rule, z_thresh=z, max_channels=cap,
                            dtype=fmt)
    blob, L = adacc.alloc_channel_blob(m, tokens, hidden)
    blob.fill_(0xA5)
    ws = adacc.alloc_channel_workspace(tokens, hidden)
    adacc.channel_compress(m, x.contiguous().cuda(), tokens, hidden, blob, ws)
    st = adacc.channel_read_status(blob, L)
    assert st == (n_ch, 1 if n_ch > cap else 0, 0, 0), st
    sec = {k: v.cpu().numpy() for k, v in adacc.channel_blob_sections(blob, L, m, tokens, hidden).items()}
    assert np.array_equal(np.unpackbits(sec["ch_mask"], bitorder="little"), is_out), "channel mask differs"
    per_byte = is_out.reshape(-1, 8).sum(axis=1)
    assert np.array_equal(sec["ch_base"], np.concatenate([[0], np.cumsum(per_byte)[:-1]])), "channel ranks differ"
    k = min(n_ch, cap)
    assert np.array_equal(sec["ch_idx"][:k], np.nonzero(is_out)[0][:k]), "channel list differs"
    dbf = torch.full((tokens * hidden,), 7.0, dtype=x.dtype, device="cuda")
    d32 = torch.full((tokens * hidden,), 7.0, dtype=torch.float32, device="cuda")
    adacc.channel_decompress(m, blob, tokens, hidden, dbf)
    adacc.channel_decompress(m, blob, tokens, hidden, d32)
    torch.cuda.synchronize()
    if n_ch > cap:  # not a usable blob: nothing else is produced, decompression leaves dst alone
        assert bool((dbf == 7.0).all()) and bool((d32 == 7.0).all())
        return oc, st
    assert np.array_equal(sec["ch_val"].view(np.uint16)[:tokens * n_ch].reshape(tokens, n_ch), oc.ch_val), \
        "channel values differ"
    assert np.array_equal(sec["codes"], oc.packed), "packed codes differ"
    assert np.array_equal(sec["scales"].view(np.uint32), oc.scale.view(np.uint32)), "scales differ"
    if asym:
        assert np.array_equal(sec["zp"].view(np.uint32), oc.zp.view(np.uint32)), "offsets differ"
    of32, obf = oracle.channel_decompress(oc)
    assert_f32_matches(d32.cpu().numpy(), of32)
    assert_bf16_matches(bits_of(dbf), obf, fmt)
    return oc, st
