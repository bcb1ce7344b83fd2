"""The C oracle against tests/bruteforce.py, field by field, on tiny tensors, for every outlier mode x
bit width x symmetric / asymmetric x scale rule (Section 3.2, Eq. 2, Eq. 3, Fig. 3(c)).  The brute
force is exact rational arithmetic with explicit binary32 rounding, one element at a time; a mistake
in the oracle's composition (scale taken before the outliers are zeroed, a code other than that of
zero at an outlier, the wrong nibble for the tail of an odd-length tensor, a dropped offset on the
way back) fails here."""
from fractions import Fraction

import numpy as np
import pytest

import bruteforce as bf
import oracle
from oracle import Method

MODES = {"none": bf.NONE, "abs": bf.ABS, "std": bf.STD, "topk": bf.TOPK}


def to_bf16_bits(a):
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def tensors(seed, n):
    """A few tiny inputs: heavy-tailed values, small integers (ties everywhere), one-sided values,
    zeros of both signs and subnormals."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n) * np.where(rng.random(n) < 0.1, 30.0, 1.0)
    b = rng.integers(-9, 10, size=n).astype(np.float64) * 0.5
    c = np.abs(rng.standard_normal(n)) + 0.125
    d = to_bf16_bits(rng.standard_normal(n) * 1e-3)
    d[::5] = 0x8000
    d[1::7] = 0x0000
    d[2::9] = rng.integers(1, 0x80, size=d[2::9].size)  # subnormal bf16
    return [to_bf16_bits(a), to_bf16_bits(b), to_bf16_bits(c), d]


def check(bits, nbits, gq, asym, rule, mode, gs=0, thresh=0.0, topk=0, fmt=bf.BF16):
    n = bits.size
    m = Method(bits=nbits, quant_group=gq, asym=asym, scale_rule=rule, outlier_mode=MODES[mode], stat_group=gs,
               thresh=thresh, topk=topk, dtype=fmt)
    oc = oracle.compress(m, bits)
    t32 = Fraction(float(np.float32(thresh)))
    want = bf.compress([int(b) for b in bits], nbits=nbits, quant_group=gq, asym=asym, rule=rule, mode=MODES[mode],
                       stat_group=gs, thresh=t32, topk=topk, fmt=fmt)
    assert list(oc.out_idx) == want["out_idx"], "outlier indices"
    assert [int(v) for v in oc.out_val] == want["out_val"], "outlier values"
    assert oc.n_out == len(want["out_idx"])
    assert [int(c) for c in oc.codes] == want["codes"], "codes"
    assert [int(p) for p in oc.packed] == want["packed"], "packed codes"
    assert [Fraction(float(s)) for s in oc.scale] == want["scale"], "scales"
    if asym:
        assert [Fraction(float(z)) for z in oc.zp] == want["zp"], "offsets"
    f, b = oracle.decompress(oc)
    xs, bs = bf.decompress(want, n=n, nbits=nbits, quant_group=gq, asym=asym, fmt=fmt)
    for i in range(n):
        if xs[i] is None:  # a non-finite outlier: the stored pattern comes back
            assert int(b[i]) == bs[i] and not np.isfinite(f[i])
        else:
            assert Fraction(float(f[i])) == xs[i], f"binary32 reconstruction of element {i}"
            assert int(b[i]) == bs[i], f"16-bit reconstruction of element {i}"
    return oc


@pytest.mark.parametrize("mode", ["none", "abs", "std", "topk"])
@pytest.mark.parametrize("nbits", [4, 8])
@pytest.mark.parametrize("asym", [0, 1])
@pytest.mark.parametrize("rule", [bf.PAPER, bf.FULLRANGE])
def test_whole_chain_on_tiny_tensors(mode, nbits, asym, rule):
    n_out = 0
    for k, bits in enumerate(tensors(7 + nbits + asym, 32)):
        kw = dict(abs=dict(thresh=1.75), std=dict(gs=16, thresh=1.5), topk=dict(gs=16, topk=3), none={})[mode]
        oc = check(bits, nbits, 8, asym, rule, mode, **kw)  # 4 groups of 8
        n_out += oc.n_out
    assert (n_out > 0) == (mode != "none")


@pytest.mark.parametrize("nbits", [4, 8])
@pytest.mark.parametrize("asym", [0, 1])
def test_groups_that_are_no_power_of_two_and_an_odd_tail(nbits, asym):
    """15 elements in groups of 5, statistics over all 15: the last byte of the int4 codes holds one
    element; the pairwise sum is padded with a zero."""
    for bits in tensors(21, 15):
        check(bits, nbits, 5, asym, bf.PAPER, "std", gs=15, thresh=1.25)
        check(bits, nbits, 5, asym, bf.FULLRANGE, "topk", gs=15, topk=2)
        check(bits, nbits, 3, asym, bf.PAPER, "abs", thresh=0.5)


@pytest.mark.parametrize("mode", ["abs", "std", "topk"])
def test_values_that_are_not_finite(mode):
    bits = tensors(33, 32)[0]
    bits[3], bits[4], bits[20] = 0x7F80, 0xFFC1, 0xFF80  # +Inf, a NaN, -Inf
    kw = dict(abs=dict(thresh=2.0), std=dict(gs=16, thresh=1.5), topk=dict(gs=16, topk=1))[mode]
    for asym in (0, 1):
        oc = check(bits, 4, 8, asym, bf.PAPER, mode, **kw)
        assert {3, 4, 20} <= set(int(i) for i in oc.out_idx)
    # more values that are not finite than the group's k: all of them are kept, and nothing else
    bits[5], bits[6] = 0x7F80, 0x7FFF
    oc = check(bits, 8, 8, 0, bf.PAPER, "topk", gs=16, topk=2)
    assert [int(i) for i in oc.out_idx if i < 16] == [3, 4, 5, 6]


def test_rounding_helpers_of_the_brute_force_against_numpy():
    """The brute force's own binary32 / bf16 rounding, checked against the hardware's."""
    rng = np.random.default_rng(5)
    for _ in range(2000):
        a, b = (float(np.float32(v)) for v in rng.standard_normal(2) * 10.0 ** rng.integers(-15, 15))
        assert bf.f32(Fraction(a) * Fraction(b)) == Fraction(float(np.float32(a) * np.float32(b)))
        assert bf.f32(Fraction(a) + Fraction(b)) == Fraction(float(np.float32(a) + np.float32(b)))
        assert bf.f32(Fraction(a) / Fraction(b)) == Fraction(float(np.float32(a) / np.float32(b)))
    import torch
    pats = np.arange(0x10000, dtype=np.uint32)
    pats = pats[(pats & 0x7F80) != 0x7F80].astype(np.uint16)
    vals = torch.from_numpy(pats.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    for p, v in zip(pats[::37], vals[::37]):
        assert bf.bf16_value(int(p)) == Fraction(float(v))
    x = torch.from_numpy((rng.standard_normal(3000) * 10.0 ** rng.integers(-38, 38, size=3000)).astype(np.float32))
    want = x.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for v, w in zip(x.numpy(), want):
        if np.isfinite(v) and (int(w) & 0x7F80) != 0x7F80:
            assert bf.bf16_bits_of(Fraction(float(v))) == int(w)


# ------------------------------------------------------------------ binary16 tensors (the paper's own format)
def to_f16_bits(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16).view(np.uint16)


def f16_tensors(seed, n):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n) * np.where(rng.random(n) < 0.1, 30.0, 1.0)
    b = rng.integers(-9, 10, size=n).astype(np.float64) * 0.5
    c = np.abs(rng.standard_normal(n)) * 300.0 + 0.125        # large: the reconstruction nears the end of the range
    d = to_f16_bits(rng.standard_normal(n) * 1e-4)
    d[::5] = 0x8000
    d[1::7] = 0x0000
    d[2::9] = rng.integers(1, 0x400, size=d[2::9].size)       # subnormal binary16
    return [to_f16_bits(a), to_f16_bits(b), to_f16_bits(c), d]


@pytest.mark.parametrize("mode", ["none", "abs", "std", "topk"])
@pytest.mark.parametrize("nbits", [4, 8])
@pytest.mark.parametrize("asym", [0, 1])
def test_whole_chain_on_tiny_binary16_tensors(mode, nbits, asym):
    n_out = 0
    for rule in (bf.PAPER, bf.FULLRANGE):
        for bits in f16_tensors(70 + nbits + asym, 32):
            kw = dict(abs=dict(thresh=1.75), std=dict(gs=16, thresh=1.5), topk=dict(gs=16, topk=3), none={})[mode]
            n_out += check(bits, nbits, 8, asym, rule, mode, fmt=bf.F16, **kw).n_out
    assert (n_out > 0) == (mode != "none")


def test_binary16_values_that_are_not_finite_and_the_largest_finite_ones():
    bits = f16_tensors(3, 32)[0]
    bits[3], bits[4], bits[20] = 0x7C00, 0xFE01, 0xFC00   # +Inf, a NaN, -Inf
    bits[8], bits[9] = 0x7BFF, 0xFBFF                       # +-65504
    for asym in (0, 1):
        oc = check(bits, 4, 8, asym, bf.PAPER, "topk", gs=16, topk=1, fmt=bf.F16)
        assert {3, 4, 20} <= set(int(i) for i in oc.out_idx)
        check(bits, 8, 8, asym, bf.FULLRANGE, "abs", thresh=70000.0, fmt=bf.F16)  # only what is not finite is kept


# ------------------------------------------------------------------ a last group that is short
@pytest.mark.parametrize("fmt", [bf.BF16, bf.F16])
@pytest.mark.parametrize("nbits", [4, 8])
@pytest.mark.parametrize("asym", [0, 1])
def test_short_last_groups(fmt, nbits, asym):
    """The group length divides the tensor's length in neither case; 27 and 29 elements in quantisation
    groups of 8 and statistics groups of 16: the last quantisation group has 3 (5) elements, the last
    statistics group 11 (13), and with int4 the last byte holds one element."""
    for n in (27, 29):
        src = f16_tensors(90 + n, n) if fmt == bf.F16 else tensors(90 + n, n)
        for bits in src:
            check(bits, nbits, 8, asym, bf.PAPER, "none", fmt=fmt)
            check(bits, nbits, 8, asym, bf.FULLRANGE, "abs", thresh=1.0, fmt=fmt)
            check(bits, nbits, 8, asym, bf.PAPER, "std", gs=16, thresh=1.25, fmt=fmt)
            check(bits, nbits, 8, asym, bf.PAPER, "topk", gs=16, topk=3, fmt=fmt)
    # a last statistics group with fewer elements than k: all of it is kept, and no more
    bits = (f16_tensors(5, 18) if fmt == bf.F16 else tensors(5, 18))[0]
    oc = check(bits, nbits, 8, asym, bf.PAPER, "topk", gs=16, topk=3, fmt=fmt)
    assert [int(i) for i in oc.out_idx if i >= 16] == [16, 17] and oc.n_out == 5


def test_a_short_last_group_is_a_group_of_its_own():
    """Groups do not see each other: the result for a tensor with a short last group is the result for
    the whole groups followed by the result for the rest taken as a tensor of its own."""
    rng = np.random.default_rng(12)
    x = to_bf16_bits(rng.standard_normal(1000) * np.where(rng.random(1000) < 0.05, 25.0, 1.0))
    for m in (Method(bits=4, quant_group=64, outlier_mode=2, stat_group=128, thresh=2.0),
              Method(bits=8, quant_group=128, asym=1, outlier_mode=3, stat_group=128, topk=2)):
        whole = oracle.compress(m, x)
        head, tail = oracle.compress(m, x[:896]), oracle.compress(m, x[896:])   # 896 = 7 * 128
        assert np.array_equal(whole.codes, np.concatenate([head.codes, tail.codes]))
        assert np.array_equal(whole.scale.view(np.uint32), np.concatenate([head.scale, tail.scale]).view(np.uint32))
        assert list(whole.out_idx) == list(head.out_idx) + [int(i) + 896 for i in tail.out_idx]
        assert tail.scale.size == -(-104 // m.quant_group)  # 104 elements: 64 + 40, or one group of 104


def test_rounding_helpers_of_the_brute_force_for_binary16_against_numpy():
    pats = np.arange(0x10000, dtype=np.uint32)
    pats = pats[(pats & 0x7C00) != 0x7C00].astype(np.uint16)
    vals = pats.view(np.float16).astype(np.float64)
    for p, v in zip(pats[::29], vals[::29]):
        assert bf.f16_value(int(p)) == Fraction(float(v))
    rng = np.random.default_rng(6)
    x = (rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 6, size=4000)).astype(np.float32)
    x = np.concatenate([x, np.float32([65504, 65519.99, 65520, -65520, 1e9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25])])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    for v, w in zip(x, want):
        assert bf.f16_bits_of(Fraction(float(v))) == int(w), float(v)


# ------------------------------------------------------------------ one element through every kind of bit pattern
@pytest.mark.parametrize("fmt", [bf.BF16, bf.F16])
def test_one_element_swept_over_the_16_bit_patterns(fmt):
    """One group of eight; seven elements fixed, the eighth takes every 13th of the 65 536 bit patterns
    (13 is odd, so both signs, every exponent, subnormals, zeros, infinities and NaNs are visited) under
    ABS outliers with symmetric int8 and asymmetric int4 codes.  Whatever the pattern, the oracle and
    the exact-arithmetic brute force agree field by field."""
    base = to_bf16_bits([0.5, -0.75, 0.0, 1.25, -0.125, 0.3125, 1.0, 0.0]) if fmt == bf.BF16 else \
        to_f16_bits([0.5, -0.75, 0.0, 1.25, -0.125, 0.3125, 1.0, 0.0])
    kept = 0
    for pattern in range(0, 0x10000, 13):
        bits = base.copy()
        bits[7] = pattern
        oc = check(bits, 8, 8, 0, bf.FULLRANGE, "abs", thresh=3.0, fmt=fmt)
        kept += oc.n_out
        if pattern % 3 == 0:
            check(bits, 4, 8, 1, bf.PAPER, "abs", thresh=3.0, fmt=fmt)
    assert 0 < kept < 0x10000 // 13
