"""Pins for the CPU oracle: every check here compares the oracle with something
that is NOT the oracle - values worked by hand from Eq. 2 / Eq. 3 for the vectors
the paper prints, exact rational arithmetic, sorting, a library routine, or an
invariant of the method.  No GPU needed."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import Method, OUT_NONE, OUT_ABS, OUT_STD, OUT_TOPK, RULE_PAPER, RULE_FULLRANGE

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers
def bf16_bits(a):
    """float array -> bf16 bit patterns through torch's own conversion (a library routine)."""
    t = torch.as_tensor(np.asarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_f32(b):
    t = torch.from_numpy(np.asarray(b, dtype=np.uint16).view(np.int16).copy()).view(torch.bfloat16)
    return t.to(torch.float32).numpy()


def frac(x):
    return Fraction(float(x))  # exact: every binary32 is a binary64


def read_golden(name):
    rows = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        rows[k] = v
    return rows


def rng_bits(seed, n, scale=1.0, heavy=False):
    g = np.random.default_rng(seed)
    x = g.standard_normal(n).astype(np.float32) * scale
    if heavy:
        k = max(1, n // 50)
        x[g.choice(n, k, replace=False)] *= 40.0
    return bf16_bits(x)


# ----------------------------------------------------------------- the paper's own vectors
def test_eq2_toy_vector_from_paper():
    g = read_golden("eq2_symmetric_toy.txt")
    x = bf16_bits([float(v) for v in g["input"]])
    c = oracle.compress(Method(bits=4, quant_group=len(x)), x)
    assert c.scale.tolist() == [float(g["scale"][0])]
    assert c.codes.tolist() == [int(v) for v in g["codes"]]
    f, b = oracle.decompress(c)
    assert f.tolist() == [float(v) for v in g["dequant"]]
    assert bits_to_f32(b).tolist() == [float(v) for v in g["dequant"]]
    assert c.n_out == 0


def test_eq3_toy_vector_from_paper():
    g = read_golden("eq3_asymmetric_toy.txt")
    x = bf16_bits([float(v) for v in g["input"]])
    c = oracle.compress(Method(bits=4, quant_group=len(x), asym=1), x)
    assert c.zp.tolist() == [float(g["offset"][0])]
    assert c.scale.tolist() == [float(g["scale"][0])]
    assert c.codes.tolist() == [int(v) for v in g["codes"]]
    f, _ = oracle.decompress(c)
    assert f.tolist() == [float(v) for v in g["dequant"]]


def test_table1_size_ratios():
    """Closed-form size against Table 1: no-outlier int4 is a quarter of the fp16 bytes;
    T2's extra 1.3 MB is its uncompressed outlier share."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_sizes.txt"))
            if l.strip() and not l.startswith("#")]
    m = Method(bits=4, quant_group=4096)  # "scaling factor for each row": per-row scales are invisible at 0.1 MB
    for name, size, comp in rows:
        size, comp = float(size), float(comp)
        n = int(size * 1e6 / 2) // 4096 * 4096
        no_out = oracle.logical_bytes(m, n, 0) / 1e6
        if name in ("T1", "T4"):
            assert abs(no_out - comp) < 0.06, (name, no_out, comp)
        else:
            # outliers stored as fp16 value + index (6 B each here): 1.3 MB of them
            n_out = round((comp - no_out) * 1e6 / 6)
            assert n_out > 0
            assert abs(oracle.logical_bytes(m, n, n_out) / 1e6 - comp) < 0.06


def test_logical_bytes_closed_form():
    for bits in (4, 8):
        for asym in (0, 1):
            for gq in (64, 128, 1024):
                m = Method(bits=bits, quant_group=gq, asym=asym)
                n = gq * 37
                for n_out in (0, 5, 1000):
                    want = n * bits // 8 + 4 * (n // gq) * (1 + asym) + 6 * n_out
                    assert oracle.logical_bytes(m, n, n_out) == want


# ----------------------------------------------------------------- conversions vs a library
def test_widen_and_round_match_torch():
    allbits = np.arange(65536, dtype=np.uint16)
    m = Method(bits=8, quant_group=65536, outlier_mode=OUT_ABS, thresh=0.0)
    # tau = 0: every non-zero element is an outlier, so decompress returns the widened input
    c = oracle.compress(m, allbits)
    f, b = oracle.decompress(c)
    want = bits_to_f32(allbits)
    nz = (allbits & 0x7FFF) != 0
    assert np.array_equal(f.view(np.uint32)[nz], want.view(np.uint32)[nz])
    assert np.array_equal(b[nz], allbits[nz])
    # binary32 -> bf16 rounding of dequantised values vs torch
    x = rng_bits(3, 4096, 3.0)
    c = oracle.compress(Method(bits=8, quant_group=64, scale_rule=RULE_FULLRANGE), x)
    f, b = oracle.decompress(c)
    assert np.array_equal(b, bf16_bits(f))
    c = oracle.compress(Method(bits=4, quant_group=64, asym=1), x)
    f, b = oracle.decompress(c)
    assert np.array_equal(b, bf16_bits(f))


def test_binary16_widen_and_round_match_torch():
    """The paper compresses FP16 activations (Section 3.2, "compressed from FP16 to INT4").  The oracle's
    binary16 -> binary32 widening on every one of the 65 536 patterns, and its binary32 -> binary16
    rounding on random values, on every tie between two neighbouring binary16 values and the binary32
    values next to it, and at the end of the range, against torch."""
    allbits = np.arange(65536, dtype=np.uint16)
    got = oracle.to_f32(allbits, oracle.DT_F16)
    want = torch.from_numpy(allbits.view(np.int16).copy()).view(torch.float16).to(torch.float32).numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan) and nan.sum() == 2 * 1023
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])
    # rounding: ties and their neighbours
    fin = allbits[(allbits & 0x7C00) != 0x7C00]
    pos = np.sort(fin[fin < 0x8000])                      # 0 .. 65504 in ascending order
    v = want[pos].astype(np.float64)
    mid = ((v[:-1] + v[1:]) / 2).astype(np.float32)       # exact in binary32: 12 significant bits
    assert np.array_equal(mid.astype(np.float64), (v[:-1] + v[1:]) / 2)
    cases = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf)),
                            np.float32([0.0, -0.0, 65504, 65519.996, 65520, 65536, 1e30, np.inf, 2.0 ** -24,
                                        2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 1e-30])])
    g = np.random.default_rng(17)
    rnd = (g.standard_normal(20000) * 10.0 ** g.integers(-10, 6, 20000)).astype(np.float32)
    cases = np.concatenate([cases, -cases, rnd])
    got = oracle.from_f32(cases, oracle.DT_F16)
    want16 = torch.from_numpy(cases).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want16)
    assert oracle.from_f32(np.float32([np.nan]), oracle.DT_F16)[0] & 0x7FFF > 0x7C00
    # and through the whole chain: with tau = 0 every non-zero element is kept and comes back bit for bit
    m = Method(bits=8, quant_group=65536, outlier_mode=OUT_ABS, thresh=0.0, dtype=oracle.DT_F16)
    f, b = oracle.decompress(oracle.compress(m, allbits))
    nz = (allbits & 0x7FFF) != 0
    assert np.array_equal(b[nz], allbits[nz])


def test_binary16_channel_scores_are_the_exactly_rounded_sums():
    import math
    g = np.random.default_rng(23)
    tokens, hidden = 300, 24
    x = (g.standard_normal((tokens, hidden)) * 10.0 ** g.integers(-7, 4, (tokens, hidden))).astype(np.float16)
    S = oracle.channel_scores(x.view(np.uint16), tokens, hidden, oracle.DT_F16)
    for h in range(hidden):
        assert S[h] == math.fsum(abs(float(v)) for v in x[:, h])


# ----------------------------------------------------------------- pairwise sum
def test_pairwise_sum_order_is_a_binary_tree():
    # hand-worked in binary32: (1e8+1)=1e8, (-1e8+1)=-1e8, sum 0.  Left-to-right would give 1.
    assert float(oracle.pairwise_sum([1e8, 1.0, -1e8, 1.0])) == 0.0
    # (1+1e8)=1e8; (1 + -1e8) = -1e8 (ulp is 8) -> 0; left-to-right gives 1+... = 0 too, so use another:
    # (3+1e8)=100000000 (ulp 8, 3 rounds down), (5-1e8) = -99999992 (5 -> 8) -> sum 8
    assert float(oracle.pairwise_sum([3.0, 1e8, 5.0, -1e8])) == 8.0
    # n = 3 pads with +0 on the right: (a+b)+(c+0)
    a, b, c = np.float32(1e8), np.float32(3.0), np.float32(5.0)
    assert float(oracle.pairwise_sum([a, b, c])) == float(np.float32(np.float32(a + b) + c))
    # n = 5: ((a+b)+(c+d)) + ((e+0)+(0+0))
    v = np.array([1e8, 3.0, -1e8, 3.0, 1.0], dtype=np.float32)
    want = np.float32(np.float32(np.float32(v[0] + v[1]) + np.float32(v[2] + v[3])) + v[4])
    assert float(oracle.pairwise_sum(v)) == float(want)


def test_pairwise_sum_exact_on_integers_and_close_to_fsum():
    g = np.random.default_rng(0)
    for n in (1, 2, 7, 64, 1000, 4096):
        v = g.integers(-100, 100, n).astype(np.float32)
        assert float(oracle.pairwise_sum(v)) == float(v.astype(np.int64).sum())
        w = g.standard_normal(n).astype(np.float32)
        exact = math.fsum(float(t) for t in w)
        bound = (math.ceil(math.log2(max(n, 2))) + 1) * 2.0 ** -24 * float(np.abs(w).sum())
        assert abs(float(oracle.pairwise_sum(w)) - exact) <= bound


# ----------------------------------------------------------------- outlier sets
def test_abs_outliers_are_exactly_the_elements_past_tau():
    x = rng_bits(11, 4096, 1.0, heavy=True)
    xf = bits_to_f32(x).astype(np.float64)
    for tau in (0.0, 0.5, 3.0, 6.0, 1e9):
        out = oracle.select_outliers(Method(quant_group=64, outlier_mode=OUT_ABS, thresh=tau), x)
        want = np.abs(xf) > float(np.float32(tau))
        assert np.array_equal(out.astype(bool), want)


def test_topk_outliers_match_a_sort():
    g = np.random.default_rng(5)
    for gs, k in ((16, 1), (64, 3), (128, 1), (2048, 2), (4096, 4)):
        x = rng_bits(int(gs + k), gs * 6, 1.0, heavy=True)
        # plant ties: repeat one magnitude with both signs
        x[3] = 0x4120
        x[gs - 1] = 0xC120
        x[gs // 2] = 0x4120
        out = oracle.select_outliers(Method(quant_group=16, outlier_mode=OUT_TOPK, stat_group=gs, topk=k), x)
        for grp in range(6):
            seg = x[grp * gs:(grp + 1) * gs]
            order = sorted(range(gs), key=lambda i: (-(int(seg[i]) & 0x7FFF), i))
            want = np.zeros(gs, dtype=bool)
            want[order[:k]] = True
            got = out[grp * gs:(grp + 1) * gs].astype(bool)
            assert np.array_equal(got, want), (gs, k, grp)
            assert got.sum() == k
            # every kept magnitude >= every dropped magnitude
            mag = seg & 0x7FFF
            assert mag[got].min() >= mag[~got].max()


def test_topk_tie_goes_to_the_earlier_element():
    x = bf16_bits([1.0, -5.0, 5.0, 2.0, 5.0, -5.0, 0.0, 1.0])
    out = oracle.select_outliers(Method(quant_group=8, outlier_mode=OUT_TOPK, stat_group=8, topk=2), x)
    assert out.tolist() == [0, 1, 1, 0, 0, 0, 0, 0]


def test_std_outliers_exact_rational_on_integer_groups():
    """Small-integer inputs: every binary32 sum is exact, so the rule can be checked
    in exact rational arithmetic: x^2 > k^2 * (mean(x^2) - mean(x)^2)."""
    g = np.random.default_rng(9)
    for gs in (8, 64, 256, 1024):
        for k in (1.0, 2.0, 3.0, 1.5):
            v = g.integers(-8, 9, gs * 4).astype(np.float32)
            v[g.integers(0, v.size, 6)] = 96.0
            v[g.integers(0, v.size, 3)] = -120.0
            x = bf16_bits(v)
            out = oracle.select_outliers(Method(quant_group=8, outlier_mode=OUT_STD, stat_group=gs, thresh=k), x)
            for grp in range(4):
                seg = [Fraction(int(t)) for t in v[grp * gs:(grp + 1) * gs]]
                mean = sum(seg) / gs
                var = sum(t * t for t in seg) / gs - mean * mean
                # mean is a dyadic rational with few bits here, so binary32 holds it exactly
                want = [t * t > Fraction(k) ** 2 * var for t in seg]
                assert out[grp * gs:(grp + 1) * gs].astype(bool).tolist() == want, (gs, k, grp)


def test_std_rule_is_strict_and_uses_the_squared_multiple():
    # [a,-a,a,-a]: mean 0, var = a^2.  k = 1: x^2 == k^2 var for every element -> none is past it.
    x = bf16_bits([3.0, -3.0, 3.0, -3.0, 1.0, -1.0, 1.0, -1.0])
    out = oracle.select_outliers(Method(quant_group=4, outlier_mode=OUT_STD, stat_group=4, thresh=1.0), x)
    assert out.tolist() == [0] * 8
    # [0,0,0,4]: mean 1, var = 4 - 1 = 3; 16 > k^2 * 3 for k = 2 (12) but not for k = 2.5 (18.75)
    y = bf16_bits([0.0, 0.0, 0.0, 4.0])
    for k, want in ((2.0, [0, 0, 0, 1]), (2.5, [0, 0, 0, 0])):
        out = oracle.select_outliers(Method(quant_group=4, outlier_mode=OUT_STD, stat_group=4, thresh=k), y)
        assert out.tolist() == want


def test_std_outliers_agree_with_float64_away_from_the_threshold():
    for seed, gs, k in ((1, 1024, 6.0), (2, 64, 2.0), (3, 2048, 4.0), (4, 128, 3.0)):
        x = rng_bits(seed, gs * 32, 1.0, heavy=True)
        xf = bits_to_f32(x).astype(np.float64).reshape(-1, gs)
        var = (xf * xf).mean(axis=1) - xf.mean(axis=1) ** 2
        lim = (k * k) * var[:, None]
        want = (xf * xf) > lim
        near = np.abs(xf * xf - lim) <= 1e-4 * lim
        out = oracle.select_outliers(Method(quant_group=8, outlier_mode=OUT_STD, stat_group=gs, thresh=k), x)
        out = out.reshape(-1, gs).astype(bool)
        assert np.array_equal(out[~near], want[~near])
        assert want.sum() > 0


def test_nonfinite_is_always_an_outlier_and_never_scales():
    x = rng_bits(21, 256)
    x[5] = 0x7F80   # +inf
    x[70] = 0xFF80  # -inf
    x[130] = 0x7FC1  # NaN
    for mode, kw in ((OUT_ABS, dict(thresh=100.0)), (OUT_STD, dict(stat_group=64, thresh=6.0)),
                     (OUT_TOPK, dict(stat_group=64, topk=1))):
        c = oracle.compress(Method(bits=8, quant_group=64, outlier_mode=mode, **kw), x)
        got = set(c.out_idx.tolist())
        assert {5, 70, 130} <= got
        assert np.all(np.isfinite(c.scale))
        _, b = oracle.decompress(c)
        assert b[5] == 0x7F80 and b[70] == 0xFF80 and b[130] == 0x7FC1


# ----------------------------------------------------------------- quantiser
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("rule", [RULE_PAPER, RULE_FULLRANGE])
def test_sym_codes_are_nearest_in_exact_arithmetic(bits, rule):
    q = 1 << (bits - 1)
    d = q if rule == RULE_PAPER else q - 1
    gq = 64
    x = rng_bits(100 + bits + rule, gq * 64, 2.0)
    c = oracle.compress(Method(bits=bits, quant_group=gq, scale_rule=rule), x)
    xf = bits_to_f32(x)
    exact_match = 0
    for h in range(x.size // gq):
        seg = xf[h * gq:(h + 1) * gq]
        a = max(abs(frac(t)) for t in seg)
        # scale: a / d, correctly rounded to binary32
        assert frac(c.scale[h]) == frac(np.float32(float(a) / d)) or rule == RULE_PAPER and frac(c.scale[h]) * d == a
        for i, t in enumerate(seg):
            code = int(c.codes[h * gq + i])
            assert -q <= code <= q - 1
            r = frac(t) * d / a  # X / S in exact arithmetic
            target = min(max(r, -q), q - 1)
            # nearest, up to the one-rounding slack of evaluating X * (D / max)
            assert abs(target - code) <= Fraction(1, 2) + abs(r) * Fraction(1, 2 ** 22)
            nearest = math.floor(target + Fraction(1, 2))
            if target + Fraction(1, 2) == nearest and nearest % 2 == 1:
                nearest -= 1  # half goes to even
            if nearest == code:
                exact_match += 1
            else:
                # only an exact or near tie may go to the other neighbour (bf16 inputs make exact
                # ties common, and D / max carries one rounding when D is not a power of two)
                assert abs(abs(target - math.floor(target)) - Fraction(1, 2)) <= abs(r) * Fraction(1, 2 ** 22)
    assert exact_match >= 0.999 * x.size


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("rule", [RULE_PAPER, RULE_FULLRANGE])
def test_asym_codes_are_nearest_in_exact_arithmetic(bits, rule):
    q = 1 << (bits - 1)
    d2 = 2 * q if rule == RULE_PAPER else 2 * q - 1
    gq = 32
    x = bf16_bits(np.abs(bits_to_f32(rng_bits(200 + bits + rule, gq * 64, 2.0))) + 0.25)  # one-sided data
    c = oracle.compress(Method(bits=bits, quant_group=gq, asym=1, scale_rule=rule), x)
    xf = bits_to_f32(x)
    for h in range(x.size // gq):
        seg = xf[h * gq:(h + 1) * gq]
        hi, lo = max(frac(t) for t in seg), min(frac(t) for t in seg)
        assert frac(c.zp[h]) == frac(np.float32(np.float32(float(hi) + float(lo)) * np.float32(0.5)))
        r32 = np.float32(np.float32(float(hi)) - np.float32(float(lo)))
        assert frac(c.scale[h]) == frac(np.float32(r32 / np.float32(d2)))
        o, rng_ = frac(c.zp[h]), frac(r32)
        for i, t in enumerate(seg):
            code = int(c.codes[h * gq + i])
            assert -q <= code <= q - 1
            # binary32 subtraction first (as Eq. 3 writes X - O), then exact division by S
            diff = frac(np.float32(np.float32(t) - c.zp[h]))
            r = diff * d2 / rng_
            target = min(max(r, -q), q - 1)
            assert abs(target - code) <= Fraction(1, 2) + abs(r) * Fraction(1, 2 ** 22)


def test_paper_rule_scale_times_divisor_is_absmax_exactly():
    x = rng_bits(7, 128 * 40, 5.0)
    xf = bits_to_f32(x).reshape(-1, 128)
    for bits in (4, 8):
        c = oracle.compress(Method(bits=bits, quant_group=128), x)
        assert np.array_equal(c.scale * np.float32(1 << (bits - 1)), np.abs(xf).max(axis=1))


def test_reconstruction_error_bounds_and_exact_outliers():
    """|x - x^| <= S/2 on every unclipped inlier (S on the clipped positive maximum under the
    paper's divisor); <= S/2 everywhere under the full-range divisor; outliers are exact."""
    x = rng_bits(31, 1024 * 16, 1.0, heavy=True)
    xf = bits_to_f32(x).astype(np.float64)
    for bits in (4, 8):
        for rule in (RULE_PAPER, RULE_FULLRANGE):
            m = Method(bits=bits, quant_group=128, scale_rule=rule, outlier_mode=OUT_STD, stat_group=1024, thresh=4.0)
            c = oracle.compress(m, x)
            assert c.n_out > 0
            f, b = oracle.decompress(c)
            assert np.array_equal(b[c.out_idx], x[c.out_idx])
            inl = np.ones(x.size, dtype=bool)
            inl[c.out_idx] = False
            s = np.repeat(c.scale.astype(np.float64), 128)
            err = np.abs(xf - f.astype(np.float64))
            q = 1 << (bits - 1)
            clipped = (c.codes == q - 1) & (xf > (q - 0.5) * s)
            # S and code*S are each rounded once to binary32: allow 2^-22 relative on top
            slack = np.abs(xf) * 2.0 ** -22
            assert np.all(err[inl & ~clipped] <= s[inl & ~clipped] / 2 + slack[inl & ~clipped])
            assert np.all(err[inl & clipped] <= s[inl & clipped] + slack[inl & clipped])
            if rule == RULE_FULLRANGE:
                assert not clipped[inl].any()
            # the code at an outlier position is the code of 0
            assert np.all(c.codes[c.out_idx] == 0)


def test_scale_is_taken_after_outliers_are_zeroed():
    v = np.ones(64, dtype=np.float32)
    v[10] = 1000.0
    v[20] = -3.0
    x = bf16_bits(v)
    c = oracle.compress(Method(bits=8, quant_group=64, outlier_mode=OUT_ABS, thresh=100.0), x)
    assert c.out_idx.tolist() == [10] and c.out_val.tolist() == [int(x[10])]
    assert float(c.scale[0]) == 3.0 / 128.0  # the 1000 no longer sets the scale
    f, _ = oracle.decompress(c)
    assert f[10] == 1000.0 and f[20] == -3.0


def test_special_case_equals_textbook_per_token_int8():
    """No outliers + symmetric + full-range + one group per row is the usual per-token
    abs-max int8 quantiser: compare with a three-line NumPy expression."""
    rows, hidden = 64, 1024
    x = rng_bits(77, rows * hidden, 1.5)
    xf = bits_to_f32(x).reshape(rows, hidden).astype(np.float64)
    amax = np.abs(xf).max(axis=1, keepdims=True)
    want = np.clip(np.rint(xf / amax * 127.0), -128, 127).astype(np.int64)
    c = oracle.compress(Method(bits=8, quant_group=hidden, scale_rule=RULE_FULLRANGE), x)
    got = c.codes.reshape(rows, hidden).astype(np.int64)
    diff = np.abs(got - want)
    assert diff.max() <= 1
    # X * (D / max) and X / max * D differ by one rounding: the codes may differ only where the
    # exact ratio sits within 1e-5 of a half-integer (bf16 inputs make such near-ties common)
    r = xf / amax * 127.0
    off = np.abs(np.abs(r - np.floor(r)) - 0.5)
    assert np.all(off[diff != 0] < 1e-5)
    assert (diff != 0).mean() < 1e-3
    assert np.allclose(c.scale.astype(np.float64), (amax / 127.0).ravel(), rtol=2e-7)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("rule", [RULE_PAPER, RULE_FULLRANGE])
@pytest.mark.parametrize("dtype", [oracle.DT_BF16, oracle.DT_F16])
def test_a_tensor_on_the_quantisation_grid_is_a_fixed_point(bits, rule, dtype):
    """x = c / 8 with integer c over the whole code range and the range's end present in every group
    (Eq. 2): the scale is exactly 1/8, the codes are c, the reconstruction is x bit for bit, and
    compressing the reconstruction gives the same codes and scales again.  Both 16-bit formats hold
    these values exactly (|c| <= 128 needs 8 significant bits)."""
    q = 1 << (bits - 1)
    d = q if rule == RULE_PAPER else q - 1
    gq, groups = 32, 16
    g = np.random.default_rng(40 + bits + rule)
    c = g.integers(-d if rule == RULE_FULLRANGE else -q, q, size=(groups, gq))
    c[:, 0] = -d                       # the end of the range: max |x| = d / 8, so S = 1 / 8
    if rule == RULE_FULLRANGE:
        c[1::2, 0] = d                 # either sign of the largest magnitude serves
    x = oracle.from_f32((c.reshape(-1) / 8.0).astype(np.float32), dtype)
    assert np.array_equal(oracle.to_f32(x, dtype), (c.reshape(-1) / 8.0).astype(np.float32))
    m = Method(bits=bits, quant_group=gq, scale_rule=rule, dtype=dtype)
    first = oracle.compress(m, x)
    assert np.all(first.scale == np.float32(0.125))
    assert np.array_equal(first.codes.astype(np.int64), c.reshape(-1))
    f, b = oracle.decompress(first)
    assert np.array_equal(b, x), "a tensor on the grid comes back bit for bit"
    assert np.array_equal(f, oracle.to_f32(x, dtype))
    second = oracle.compress(m, b)
    assert np.array_equal(second.codes, first.codes) and np.array_equal(second.scale, first.scale)
    assert np.array_equal(second.packed, first.packed)


def test_symmetry_and_monotonicity_of_codes():
    # every positive bf16 below 4 plus the negatives, in one group with absmax 4
    pos = np.arange(0x0080, 0x4080, 37, dtype=np.uint16)
    v = np.concatenate([pos, pos | 0x8000, np.array([0x4080, 0xC080], dtype=np.uint16)])
    pad = (-v.size) % 8
    v = np.concatenate([v, np.zeros(pad, dtype=np.uint16)])
    for bits in (4, 8):
        c = oracle.compress(Method(bits=bits, quant_group=v.size, scale_rule=RULE_FULLRANGE), v)
        cp, cn = c.codes[:pos.size].astype(int), c.codes[pos.size:2 * pos.size].astype(int)
        assert np.array_equal(cp, -cn)                    # q(-y) = -q(y)
        assert np.all(np.diff(cp) >= 0)                   # monotone in y


def test_int4_nibble_order_and_int8_bytes():
    v = bf16_bits([1, -1, 2, -2, 3, -3, 7, -8])
    c = oracle.compress(Method(bits=4, quant_group=8), v)
    assert c.codes.tolist() == [1, -1, 2, -2, 3, -3, 7, -8]
    assert c.packed.tolist() == [0xF1, 0xE2, 0xD3, 0x87]  # element 2j low nibble, 2j+1 high
    c8 = oracle.compress(Method(bits=8, quant_group=8), v)
    assert c8.packed.tolist() == [(t * 16) & 0xFF for t in [1, -1, 2, -2, 3, -3, 7, -8]]


def test_degenerate_groups():
    z = np.zeros(64, dtype=np.uint16)
    z[3] = 0x8000  # negative zero
    for asym in (0, 1):
        c = oracle.compress(Method(bits=8, quant_group=64, asym=asym), z)
        assert c.scale.tolist() == [0.0] and np.all(c.codes == 0)
        f, _ = oracle.decompress(c)
        assert np.all(f == 0)
    # constant group, asymmetric: O = the constant, S = 0, exact reconstruction
    k = bf16_bits(np.full(64, 0.75, dtype=np.float32))
    c = oracle.compress(Method(bits=4, quant_group=64, asym=1), k)
    assert c.zp.tolist() == [0.75] and c.scale.tolist() == [0.0]
    f, _ = oracle.decompress(c)
    assert np.all(f == 0.75)
    # a group so small that D / max overflows still gives finite, in-range codes
    t = np.zeros(64, dtype=np.uint16)
    t[0] = 0x0001
    t[1] = 0x8001
    c = oracle.compress(Method(bits=8, quant_group=64), t)
    # hand-worked: max = 2^-133, D/max = 2^140 overflows and is held at FLT_MAX < 2^128,
    # so |x * inv| < 2^-5 and every code rounds to 0; S = 2^-140 is still a (denormal) number
    assert np.all(c.codes == 0) and float(c.scale[0]) == 2.0 ** -140
    f, _ = oracle.decompress(c)
    assert np.all(np.isfinite(f))
    # empty tensor
    e = oracle.compress(Method(bits=8, quant_group=64), np.zeros(0, dtype=np.uint16))
    assert e.n_out == 0 and e.codes.size == 0


def test_capacity_truncates_the_stream_but_not_the_count():
    x = rng_bits(41, 2048, 1.0, heavy=True)
    m = Method(bits=8, quant_group=64, outlier_mode=OUT_ABS, thresh=1.0)
    full = oracle.compress(m, x)
    cut = oracle.compress(m, x, cap=10)
    assert cut.n_out == full.n_out > 10
    assert np.array_equal(cut.out_idx, full.out_idx[:10])
    assert np.array_equal(cut.codes, full.codes)
    assert np.all(np.diff(full.out_idx) > 0)


def test_malformed_methods_are_rejected():
    x = np.zeros(128, dtype=np.uint16)
    for m in (Method(bits=5, quant_group=64), Method(bits=8, quant_group=0), Method(bits=8, quant_group=64, dtype=2),
              Method(bits=8, quant_group=64, outlier_mode=OUT_STD, stat_group=0, thresh=1.0),
              Method(bits=8, quant_group=64, outlier_mode=OUT_TOPK, stat_group=64, topk=0)):
        with pytest.raises(ValueError):
            oracle.compress(m, x)


# ----------------------------------------------------------------- outlier channels (Section 3.2, Eq. 1)
def _planted(tokens, hidden, channels, seed, gain=50.0):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(tokens, hidden, generator=g)
    x[:, channels] *= gain
    return bf16_bits(x.numpy()).reshape(tokens, hidden)


def test_channel_scores_are_exact_integer_sums_on_small_integers():
    """Small integers: S_h must be the integer column sum of |x| - over the tokens (axis 0), not the
    channels - for square and non-square shapes.  A channel holding an Inf sums to +Inf, one holding
    a NaN to NaN."""
    rng = np.random.default_rng(11)
    for tokens, hidden in ((1, 8), (64, 8), (65, 24), (200, 24), (333, 7)):
        xi = rng.integers(-8, 9, size=(tokens, hidden))
        S = oracle.channel_scores(bf16_bits(xi.astype(np.float32)), tokens, hidden)
        assert np.array_equal(S, np.abs(xi).sum(axis=0).astype(np.float64))
    xb = bf16_bits(np.ones((5, 4), dtype=np.float32)).reshape(5, 4)
    xb[2, 1], xb[3, 2], xb[4, 2] = 0xFF80, 0x7FC0, 0x7F80  # -Inf;  NaN and +Inf in one channel
    S = oracle.channel_scores(xb, 5, 4)
    assert S[0] == 5.0 and S[1] == np.inf and np.isnan(S[2]) and S[3] == 5.0


def test_channel_scores_are_the_exactly_rounded_sums():
    """Against math.fsum (exact sum of binary64 values, rounded once): equal to the last bit, on
    ordinary activations and on columns whose magnitudes span the whole bf16 range (where adding
    one value after the other in binary64 loses the small terms)."""
    tokens, hidden = 1000, 40
    xb = _planted(tokens, hidden, [3], seed=12)
    rng = np.random.default_rng(120)
    wide = rng.integers(0, 0x7F80, size=(tokens, 8)).astype(np.uint16)          # any finite magnitude
    wide |= (rng.integers(0, 2, size=wide.shape).astype(np.uint16) << 15)       # any sign
    wide[:, 1] &= 0x807F                                                        # subnormals only
    wide[0, 2], wide[1:, 2] = 0x7F7F, rng.integers(0, 0x0100, size=tokens - 1)  # one huge, many tiny
    xb = np.concatenate([xb, wide], axis=1)
    hidden += 8
    S = oracle.channel_scores(xb, tokens, hidden)
    xf = np.abs(bits_to_f32(xb.reshape(-1)).reshape(tokens, hidden)).astype(np.float64)
    lossy = 0
    for h in range(hidden):
        assert S[h] == math.fsum(xf[:, h])
        lossy += float(np.cumsum(xf[:, h])[-1]) != S[h]
    assert lossy > 0  # the test data does tell an exact sum from a running binary64 sum


def test_channel_selection_is_the_z_score_rule():
    """Against numpy's mean / population std: Z = (S - mu) / sigma > threshold."""
    rng = np.random.default_rng(13)
    for hidden, thr in ((11, 3.0), (256, 3.0), (1000, 2.0), (4096, 3.0), (777, 1.0)):
        S = rng.gamma(50.0, 1.0, size=hidden)
        S[rng.integers(0, hidden, size=max(1, hidden // 100))] *= 3.0
        z = (S - S.mean()) / S.std()
        assert np.all(np.abs(z - thr) > 1e-9)  # no decision rests on the last bits
        got, mu, sigma = oracle.channel_select(S, thr)
        assert np.array_equal(got.astype(bool), z > thr)
        assert math.isclose(mu, S.mean(), rel_tol=1e-12) and math.isclose(sigma, S.std(), rel_tol=1e-12)


def test_one_deviating_channel_scores_sqrt_of_hidden_minus_one():
    """Closed form: if all channels but one are alike, that one has Z = sqrt(hidden - 1).  So with the
    paper's threshold of 3 it is selected for hidden = 11 (Z = 3.16) and not for hidden = 9 (2.83),
    and no tensor with at most 9 channels can have an outlier channel at all."""
    for hidden, want in ((9, 0), (11, 1), (64, 1)):
        S = np.full(hidden, 7.0)
        S[hidden // 2] = 9.5
        got, _, _ = oracle.channel_select(S, 3.0)
        assert got.sum() == want and (want == 0 or got[hidden // 2] == 1)
    rng = np.random.default_rng(14)
    for _ in range(200):
        hidden = int(rng.integers(1, 10))
        got, _, _ = oracle.channel_select(rng.lognormal(0.0, 3.0, size=hidden), 3.0)
        assert got.sum() == 0


def test_channel_selection_degenerate_cases():
    got, mu, sigma = oracle.channel_select(np.full(32, 5.0), 3.0)  # sigma = 0: nothing stands out
    assert got.sum() == 0 and mu == 5.0 and sigma == 0.0
    S = np.full(32, 5.0)
    S[4] = np.inf  # a channel that cannot be summed is kept whole and stays out of the statistics
    got, mu, sigma = oracle.channel_select(S, 3.0)
    assert list(np.nonzero(got)[0]) == [4] and mu == 5.0 and sigma == 0.0
    S[7] = 1e6
    got, mu, sigma = oracle.channel_select(S, 3.0)
    assert list(np.nonzero(got)[0]) == [4, 7]
    S[9] = np.nan  # a NaN sum (a NaN in the channel) has no Z at all and is kept whole all the same
    got, mu, sigma = oracle.channel_select(S, 3.0)
    assert list(np.nonzero(got)[0]) == [4, 7, 9] and np.isfinite(mu) and np.isfinite(sigma)


@pytest.mark.parametrize("bits,asym", [(4, 0), (8, 0), (4, 1), (8, 1)])
def test_channel_compression_keeps_channels_whole_and_quantises_the_rest(bits, asym):
    """Structure of Section 3.2: the outlier channels and their indices are kept uncompressed, they
    are zero in what gets quantised (so the rest equals plain group quantisation, pinned above, of
    the tensor with those channels cleared), and decompression puts them back bit for bit."""
    tokens, hidden, planted = 130, 64, [5, 40]
    xb = _planted(tokens, hidden, planted, seed=15)
    m = Method(bits=bits, quant_group=32, asym=asym)
    c = oracle.channel_compress(m, xb, tokens, hidden, 3.0)
    assert c.n_ch == 2 and list(c.ch_idx) == planted
    assert np.array_equal(c.ch_val, xb[:, planted])
    cleared = xb.copy()
    cleared[:, planted] = 0
    plain = oracle.compress(m, cleared)
    assert np.array_equal(c.packed, plain.packed) and np.array_equal(c.codes, plain.codes)
    assert np.array_equal(c.scale.view(np.uint32), plain.scale.view(np.uint32))
    assert np.array_equal(c.zp.view(np.uint32), plain.zp.view(np.uint32))
    f, b = oracle.channel_decompress(c)
    pf, pb = oracle.decompress(plain)
    f, b, pf, pb = (a.reshape(tokens, hidden) for a in (f, b, pf, pb))
    rest = np.setdiff1d(np.arange(hidden), planted)
    assert np.array_equal(b[:, planted], xb[:, planted])
    assert np.array_equal(f[:, planted], bits_to_f32(xb[:, planted].reshape(-1)).reshape(tokens, 2))
    assert np.array_equal(b[:, rest], pb[:, rest]) and np.array_equal(f[:, rest].view(np.uint32), pf[:, rest].view(np.uint32))


def test_channel_compression_reports_more_channels_than_fit():
    tokens, hidden = 70, 64
    xb = _planted(tokens, hidden, [5, 40], seed=16)
    c = oracle.channel_compress(Method(bits=8, quant_group=32), xb, tokens, hidden, 3.0, cap=1)
    assert c.n_ch == 2 and list(c.ch_idx) == [5]


def test_no_outlier_channel_means_plain_quantisation():
    tokens, hidden = 64, 128
    rng = np.random.default_rng(17)  # every channel has the same magnitudes in another order: all S_h alike
    mags = np.stack([rng.permutation(np.arange(1, tokens + 1)) for _ in range(hidden)], axis=1)
    xb = bf16_bits((mags * rng.choice([-0.25, 0.25], size=(tokens, hidden))).astype(np.float32))
    m = Method(bits=4, quant_group=64)
    c = oracle.channel_compress(m, xb, tokens, hidden, 3.0)
    plain = oracle.compress(m, xb)
    assert c.n_ch == 0 and np.array_equal(c.packed, plain.packed)
    assert np.array_equal(c.scale.view(np.uint32), plain.scale.view(np.uint32))


# ----------------------------------------------------------------- dropout mask, byte -> bit (Section 3.2)
def test_mask_bit_format_is_an_eighth_and_lossless():
    """The paper's two statements about the scheme: bit format instead of byte format (an eighth of
    the bytes, rounded up) and no loss.  The bit order is pinned with numpy's packbits (a library
    routine) and one hand-written byte."""
    rng = np.random.default_rng(31)
    for n in (0, 1, 7, 8, 9, 31, 32, 33, 1000, 4099):
        mask = (rng.random(n) < 0.9).astype(np.uint8)  # keep probability 0.9, as a dropout of 0.1
        bits = oracle.mask_pack(mask)
        assert bits.size == (n + 7) // 8
        assert np.array_equal(bits, np.packbits(mask, bitorder="little"))
        assert np.array_equal(oracle.mask_unpack(bits, n), mask)
        assert np.array_equal(oracle.mask_unpack(bits, n), np.unpackbits(bits, bitorder="little")[:n])
    assert list(oracle.mask_pack(np.array([1, 0, 0, 1, 0, 0, 0, 0, 1], dtype=np.uint8))) == [0b00001001, 0b1]
    # any non-zero byte counts as kept and comes back as 1
    assert list(oracle.mask_unpack(oracle.mask_pack(np.array([255, 0, 2], dtype=np.uint8)), 3)) == [1, 0, 1]


# ----------------------------------------------------------------- channel-wise symmetric quantisation (Section 3.2, Q/K/V)
def test_channelwise_toy_vector_as_a_column():
    """The vector printed with Eq. 2 placed in one channel of a [5, 3] matrix: that channel gets the
    hand-worked scale and codes of the golden file whatever its neighbours hold."""
    g = read_golden("eq2_symmetric_toy.txt")
    col = np.array([float(v) for v in g["input"]], dtype=np.float32)
    x = np.stack([col * 100.0, col, np.zeros(5, dtype=np.float32)], axis=1)  # [tokens=5, hidden=3]
    codes, packed, scale = oracle.channelwise_compress(4, bf16_bits(x), 5, 3)
    codes = codes.reshape(5, 3)
    assert float(scale[1]) == float(g["scale"][0]) and codes[:, 1].tolist() == [int(v) for v in g["codes"]]
    assert float(scale[0]) == 25.0 and codes[:, 0].tolist() == codes[:, 1].tolist()
    assert float(scale[2]) == 0.0 and codes[:, 2].tolist() == [0] * 5
    f, _ = oracle.channelwise_decompress(4, packed, scale, 5, 3)
    assert f.reshape(5, 3)[:, 1].tolist() == [float(v) for v in g["dequant"]]


@pytest.mark.parametrize("bits,rule", [(4, RULE_PAPER), (8, RULE_PAPER), (8, RULE_FULLRANGE)])
def test_channelwise_is_group_quantisation_of_the_transposed_tensor(bits, rule):
    """One scale per channel over all tokens = plain group quantisation (pinned above) of the
    transposed matrix with one group per row; the transposition is numpy's."""
    tokens, hidden = 96, 40
    rng = np.random.default_rng(41)
    x = rng.standard_normal((tokens, hidden)).astype(np.float32) * rng.lognormal(0, 1.5, size=hidden).astype(np.float32)
    xb = bf16_bits(x).reshape(tokens, hidden)
    xb[3, 5] = 0x7F80   # +Inf: counts as zero
    xb[4, 5] = 0x8000   # -0
    xb[:, 7] = 0        # an empty channel
    codes, packed, scale = oracle.channelwise_compress(bits, xb, tokens, hidden, rule)
    t = oracle.compress(Method(bits=bits, quant_group=tokens, scale_rule=rule), np.ascontiguousarray(xb.T))
    assert np.array_equal(codes.reshape(tokens, hidden), t.codes.reshape(hidden, tokens).T)
    assert np.array_equal(scale.view(np.uint32), t.scale.view(np.uint32))
    # packing follows the tensor's own order
    if bits == 8:
        assert np.array_equal(packed.view(np.int8), codes)
    else:
        assert np.array_equal(packed & 0xF, codes[0::2].astype(np.uint8) & 0xF)
        assert np.array_equal(packed >> 4, codes[1::2].astype(np.uint8) & 0xF)
    f, b = oracle.channelwise_decompress(bits, packed, scale, tokens, hidden)
    tf, tb = oracle.decompress(t)
    assert np.array_equal(f.reshape(tokens, hidden).view(np.uint32), tf.reshape(hidden, tokens).T.view(np.uint32))
    assert np.array_equal(b.reshape(tokens, hidden), tb.reshape(hidden, tokens).T)
    # the error bound of Eq. 2 per channel: half a step, a whole step for the capped maximum
    xf = bits_to_f32(xb.reshape(-1)).reshape(tokens, hidden)
    xf[~np.isfinite(xf)] = 0.0
    err = np.abs(f.reshape(tokens, hidden).astype(np.float64) - xf)
    # (plus the binary32 rounding of S, D/max and code * S: well below a thousandth of a step)
    assert np.all(err <= scale.astype(np.float64)[None, :] * ((1.0 if rule == RULE_PAPER else 0.5) + 1e-3) + 1e-30)
