"""A second, independent statement of the whole compression chain of Section 3.2 / Fig. 3(c), for tiny
tensors: pure Python, one element at a time, exact rational arithmetic (`fractions.Fraction`) with an
explicit round-to-nearest-even to binary32 after every operation that the method performs in
binary32.  It shares nothing with the C oracle (no numpy float32 arithmetic, no C library rounding)
and exists to pin the oracle's *composition*: select -> keep -> zero -> scale -> quantise -> pack ->
dequantise -> put the outliers back.

Restricted to what exact rationals can express: a group whose range overflows binary32 is not
supported (the oracle's own tests cover that case).
"""
from fractions import Fraction

FLT_MAX = Fraction((2 ** 24 - 1) * 2 ** 104)
NONE, ABS, STD, TOPK = 0, 1, 2, 3
PAPER, FULLRANGE = 0, 1
BF16, F16 = 0, 1   # the tensor's 16-bit format


def round_half_even(q: Fraction) -> int:
    f = q.numerator // q.denominator  # floor
    rest = q - f
    if rest > Fraction(1, 2) or (rest == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return f


def to_grid(q: Fraction, sig_bits: int, min_exp: int) -> Fraction:
    """q rounded to the nearest number with `sig_bits` significant bits (ties to even), with the
    spacing never finer than 2^min_exp (the subnormal range)."""
    if q == 0:
        return Fraction(0)
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()  # 2^(e-1) <= a < 2^(e+1)
    if Fraction(2) ** e > a:
        e -= 1                                                   # now 2^e <= a < 2^(e+1)
    quantum = Fraction(2) ** max(e - (sig_bits - 1), min_exp)
    r = round_half_even(a / quantum) * quantum
    return r if q > 0 else -r


def f32(q: Fraction) -> Fraction:
    """Round to binary32 (24 significant bits, spacing at least 2^-149).  Overflow is not handled."""
    r = to_grid(q, 24, -149)
    assert abs(r) <= FLT_MAX, "outside binary32"
    return r


def bf16_value(bits: int):
    """Value of a bf16 bit pattern as a Fraction; None for Inf / NaN."""
    e, f = (bits >> 7) & 0xFF, bits & 0x7F
    if e == 0xFF:
        return None
    mag = Fraction(f, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(f, 128)) * Fraction(2) ** (e - 127)
    return -mag if bits >> 15 else mag


def bf16_bits_of(q: Fraction) -> int:
    """binary32 value -> bf16 bit pattern, round to nearest even (finite values only)."""
    r = to_grid(q, 8, -133)
    sign = 0x8000 if (r < 0) else 0
    a = abs(r)
    if a == 0:
        return 0x8000 if q < 0 else 0  # a negative value that rounds to zero keeps its sign
    if a < Fraction(2) ** -126:
        return sign | int(a / Fraction(2) ** -133)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    return sign | ((e + 127) << 7) | int((a / Fraction(2) ** e - 1) * 128)


def f16_value(bits: int):
    """Value of a binary16 bit pattern (5 exponent bits, bias 15, 10 fraction bits); None for Inf / NaN."""
    e, f = (bits >> 10) & 0x1F, bits & 0x3FF
    if e == 0x1F:
        return None
    mag = Fraction(f, 1024) * Fraction(2) ** -14 if e == 0 else (1 + Fraction(f, 1024)) * Fraction(2) ** (e - 15)
    return -mag if bits >> 15 else mag


def f16_bits_of(q: Fraction) -> int:
    """binary32 value -> binary16 bit pattern, round to nearest even; what rounds past the largest finite
    value (65504) is infinite."""
    r = to_grid(q, 11, -24)
    sign = 0x8000 if (r < 0 or (r == 0 and q < 0)) else 0
    a = abs(r)
    if a == 0:
        return sign
    if a > 65504:
        return sign | 0x7C00
    if a < Fraction(2) ** -14:
        return sign | int(a / Fraction(2) ** -24)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    return sign | ((e + 15) << 10) | int((a / Fraction(2) ** e - 1) * 1024)


def value_of(bits: int, fmt: int):
    return f16_value(bits) if fmt == F16 else bf16_value(bits)


def bits_of_value(q: Fraction, fmt: int) -> int:
    return f16_bits_of(q) if fmt == F16 else bf16_bits_of(q)


def pairwise(v):
    """Canonical pairwise binary32 sum: pad with zeros to a power of two, split in halves."""
    n = 1
    while n < len(v):
        n *= 2
    v = list(v) + [Fraction(0)] * (n - len(v))

    def rec(lo, hi):
        if hi - lo == 1:
            return v[lo]
        mid = (lo + hi) // 2
        return f32(rec(lo, mid) + rec(mid, hi))
    return rec(0, n)


def select(bits, mode, stat_group, thresh: Fraction, topk, fmt=BF16):
    n = len(bits)
    vals = [value_of(b, fmt) for b in bits]
    out = [False] * n
    if mode == ABS:
        out = [v is not None and abs(v) > thresh for v in vals]
    elif mode == STD:
        k2 = f32(thresh * thresh)
        for g0 in range(0, n, stat_group):
            grp = vals[g0:g0 + stat_group]
            if any(v is None for v in grp):
                continue  # the statistics are not numbers: nothing passes the threshold
            s1 = pairwise(grp)
            s2 = pairwise([v * v for v in grp])  # squares of 16-bit values are exact in binary32
            mean = f32(s1 / len(grp))                      # a short last group has its own count
            var = f32(f32(s2 / len(grp)) - mean * mean)    # fused: one rounding
            if var < 0:
                var = Fraction(0)
            limit = f32(k2 * var)
            for i, v in enumerate(grp):
                out[g0 + i] = v * v > limit
    elif mode == TOPK:
        for g0 in range(0, n, stat_group):
            order = sorted(range(g0, min(n, g0 + stat_group)), key=lambda i: (-(bits[i] & 0x7FFF), i))
            for i in order[:topk]:
                out[i] = True
    if mode != NONE:
        for i, v in enumerate(vals):
            if v is None:
                out[i] = True
    return out


def compress(bits, *, nbits, quant_group, asym, rule, mode, stat_group=0, thresh=Fraction(0), topk=0, fmt=BF16):
    """Returns a dict: codes, packed, scale, zp (Fractions), out_idx, out_val.  Groups are cut from the
    start of the flat array; the last one of either kind may be short."""
    n = len(bits)
    q = 1 << (nbits - 1)
    out = select(bits, mode, stat_group, thresh, topk, fmt)
    out_idx = [i for i in range(n) if out[i]]
    out_val = [bits[i] for i in out_idx]
    y = []
    for i, b in enumerate(bits):
        v = value_of(b, fmt)
        y.append(Fraction(0) if (out[i] or v is None) else v)
    codes, scale, zp = [], [], []
    for g0 in range(0, n, quant_group):
        grp = y[g0:g0 + quant_group]
        if not asym:
            d = q if rule == PAPER else q - 1
            a = max(abs(v) for v in grp)
            scale.append(f32(a / d))
            inv = Fraction(0) if a == 0 else min(to_grid(Fraction(d) / a, 24, -149), FLT_MAX)
            for v in grp:
                codes.append(min(max(round_half_even(f32(v * inv)), -q), q - 1))
        else:
            d2 = 2 * q if rule == PAPER else 2 * q - 1
            hi, lo = max(grp), min(grp)
            o = f32(f32(hi + lo) / 2)
            r = f32(hi - lo)
            zp.append(o)
            scale.append(f32(r / d2))
            inv = Fraction(0) if r == 0 else min(to_grid(Fraction(d2) / r, 24, -149), FLT_MAX)
            for v in grp:
                codes.append(min(max(round_half_even(f32(f32(v - o) * inv)), -q), q - 1))
    if nbits == 8:
        packed = [c & 0xFF for c in codes]
    else:
        packed = []
        for j in range((n + 1) // 2):
            hi_nib = (codes[2 * j + 1] & 0xF) if 2 * j + 1 < n else 0
            packed.append((codes[2 * j] & 0xF) | (hi_nib << 4))
    return dict(codes=codes, packed=packed, scale=scale, zp=zp, out_idx=out_idx, out_val=out_val)


def decompress(c, *, n, nbits, quant_group, asym, fmt=BF16):
    """Returns (list of Fractions or None for a non-finite outlier, list of 16-bit patterns)."""
    xs, bs = [], []
    for i in range(n):
        if nbits == 8:
            code = c["packed"][i] - 256 if c["packed"][i] >= 128 else c["packed"][i]
        else:
            nib = (c["packed"][i // 2] >> (4 * (i & 1))) & 0xF
            code = nib - 16 if nib >= 8 else nib
        s = c["scale"][i // quant_group]
        v = f32(code * s + c["zp"][i // quant_group]) if asym else f32(code * s)
        xs.append(v)
        bs.append(bits_of_value(v, fmt))
    for i, b in zip(c["out_idx"], c["out_val"]):
        xs[i] = value_of(b, fmt)
        bs[i] = b
    return xs, bs
