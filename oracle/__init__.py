"""ctypes front end of the CPU oracle (oracle/adacc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  The product package never imports this module
and this module never imports the product package.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np

from .build import build as _build, LIB as _LIB

OUT_NONE, OUT_ABS, OUT_STD, OUT_TOPK = 0, 1, 2, 3
RULE_PAPER, RULE_FULLRANGE = 0, 1
DT_BF16, DT_F16 = 0, 1


class _CMethod(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_uint32), ("quant_group", ctypes.c_uint32), ("asym", ctypes.c_uint32),
                ("scale_rule", ctypes.c_uint32), ("outlier_mode", ctypes.c_uint32),
                ("stat_group", ctypes.c_uint32), ("thresh", ctypes.c_float), ("topk", ctypes.c_uint32),
                ("dtype", ctypes.c_uint32)]


@dataclass
class Method:
    bits: int = 8
    quant_group: int = 64
    asym: int = 0
    scale_rule: int = RULE_PAPER
    outlier_mode: int = OUT_NONE
    stat_group: int = 0
    thresh: float = 0.0
    topk: int = 0
    dtype: int = DT_BF16

    def c(self):
        return _CMethod(self.bits, self.quant_group, self.asym, self.scale_rule, self.outlier_mode,
                        self.stat_group, float(self.thresh), self.topk, self.dtype)


MODE_BY_NAME = {"none": OUT_NONE, "abs": OUT_ABS, "std": OUT_STD, "topk": OUT_TOPK}


def method_from_dict(md, scale_rule: int = RULE_PAPER, dtype: int = DT_BF16) -> Method:
    """A method written as a plain dictionary (outlier_mode by name) as the oracle's descriptor."""
    return Method(bits=md["bits"], quant_group=md["quant_group"], asym=md["asym"], scale_rule=scale_rule,
                  outlier_mode=MODE_BY_NAME[md["outlier_mode"]], stat_group=md["stat_group"],
                  thresh=md["thresh"], topk=md["topk"], dtype=dtype)


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            _build(force=True)
        L = ctypes.CDLL(_LIB)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.oracle_select_outliers.argtypes = [ctypes.POINTER(_CMethod), vp, sz, vp]
        L.oracle_select_outliers.restype = ctypes.c_int
        L.oracle_compress.argtypes = [ctypes.POINTER(_CMethod), vp, sz, vp, vp, vp, vp, vp, vp, sz,
                                      ctypes.POINTER(sz)]
        L.oracle_compress.restype = ctypes.c_int
        L.oracle_decompress.argtypes = [ctypes.POINTER(_CMethod), vp, vp, vp, vp, vp, sz, sz, vp, vp]
        L.oracle_decompress.restype = ctypes.c_int
        L.oracle_logical_bytes.argtypes = [ctypes.POINTER(_CMethod), sz, sz]
        L.oracle_logical_bytes.restype = ctypes.c_uint64
        L.oracle_pairwise_sum.argtypes = [vp, sz]
        L.oracle_pairwise_sum.restype = ctypes.c_float
        dp = ctypes.POINTER(ctypes.c_double)
        L.oracle_to_f32.argtypes = [ctypes.POINTER(_CMethod), ctypes.c_uint16]
        L.oracle_to_f32.restype = ctypes.c_float
        L.oracle_from_f32.argtypes = [ctypes.POINTER(_CMethod), ctypes.c_float]
        L.oracle_from_f32.restype = ctypes.c_uint16
        L.oracle_channel_scores.argtypes = [ctypes.c_uint32, vp, sz, sz, vp]
        L.oracle_channel_scores.restype = None
        L.oracle_channel_select.argtypes = [vp, sz, ctypes.c_float, vp, vp]
        L.oracle_channel_select.restype = None
        L.oracle_channel_compress.argtypes = [ctypes.POINTER(_CMethod), vp, sz, sz, ctypes.c_float, vp, vp, vp,
                                              vp, vp, vp, sz, ctypes.POINTER(sz)]
        L.oracle_channel_compress.restype = ctypes.c_int
        L.oracle_channel_decompress.argtypes = [ctypes.POINTER(_CMethod), vp, vp, vp, vp, vp, sz, sz, sz, vp, vp]
        L.oracle_channel_decompress.restype = ctypes.c_int
        L.oracle_channelwise_compress.argtypes = [ctypes.POINTER(_CMethod), vp, sz, sz, vp, vp, vp]
        L.oracle_channelwise_compress.restype = ctypes.c_int
        L.oracle_channelwise_decompress.argtypes = [ctypes.POINTER(_CMethod), vp, vp, sz, sz, vp, vp]
        L.oracle_channelwise_decompress.restype = ctypes.c_int
        L.oracle_mask_pack.argtypes = [vp, sz, vp]
        L.oracle_mask_pack.restype = None
        L.oracle_mask_unpack.argtypes = [vp, sz, vp]
        L.oracle_mask_unpack.restype = None
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _as_u16(x):
    x = np.ascontiguousarray(x)
    if x.dtype != np.uint16:
        raise TypeError("oracle input is an array of 16-bit patterns (uint16)")
    return x.reshape(-1)


@dataclass
class Compressed:
    method: Method
    n: int
    codes: np.ndarray      # int8 [n]
    packed: np.ndarray     # uint8 [n*bits/8]
    scale: np.ndarray      # float32 [n/Gq]
    zp: np.ndarray         # float32 [n/Gq] (asym) or empty
    out_idx: np.ndarray    # int32 [min(n_out, cap)]
    out_val: np.ndarray    # uint16 [min(n_out, cap)]
    n_out: int


def select_outliers(m: Method, x_bits) -> np.ndarray:
    x = _as_u16(x_bits)
    out = np.zeros(x.size, dtype=np.uint8)
    cm = m.c()
    rc = lib().oracle_select_outliers(ctypes.byref(cm), _p(x), x.size, _p(out))
    if rc != 0:
        raise ValueError("oracle: malformed method")
    return out


def compress(m: Method, x_bits, cap=None) -> Compressed:
    x = _as_u16(x_bits)
    n = x.size
    cap = n if cap is None else int(cap)
    groups = -(-n // m.quant_group) if m.quant_group else 0
    codes = np.zeros(n, dtype=np.int8)
    packed = np.zeros((n * m.bits + 7) // 8, dtype=np.uint8)
    scale = np.zeros(groups, dtype=np.float32)
    zp = np.zeros(groups if m.asym else 0, dtype=np.float32)
    oi = np.zeros(max(cap, 1), dtype=np.int32)
    ov = np.zeros(max(cap, 1), dtype=np.uint16)
    n_out = ctypes.c_size_t(0)
    cm = m.c()
    rc = lib().oracle_compress(ctypes.byref(cm), _p(x), n, _p(codes), _p(packed), _p(scale),
                               _p(zp) if m.asym else None, _p(oi), _p(ov), cap, ctypes.byref(n_out))
    if rc != 0:
        raise ValueError("oracle: malformed method")
    k = min(n_out.value, cap)
    return Compressed(m, n, codes, packed, scale, zp, oi[:k].copy(), ov[:k].copy(), n_out.value)


def decompress(c: Compressed):
    """Returns (xhat_f32, xhat_bf16_bits)."""
    f = np.zeros(c.n, dtype=np.float32)
    b = np.zeros(c.n, dtype=np.uint16)
    cm = c.method.c()
    oi = np.ascontiguousarray(c.out_idx)
    ov = np.ascontiguousarray(c.out_val)
    rc = lib().oracle_decompress(ctypes.byref(cm), _p(c.packed), _p(c.scale),
                                 _p(c.zp) if c.method.asym else None, _p(oi), _p(ov), oi.size, c.n,
                                 _p(f), _p(b))
    if rc != 0:
        raise ValueError("oracle: decompress failed")
    return f, b


def logical_bytes(m: Method, n: int, n_out: int) -> int:
    cm = m.c()
    return int(lib().oracle_logical_bytes(ctypes.byref(cm), n, n_out))


def pairwise_sum(v) -> np.float32:
    v = np.ascontiguousarray(v, dtype=np.float32)
    return np.float32(lib().oracle_pairwise_sum(_p(v), v.size))


# ---- outlier channels (Section 3.2, Eq. 1) ----

@dataclass
class ChannelCompressed:
    method: Method
    tokens: int
    hidden: int
    codes: np.ndarray      # int8 [tokens*hidden]
    packed: np.ndarray     # uint8
    scale: np.ndarray      # float32 [n/Gq]
    zp: np.ndarray         # float32 [n/Gq] (asym) or empty
    ch_idx: np.ndarray     # int32 [min(n_ch, cap)]
    ch_val: np.ndarray     # uint16 [tokens, n_ch] (empty if n_ch > cap)
    n_ch: int


def channel_scores(x_bits, tokens: int, hidden: int, dtype: int = DT_BF16) -> np.ndarray:
    x = _as_u16(x_bits)
    assert x.size == tokens * hidden
    S = np.zeros(hidden, dtype=np.float64)
    lib().oracle_channel_scores(dtype, _p(x), tokens, hidden, _p(S))
    return S


def to_f32(x_bits, dtype: int = DT_BF16) -> np.ndarray:
    """The oracle's own widening of 16-bit patterns, element by element."""
    cm = Method(dtype=dtype).c()
    f = lib().oracle_to_f32
    return np.array([f(ctypes.byref(cm), int(b)) for b in _as_u16(x_bits)], dtype=np.float32)


def from_f32(values, dtype: int = DT_BF16) -> np.ndarray:
    """The oracle's own rounding of binary32 values to the 16-bit format, element by element."""
    cm = Method(dtype=dtype).c()
    f = lib().oracle_from_f32
    return np.array([f(ctypes.byref(cm), float(v)) for v in np.asarray(values, dtype=np.float32).reshape(-1)],
                    dtype=np.uint16)


def channel_select(S, z_thresh: float):
    """Returns (is_out uint8[hidden], mu, sigma)."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    out = np.zeros(S.size, dtype=np.uint8)
    stats = np.zeros(2, dtype=np.float64)
    lib().oracle_channel_select(_p(S), S.size, float(z_thresh), _p(out), _p(stats))
    return out, float(stats[0]), float(stats[1])


def channel_compress(m: Method, x_bits, tokens: int, hidden: int, z_thresh: float = 3.0, cap=None) -> ChannelCompressed:
    x = _as_u16(x_bits)
    n = tokens * hidden
    assert x.size == n
    cap = hidden if cap is None else int(cap)
    groups = -(-n // m.quant_group) if m.quant_group else 0
    codes = np.zeros(n, dtype=np.int8)
    packed = np.zeros((n * m.bits + 7) // 8, dtype=np.uint8)
    scale = np.zeros(groups, dtype=np.float32)
    zp = np.zeros(groups if m.asym else 0, dtype=np.float32)
    ci = np.zeros(max(cap, 1), dtype=np.int32)
    cv = np.zeros(max(tokens * cap, 1), dtype=np.uint16)
    n_ch = ctypes.c_size_t(0)
    cm = m.c()
    rc = lib().oracle_channel_compress(ctypes.byref(cm), _p(x), tokens, hidden, float(z_thresh), _p(codes),
                                       _p(packed), _p(scale), _p(zp) if m.asym else None, _p(ci), _p(cv), cap,
                                       ctypes.byref(n_ch))
    if rc != 0:
        raise ValueError("oracle: malformed method")
    k = n_ch.value
    if k <= cap:
        vals = cv[:tokens * k].copy().reshape(tokens, k)
    else:
        vals = np.zeros((tokens, 0), dtype=np.uint16)
    return ChannelCompressed(m, tokens, hidden, codes, packed, scale, zp, ci[:min(k, cap)].copy(), vals, k)


def channel_decompress(c: ChannelCompressed):
    """Returns (xhat_f32, xhat_bf16_bits)."""
    n = c.tokens * c.hidden
    f = np.zeros(n, dtype=np.float32)
    b = np.zeros(n, dtype=np.uint16)
    cm = c.method.c()
    ci = np.ascontiguousarray(c.ch_idx)
    cv = np.ascontiguousarray(c.ch_val).reshape(-1)
    rc = lib().oracle_channel_decompress(ctypes.byref(cm), _p(c.packed), _p(c.scale),
                                         _p(c.zp) if c.method.asym else None, _p(ci), _p(cv), ci.size, c.tokens,
                                         c.hidden, _p(f), _p(b))
    if rc != 0:
        raise ValueError("oracle: channel decompress failed")
    return f, b


# ---- dropout mask: byte format <-> bit format (Section 3.2) ----

def mask_pack(mask) -> np.ndarray:
    m = np.ascontiguousarray(mask).view(np.uint8).reshape(-1)
    bits = np.zeros((m.size + 7) // 8, dtype=np.uint8)
    lib().oracle_mask_pack(_p(m), m.size, _p(bits))
    return bits


def mask_unpack(bits, n: int) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint8).reshape(-1)
    assert b.size >= (n + 7) // 8
    m = np.zeros(n, dtype=np.uint8)
    lib().oracle_mask_unpack(_p(b), n, _p(m))
    return m


# ---- channel-wise symmetric quantisation (Section 3.2: Query, Key, Value) ----

def channelwise_compress(bits: int, x_bits, tokens: int, hidden: int, scale_rule: int = RULE_PAPER, dtype: int = DT_BF16):
    """Returns (codes int8 [tokens*hidden], packed uint8, scale float32 [hidden])."""
    x = _as_u16(x_bits)
    n = tokens * hidden
    assert x.size == n
    codes = np.zeros(n, dtype=np.int8)
    packed = np.zeros((n * bits + 7) // 8, dtype=np.uint8)
    scale = np.zeros(hidden, dtype=np.float32)
    cm = Method(bits=bits, quant_group=1, scale_rule=scale_rule, dtype=dtype).c()
    if lib().oracle_channelwise_compress(ctypes.byref(cm), _p(x), tokens, hidden, _p(codes), _p(packed), _p(scale)) != 0:
        raise ValueError("oracle: malformed method")
    return codes, packed, scale


def channelwise_decompress(bits: int, packed, scale, tokens: int, hidden: int, dtype: int = DT_BF16):
    """Returns (xhat_f32, xhat_bf16_bits)."""
    n = tokens * hidden
    f = np.zeros(n, dtype=np.float32)
    b = np.zeros(n, dtype=np.uint16)
    cm = Method(bits=bits, quant_group=1, dtype=dtype).c()
    pk = np.ascontiguousarray(packed, dtype=np.uint8)
    sc = np.ascontiguousarray(scale, dtype=np.float32)
    if lib().oracle_channelwise_decompress(ctypes.byref(cm), _p(pk), _p(sc), tokens, hidden, _p(f), _p(b)) != 0:
        raise ValueError("oracle: channel-wise decompress failed")
    return f, b
