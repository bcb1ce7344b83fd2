"""Thin Python binding of libadacc (see include/adacc.h).

Argument marshalling only: every step of compression and decompression runs in the
HIP kernels of libadacc.so.  PyTorch tensors are used as device buffers; the current
torch stream is the stream the work is enqueued on.  There is no CPU fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadacc.so")

# ---- constants of include/adacc.h
OK, EINVAL, ENULL, ESIZE, EALIGN, EHIP, ELIMIT = 0, -1, -2, -3, -4, -5, -6
KIND_NOOP, KIND_QUANT = 0, 1
OUTLIER_NONE, OUTLIER_ABS, OUTLIER_STD, OUTLIER_TOPK = 0, 1, 2, 3
SCALE_PAPER, SCALE_FULLRANGE = 0, 1
DST_16, DST_F32 = 0, 1
DST_BF16 = DST_16
DTYPE_BF16, DTYPE_F16 = 0, 1

EXPORTS = ("adacc_layout_of", "adacc_workspace_bytes", "adacc_workspace_init", "adacc_compress", "adacc_compress_noalloc",
           "adacc_decompress", "adacc_batch_workspace_bytes", "adacc_compress_batch",
           "adacc_decompress_batch", "adacc_read_status", "adacc_hbm_copy", "adacc_hbm_stream", "adacc_strerror",
           "adacc_version", "adacc_channel_layout_of", "adacc_channel_workspace_bytes",
           "adacc_channel_compress", "adacc_channel_decompress", "adacc_channel_read_status",
           "adacc_mask_packed_bytes", "adacc_mask_pack", "adacc_mask_unpack", "adacc_compressed_bytes",
           "adacc_channel_compressed_bytes",
           "adacc_channelwise_layout_of", "adacc_channelwise_workspace_bytes", "adacc_channelwise_compress",
           "adacc_channelwise_decompress")


class CMethod(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_uint32), ("bits", ctypes.c_uint32), ("quant_group", ctypes.c_uint32),
                ("asym", ctypes.c_uint32), ("scale_rule", ctypes.c_uint32), ("outlier_mode", ctypes.c_uint32),
                ("stat_group", ctypes.c_uint32), ("thresh", ctypes.c_float), ("topk", ctypes.c_uint32),
                ("max_outliers", ctypes.c_uint32), ("dtype", ctypes.c_uint32)]


class CLayout(ctypes.Structure):
    _fields_ = [("codes_off", ctypes.c_uint64), ("scales_off", ctypes.c_uint64), ("zp_off", ctypes.c_uint64),
                ("tile_ptr_off", ctypes.c_uint64), ("idx_off", ctypes.c_uint64), ("val_off", ctypes.c_uint64),
                ("status_off", ctypes.c_uint64), ("total_bytes", ctypes.c_uint64),
                ("tile_elems", ctypes.c_uint32), ("n_tiles", ctypes.c_uint32)]


class CWorkspace(ctypes.Structure):
    _fields_ = [("device_mem", ctypes.c_void_p), ("bytes", ctypes.c_uint64), ("epoch", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]


class CChannelMethod(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_uint32), ("quant_group", ctypes.c_uint32), ("asym", ctypes.c_uint32),
                ("scale_rule", ctypes.c_uint32), ("z_thresh", ctypes.c_float), ("max_channels", ctypes.c_uint32),
                ("dtype", ctypes.c_uint32)]


class CChannelLayout(ctypes.Structure):
    _fields_ = [(k, ctypes.c_uint64) for k in ("codes_off", "scales_off", "zp_off", "ch_mask_off", "ch_base_off",
                                                "ch_idx_off", "ch_val_off", "status_off", "total_bytes")]


class CChannelwiseLayout(ctypes.Structure):
    _fields_ = [("codes_off", ctypes.c_uint64), ("scales_off", ctypes.c_uint64), ("total_bytes", ctypes.c_uint64)]


@dataclass
class ChannelMethod:
    """Outlier channels by Z-score (adacc_channel_method)."""
    bits: int = 4
    quant_group: int = 128
    asym: int = 0
    scale_rule: int = SCALE_PAPER
    z_thresh: float = 3.0
    max_channels: int = 64
    dtype: int = DTYPE_BF16

    def c(self) -> CChannelMethod:
        return CChannelMethod(self.bits, self.quant_group, self.asym, self.scale_rule, float(self.z_thresh),
                              self.max_channels, self.dtype)


@dataclass
class Method:
    kind: int = KIND_QUANT
    bits: int = 8
    quant_group: int = 64
    asym: int = 0
    scale_rule: int = SCALE_PAPER
    outlier_mode: int = OUTLIER_NONE
    stat_group: int = 0
    thresh: float = 0.0
    topk: int = 0
    max_outliers: int = 0
    dtype: int = DTYPE_BF16

    def c(self) -> CMethod:
        return CMethod(self.kind, self.bits, self.quant_group, self.asym, self.scale_rule, self.outlier_mode,
                       self.stat_group, float(self.thresh), self.topk, self.max_outliers, self.dtype)


NOOP = Method(kind=KIND_NOOP, bits=0, quant_group=0)

OUTLIER_MODE_BY_NAME = {"none": OUTLIER_NONE, "abs": OUTLIER_ABS, "std": OUTLIER_STD, "topk": OUTLIER_TOPK}


def method_from_dict(md, max_outliers: int, scale_rule: int = SCALE_PAPER, dtype: int = DTYPE_BF16) -> Method:
    """A method written as a plain dictionary (keys bits, quant_group, asym, outlier_mode by name,
    stat_group, thresh, topk) as the library's descriptor; None = retain the tensor as it is."""
    if md is None:
        return NOOP
    return Method(kind=KIND_QUANT, bits=md["bits"], quant_group=md["quant_group"], asym=md["asym"],
                  scale_rule=scale_rule, outlier_mode=OUTLIER_MODE_BY_NAME[md["outlier_mode"]],
                  stat_group=md["stat_group"], thresh=md["thresh"], topk=md["topk"], max_outliers=max_outliers,
                  dtype=dtype)


class AdaccError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib():
    """Load libadacc.so (built by paper_2508_00806_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2508_00806_amd.build` first "
                              "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, u64, u32, ci = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        pm, pl = ctypes.POINTER(CMethod), ctypes.POINTER(CLayout)
        L.adacc_layout_of.argtypes = [pm, u64, pl]
        L.adacc_layout_of.restype = ci
        L.adacc_workspace_bytes.argtypes = [pm, u64]
        L.adacc_workspace_bytes.restype = u64
        pw = ctypes.POINTER(CWorkspace)
        L.adacc_workspace_init.argtypes = [pw, vp, u64, vp]
        L.adacc_workspace_init.restype = ci
        L.adacc_compress.argtypes = [pm, vp, u64, vp, u64, pw, vp]
        L.adacc_compress.restype = ci
        L.adacc_compress_noalloc.argtypes = [pm, vp, u64, vp, u64, vp]
        L.adacc_compress_noalloc.restype = ci
        L.adacc_decompress.argtypes = [pm, vp, u64, u64, vp, ci, vp]
        L.adacc_decompress.restype = ci
        pvp, pu64 = ctypes.POINTER(vp), ctypes.POINTER(u64)
        L.adacc_batch_workspace_bytes.argtypes = [u32, pm, pu64]
        L.adacc_batch_workspace_bytes.restype = u64
        L.adacc_compress_batch.argtypes = [u32, pm, pvp, pu64, pvp, pu64, pw, vp]
        L.adacc_compress_batch.restype = ci
        L.adacc_decompress_batch.argtypes = [u32, pm, pvp, pu64, pu64, pvp, ci, pw, vp]
        L.adacc_decompress_batch.restype = ci
        L.adacc_read_status.argtypes = [vp, pl, vp, ctypes.POINTER(u32 * 4)]
        L.adacc_read_status.restype = ci
        L.adacc_hbm_copy.argtypes = [vp, vp, u64, vp]
        L.adacc_hbm_copy.restype = ci
        L.adacc_hbm_stream.argtypes = [ci, vp, vp, vp, u64, vp]
        L.adacc_hbm_stream.restype = ci
        L.adacc_strerror.argtypes = [ci]
        L.adacc_strerror.restype = ctypes.c_char_p
        pcm, pcl = ctypes.POINTER(CChannelMethod), ctypes.POINTER(CChannelLayout)
        L.adacc_channel_layout_of.argtypes = [pcm, u64, u32, pcl]
        L.adacc_channel_layout_of.restype = ci
        L.adacc_channel_workspace_bytes.argtypes = [u64, u32]
        L.adacc_channel_workspace_bytes.restype = u64
        L.adacc_channel_compress.argtypes = [pcm, vp, u64, u32, vp, u64, vp, u64, vp]
        L.adacc_channel_compress.restype = ci
        L.adacc_channel_decompress.argtypes = [pcm, vp, u64, u64, u32, vp, ci, vp]
        L.adacc_channel_decompress.restype = ci
        L.adacc_channel_read_status.argtypes = [vp, pcl, vp, ctypes.POINTER(u32 * 4)]
        L.adacc_channel_read_status.restype = ci
        L.adacc_mask_packed_bytes.argtypes = [u64]
        L.adacc_mask_packed_bytes.restype = u64
        L.adacc_mask_pack.argtypes = [vp, u64, vp, vp]
        L.adacc_mask_pack.restype = ci
        L.adacc_mask_unpack.argtypes = [vp, u64, vp, vp]
        L.adacc_mask_unpack.restype = ci
        L.adacc_compressed_bytes.argtypes = [pm, u64, u64]
        L.adacc_compressed_bytes.restype = u64
        L.adacc_channel_compressed_bytes.argtypes = [pcm, u64, u32, u64]
        L.adacc_channel_compressed_bytes.restype = u64
        L.adacc_channelwise_layout_of.argtypes = [u32, u64, u32, ctypes.POINTER(CChannelwiseLayout)]
        L.adacc_channelwise_layout_of.restype = ci
        L.adacc_channelwise_workspace_bytes.argtypes = [u64, u32]
        L.adacc_channelwise_workspace_bytes.restype = u64
        L.adacc_channelwise_compress.argtypes = [u32, u32, u32, vp, u64, u32, vp, u64, vp, u64, vp]
        L.adacc_channelwise_compress.restype = ci
        L.adacc_channelwise_decompress.argtypes = [u32, u32, vp, u64, u64, u32, vp, ci, vp]
        L.adacc_channelwise_decompress.restype = ci
        L.adacc_version.argtypes = []
        L.adacc_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().adacc_strerror(int(code)).decode()


def version() -> str:
    return lib().adacc_version().decode()


def _check(rc, where):
    if rc != OK:
        raise AdaccError(rc, where)


def torch_dtype(dtype: int):
    """The torch dtype of a tensor in the 16-bit format DTYPE_*."""
    import torch
    return torch.float16 if dtype == DTYPE_F16 else torch.bfloat16


def _dst_dtype(dst, dtype: int) -> int:
    """ABI code for the element type of dst: binary32, or the 16-bit format `dtype` names."""
    import torch
    if dst.dtype == torch.float32:
        return DST_F32
    if dst.dtype != torch_dtype(dtype):
        raise TypeError(f"dst must be float32 or {torch_dtype(dtype)}, the tensor's own format")
    return DST_16


def _ptr(t):
    """Device pointer of a torch tensor (or an int / None passed through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t):
    return t.numel() * t.element_size()


def _stream(stream):
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


# ---------------------------------------------------------------- host-only helpers
def layout_of(method: Method, numel: int) -> CLayout:
    L = CLayout()
    cm = method.c()
    _check(lib().adacc_layout_of(ctypes.byref(cm), numel, ctypes.byref(L)), "adacc_layout_of")
    return L


def workspace_bytes(method: Method, numel: int) -> int:
    cm = method.c()
    return int(lib().adacc_workspace_bytes(ctypes.byref(cm), numel))


def compressed_bytes(method: Method, numel: int, n_outliers: int) -> int:
    """Information-carrying bytes of a blob; CRate_i of Section 3.3 = this / (2 * numel)."""
    cm = method.c()
    return int(lib().adacc_compressed_bytes(ctypes.byref(cm), numel, n_outliers))


def batch_workspace_bytes(methods, numels) -> int:
    n = len(methods)
    cms = (CMethod * n)(*[m.c() for m in methods])
    cn = (ctypes.c_uint64 * n)(*numels)
    return int(lib().adacc_batch_workspace_bytes(n, cms, cn))


# ---------------------------------------------------------------- device calls
class Workspace:
    """A workspace of compression with outliers: the adacc_workspace struct plus the torch buffer it points to."""

    def __init__(self, buffer, stream=None):
        self.buffer = buffer  # keeps the device memory alive
        self.c = CWorkspace()
        _check(lib().adacc_workspace_init(ctypes.byref(self.c), _ptr(buffer), _nbytes(buffer), _stream(stream)),
               "adacc_workspace_init")

    @property
    def ref(self):
        return ctypes.byref(self.c)


def _ws(workspace):
    return None if workspace is None else workspace.ref


def compress(method: Method, src, blob, workspace=None, numel=None, stream=None):
    numel = src.numel() if numel is None else numel
    cm = method.c()
    _check(lib().adacc_compress(ctypes.byref(cm), _ptr(src), numel, _ptr(blob), _nbytes(blob), _ws(workspace),
                                _stream(stream)), "adacc_compress")


NOALLOC_MAX_NUMEL = 1 << 27


def compress_noalloc(method: Method, src, blob, numel=None, stream=None):
    """adacc_compress_noalloc: no workspace argument, nothing is allocated by the call."""
    numel = src.numel() if numel is None else numel
    cm = method.c()
    _check(lib().adacc_compress_noalloc(ctypes.byref(cm), _ptr(src), numel, _ptr(blob), _nbytes(blob),
                                        _stream(stream)), "adacc_compress_noalloc")


def decompress(method: Method, blob, dst, numel=None, stream=None):
    import torch
    numel = dst.numel() if numel is None else numel
    dtype = _dst_dtype(dst, method.dtype)
    cm = method.c()
    _check(lib().adacc_decompress(ctypes.byref(cm), _ptr(blob), _nbytes(blob), numel, _ptr(dst), dtype,
                                  _stream(stream)), "adacc_decompress")


def _batch_args(methods, tensors_a, numels, tensors_b):
    n = len(methods)
    cms = (CMethod * n)(*[m.c() for m in methods])
    pa = (ctypes.c_void_p * n)(*[_ptr(t) for t in tensors_a])
    pb = (ctypes.c_void_p * n)(*[_ptr(t) for t in tensors_b])
    cn = (ctypes.c_uint64 * n)(*numels)
    return n, cms, pa, cn, pb


class BatchArgs:
    """The argument arrays of a batch call, marshalled once.  A training loop that compresses the
    same set of buffers every step builds this once and calls it every step; the tensors are kept
    alive by the object."""

    def __init__(self, methods, tensors_a, tensors_b, numels, blobs):
        self.n, self.methods, self.pa, self.numels, self.pb = _batch_args(methods, tensors_a, numels, tensors_b)
        self.blob_bytes = (ctypes.c_uint64 * self.n)(*[0 if b is None else _nbytes(b) for b in blobs])
        self.keep = (list(tensors_a), list(tensors_b))


def prepare_compress_batch(methods, srcs, blobs) -> BatchArgs:
    return BatchArgs(methods, srcs, blobs, [0 if s is None else s.numel() for s in srcs], blobs)


def prepare_decompress_batch(methods, blobs, dsts) -> BatchArgs:
    import torch
    kinds = {_dst_dtype(d, m.dtype) for m, d in zip(methods, dsts) if d is not None}
    if len(kinds) > 1:
        raise TypeError("the dsts of a batch are all float32 or all in their tensors' own formats")
    args = BatchArgs(methods, blobs, dsts, [0 if d is None else d.numel() for d in dsts], blobs)
    args.dst_dtype = DST_F32 if kinds == {DST_F32} else DST_16
    return args


def compress_batch(methods, srcs, blobs, workspace, stream=None, prepared: BatchArgs = None):
    a = prepared or prepare_compress_batch(methods, srcs, blobs)
    _check(lib().adacc_compress_batch(a.n, a.methods, a.pa, a.numels, a.pb, a.blob_bytes, _ws(workspace),
                                      _stream(stream)), "adacc_compress_batch")


def decompress_batch(methods, blobs, dsts, workspace, stream=None, prepared: BatchArgs = None):
    a = prepared or prepare_decompress_batch(methods, blobs, dsts)
    _check(lib().adacc_decompress_batch(a.n, a.methods, a.pa, a.blob_bytes, a.numels, a.pb, a.dst_dtype,
                                        _ws(workspace), _stream(stream)), "adacc_decompress_batch")


def read_status(blob, layout: CLayout, stream=None):
    """(n_outliers, overflow, 0, 0) - waits for the stream."""
    out = (ctypes.c_uint32 * 4)()
    _check(lib().adacc_read_status(_ptr(blob), ctypes.byref(layout), _stream(stream), ctypes.byref(out)),
           "adacc_read_status")
    return tuple(int(v) for v in out)


def hbm_copy(dst, src, nbytes=None, stream=None):
    nbytes = _nbytes(src) if nbytes is None else nbytes
    _check(lib().adacc_hbm_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "adacc_hbm_copy")


STREAM_READ, STREAM_WRITE, STREAM_COPY, STREAM_READ2_WRITE = 0, 1, 2, 3


def hbm_stream(mix: int, dst, src_a, src_b, nbytes: int, stream=None):
    p = lambda t: None if t is None else _ptr(t)
    _check(lib().adacc_hbm_stream(mix, p(dst), p(src_a), p(src_b), nbytes, _stream(stream)), "adacc_hbm_stream")


# ---------------------------------------------------------------- outlier channels (Section 3.2, Eq. 1)
def channel_layout_of(method: ChannelMethod, tokens: int, hidden: int) -> CChannelLayout:
    L = CChannelLayout()
    cm = method.c()
    _check(lib().adacc_channel_layout_of(ctypes.byref(cm), tokens, hidden, ctypes.byref(L)),
           "adacc_channel_layout_of")
    return L


def channel_compressed_bytes(method: ChannelMethod, tokens: int, hidden: int, n_channels: int) -> int:
    """Information-carrying bytes of a channel blob that holds n_channels outlier channels."""
    cm = method.c()
    return int(lib().adacc_channel_compressed_bytes(ctypes.byref(cm), tokens, hidden, n_channels))


def channel_workspace_bytes(tokens: int, hidden: int) -> int:
    return int(lib().adacc_channel_workspace_bytes(tokens, hidden))


def channel_compress(method: ChannelMethod, src, tokens: int, hidden: int, blob, workspace, stream=None):
    cm = method.c()
    _check(lib().adacc_channel_compress(ctypes.byref(cm), _ptr(src), tokens, hidden, _ptr(blob), _nbytes(blob),
                                        _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "adacc_channel_compress")


def channel_decompress(method: ChannelMethod, blob, tokens: int, hidden: int, dst, stream=None):
    import torch
    dtype = _dst_dtype(dst, method.dtype)
    cm = method.c()
    _check(lib().adacc_channel_decompress(ctypes.byref(cm), _ptr(blob), _nbytes(blob), tokens, hidden, _ptr(dst),
                                          dtype, _stream(stream)), "adacc_channel_decompress")


def channel_read_status(blob, layout: CChannelLayout, stream=None):
    """(n_channels, overflow, 0, 0) - waits for the stream."""
    out = (ctypes.c_uint32 * 4)()
    _check(lib().adacc_channel_read_status(_ptr(blob), ctypes.byref(layout), _stream(stream), ctypes.byref(out)),
           "adacc_channel_read_status")
    return tuple(int(v) for v in out)


def alloc_channel_blob(method: ChannelMethod, tokens: int, hidden: int, device="cuda"):
    import torch
    L = channel_layout_of(method, tokens, hidden)
    return torch.empty(int(L.total_bytes), dtype=torch.uint8, device=device), L


def alloc_channel_workspace(tokens: int, hidden: int, device="cuda"):
    import torch
    return torch.empty(max(channel_workspace_bytes(tokens, hidden), 256), dtype=torch.uint8, device=device)


def channel_blob_sections(blob, layout: CChannelLayout, method: ChannelMethod, tokens: int, hidden: int):
    """Typed views of the sections of a channel blob (no copies)."""
    import torch
    numel = tokens * hidden
    groups = numel // method.quant_group

    def view(off, nbytes, dtype):
        return blob[off:off + nbytes].view(dtype)

    sec = {
        "codes": view(layout.codes_off, (numel * method.bits + 7) // 8, torch.uint8),
        "scales": view(layout.scales_off, 4 * groups, torch.float32),
        "ch_mask": view(layout.ch_mask_off, hidden // 8, torch.uint8),
        "ch_base": view(layout.ch_base_off, 4 * (hidden // 8), torch.int32),
        "ch_idx": view(layout.ch_idx_off, 4 * method.max_channels, torch.int32),
        "ch_val": view(layout.ch_val_off, 2 * tokens * method.max_channels, torch.int16),
        "status": view(layout.status_off, 16, torch.int32),
    }
    if method.asym:
        sec["zp"] = view(layout.zp_off, 4 * groups, torch.float32)
    return sec


# ---------------------------------------------------------------- channel-wise symmetric quantisation (Q / K / V)
def channelwise_layout_of(bits: int, tokens: int, hidden: int) -> CChannelwiseLayout:
    L = CChannelwiseLayout()
    _check(lib().adacc_channelwise_layout_of(bits, tokens, hidden, ctypes.byref(L)), "adacc_channelwise_layout_of")
    return L


def channelwise_workspace_bytes(tokens: int, hidden: int) -> int:
    return int(lib().adacc_channelwise_workspace_bytes(tokens, hidden))


def channelwise_compress(bits: int, src, tokens: int, hidden: int, blob, workspace, scale_rule=SCALE_PAPER, stream=None):
    import torch
    dtype = DTYPE_F16 if getattr(src, "dtype", None) == torch.float16 else DTYPE_BF16
    _check(lib().adacc_channelwise_compress(bits, scale_rule, dtype, _ptr(src), tokens, hidden, _ptr(blob), _nbytes(blob),
                                            _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "adacc_channelwise_compress")


def channelwise_decompress(bits: int, blob, tokens: int, hidden: int, dst, stream=None):
    import torch
    if dst.dtype not in (torch.float32, torch.bfloat16, torch.float16):
        raise TypeError("dst must be bfloat16, float16 or float32")
    fmt = DTYPE_F16 if dst.dtype == torch.float16 else DTYPE_BF16
    dtype = DST_F32 if dst.dtype == torch.float32 else DST_16
    _check(lib().adacc_channelwise_decompress(bits, fmt, _ptr(blob), _nbytes(blob), tokens, hidden, _ptr(dst), dtype,
                                              _stream(stream)), "adacc_channelwise_decompress")


def alloc_channelwise(bits: int, tokens: int, hidden: int, device="cuda"):
    """(blob, layout, workspace) for one tensor."""
    import torch
    L = channelwise_layout_of(bits, tokens, hidden)
    blob = torch.empty(int(L.total_bytes), dtype=torch.uint8, device=device)
    ws = torch.empty(max(channelwise_workspace_bytes(tokens, hidden), 256), dtype=torch.uint8, device=device)
    return blob, L, ws


# ---------------------------------------------------------------- dropout mask, byte <-> bit (Section 3.2)
def mask_packed_bytes(n: int) -> int:
    return int(lib().adacc_mask_packed_bytes(n))


def mask_pack(mask, bits, n=None, stream=None):
    """mask: bool / uint8 tensor of n elements; bits: uint8 tensor of at least mask_packed_bytes(n)."""
    n = mask.numel() if n is None else n
    if _nbytes(bits) < mask_packed_bytes(n) or _nbytes(mask) < n:
        raise AdaccError(ESIZE, "adacc_mask_pack")
    _check(lib().adacc_mask_pack(_ptr(mask), n, _ptr(bits), _stream(stream)), "adacc_mask_pack")


def mask_unpack(bits, mask, n=None, stream=None):
    n = mask.numel() if n is None else n
    if _nbytes(bits) < mask_packed_bytes(n) or _nbytes(mask) < n:
        raise AdaccError(ESIZE, "adacc_mask_unpack")
    _check(lib().adacc_mask_unpack(_ptr(bits), n, _ptr(mask), _stream(stream)), "adacc_mask_unpack")


# ---------------------------------------------------------------- buffer helpers (allocation = plumbing)
def alloc_blob(method: Method, numel: int, device="cuda"):
    import torch
    L = layout_of(method, numel)
    return torch.empty(max(int(L.total_bytes), 256), dtype=torch.uint8, device=device), L


def alloc_workspace(nbytes: int, device="cuda", stream=None) -> Workspace:
    """A cleared workspace of at least nbytes."""
    import torch
    buf = torch.empty(max((int(nbytes) + 255) // 256 * 256, 512), dtype=torch.uint8, device=device)
    return Workspace(buf, stream)


def blob_sections(blob, layout: CLayout, method: Method, numel: int):
    """Typed views of the sections of a blob (no copies)."""
    import torch
    groups = -(-numel // method.quant_group)  # the last group may be short
    has_out = method.outlier_mode != OUTLIER_NONE

    def view(off, nbytes, dtype):
        return blob[off:off + nbytes].view(dtype)

    sec = {
        "codes": view(layout.codes_off, (numel * method.bits + 7) // 8, torch.uint8),
        "scales": view(layout.scales_off, 4 * groups, torch.float32),
        "status": view(layout.status_off, 16, torch.int32),
    }
    if method.asym:
        sec["zp"] = view(layout.zp_off, 4 * groups, torch.float32)
    if has_out:
        sec["tile_ptr"] = view(layout.tile_ptr_off, 4 * (layout.n_tiles + 1), torch.int32)
        sec["idx"] = view(layout.idx_off, 4 * method.max_outliers, torch.int32)
        sec["val"] = view(layout.val_off, 2 * method.max_outliers, torch.int16)
    return sec
