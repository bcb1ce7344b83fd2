"""Saved-activation compression for a real forward / backward pass, and the per-tensor figures
the policy maker consumes.

Adacc compresses the activations an operator saves for its backward pass and decompresses them
when the backward pass needs them (Fig. 3(c)); which tensors, and how, is the per-tensor policy
R_{i,t} of Section 3.3, whose inputs are the compression rate CRate_i and the times Tc_i / Tdc_i
(Section 3.3, and re-evaluated during training, Section 3.4).  `SavedActivationCompression` is a
`torch.autograd.graph.saved_tensors_hooks` context that does exactly that with libadacc, and keeps
those three figures per saved tensor.

Dropout masks (`torch.bool` tensors saved for the backward pass) are kept in bit format, the
fourth of the layer-specific schemes of Section 3.2, when `pack_masks` is set.

Plumbing only: the hooks allocate buffers and call the library; every step of compression and
decompression runs in the HIP kernels.  A tensor the policy does not cover is saved as it is.
"""
import dataclasses

import torch

from . import (DTYPE_BF16, DTYPE_F16, AdaccError, ChannelMethod, Method, KIND_NOOP, OUTLIER_NONE, alloc_blob, alloc_channel_blob,
               alloc_channel_workspace, alloc_workspace, channel_compress, channel_compressed_bytes,
               channel_decompress, channel_layout_of, channel_workspace_bytes, compress, compressed_bytes, decompress,
               layout_of, mask_pack, mask_packed_bytes, mask_unpack, workspace_bytes)


class CompressedActivationLost(RuntimeError):
    """A saved activation needed more room for its outliers than its method allowed: the blob does not
    hold the tensor, and the backward pass must not go on with it."""


class _StatusPool:
    """Pinned host words for the status of every compressed tensor, filled by asynchronous copies."""
    CHUNK = 1024

    def __init__(self):
        self.chunks, self.used = [], 0

    def take(self):
        if self.used % self.CHUNK == 0 and self.used // self.CHUNK == len(self.chunks):
            self.chunks.append(torch.zeros((self.CHUNK, 4), dtype=torch.int32, pin_memory=True))
        slot = self.chunks[self.used // self.CHUNK][self.used % self.CHUNK]
        self.used += 1
        return slot


class _Saved:
    """What the autograd graph holds instead of the activation."""
    __slots__ = ("method", "blob", "layout", "shape", "numel", "record")

    def __init__(self, method, blob, layout, shape, numel, record):
        self.method, self.blob, self.layout, self.shape, self.numel, self.record = method, blob, layout, shape, numel, record


class _SavedMask:
    """A boolean mask in bit format."""
    __slots__ = ("bits", "shape", "numel", "record")

    def __init__(self, bits, shape, numel, record):
        self.bits, self.shape, self.numel, self.record = bits, shape, numel, record


class SavedActivationCompression(torch.autograd.graph.saved_tensors_hooks):
    """`with SavedActivationCompression(policy): loss = model(x)` then `loss.backward()`.

    policy(tensor) returns an adacc `Method` (element outliers), a `ChannelMethod` (outlier channels
    by Z-score; the tensor is taken as [numel / last_dim, last_dim]) or None (retain).  Only contiguous
    bf16 and float16 CUDA tensors are offered to the policy; the method's dtype field follows the tensor.  timing=True brackets every library call with events
    so that `report()` can give Tc_i and Tdc_i (it costs a synchronisation in `report()` only).

    The number of outliers moves while a model trains (Section 3.4), so a method's `max_outliers` /
    `max_channels` can turn out too small.  The status words of every blob are copied to the host as
    soon as the blob is written (asynchronously), and looked at before the blob is used:
    on_overflow="raise" (the default) makes the backward pass raise `CompressedActivationLost`;
    on_overflow="retain" waits for the status right after compression and saves the tensor as it is when
    the blob can not hold it (one synchronisation per compressed tensor in the forward pass).
    A tensor whose address or shape the library does not take (not 16-byte aligned; for outlier channels a
    size the groups do not divide or a last dimension that is no multiple of 8) is saved as it is.
    """

    def __init__(self, policy, timing=True, pack_masks=True, on_overflow="raise"):
        if on_overflow not in ("raise", "retain"):
            raise ValueError("on_overflow is 'raise' or 'retain'")
        self.policy = policy
        self.timing = timing
        self.pack_masks = pack_masks
        self.on_overflow = on_overflow
        self.records = []
        self.retained = []   # (shape, reason) of tensors offered to the policy and saved as they are
        self._status = _StatusPool()
        self._ws = None      # workspace of compression with outliers, grown on demand, reused by every tensor (one stream)
        self._cws = None     # workspace of the channel statistics
        super().__init__(self._pack, self._unpack)

    # ---- hooks
    def _eligible(self, t):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype in (torch.bfloat16, torch.float16) and t.is_contiguous()
                and t.numel() > 0 and t.data_ptr() % 16 == 0):
            return False
        return not (t.is_leaf and t.requires_grad)  # parameters are not activations

    def _pack_mask(self, t):
        numel = t.numel()
        rec = {"shape": tuple(t.shape), "numel": numel, "method": "mask", "events": {}}
        ev = self._events(rec, "compress")
        bits = torch.empty(mask_packed_bytes(numel), dtype=torch.uint8, device=t.device)
        mask_pack(t, bits, numel)
        if ev:
            ev[1].record()
        self.records.append(rec)
        return _SavedMask(bits, t.shape, numel, rec)

    def _pack(self, t):
        if (self.pack_masks and isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bool
                and t.is_contiguous() and t.numel() > 0 and t.data_ptr() % 16 == 0):
            return self._pack_mask(t)
        if not self._eligible(t):
            return t
        m = self.policy(t)
        if m is None or (isinstance(m, Method) and m.kind == KIND_NOOP):
            return t
        fmt = DTYPE_F16 if t.dtype == torch.float16 else DTYPE_BF16
        if m.dtype != fmt:  # the policy names the method; the format is the tensor's
            m = dataclasses.replace(m, dtype=fmt)
        numel = t.numel()
        try:  # a shape the method can not take is no error of the training run: the tensor is retained
            if isinstance(m, ChannelMethod):
                channel_layout_of(m, numel // t.shape[-1], t.shape[-1])
            else:
                layout_of(m, numel)
        except AdaccError as e:
            self.retained.append((tuple(t.shape), str(e)))
            return t
        rec = {"shape": tuple(t.shape), "numel": numel, "method": m, "events": {}}
        ev = self._events(rec, "compress")
        if isinstance(m, ChannelMethod):
            hidden = t.shape[-1]
            tokens = numel // hidden
            blob, layout = alloc_channel_blob(m, tokens, hidden, device=t.device)
            if self._cws is None or self._cws.numel() < channel_workspace_bytes(tokens, hidden):
                self._cws = alloc_channel_workspace(tokens, hidden, device=t.device)
            channel_compress(m, t, tokens, hidden, blob, self._cws)
        else:
            blob, layout = alloc_blob(m, numel, device=t.device)
            ws = None
            if m.outlier_mode != OUTLIER_NONE:
                want = workspace_bytes(m, numel)
                if self._ws is None or self._ws.c.bytes < want:
                    self._ws = alloc_workspace(want, device=t.device)
                ws = self._ws
            compress(m, t, blob, ws)
        if ev:
            ev[1].record()
        # the record keeps a host copy of the 16 status bytes, not the blob: the compressed activation is
        # freed as soon as autograd drops it
        rec["status"] = self._status.take()
        rec["status"].copy_(blob[layout.status_off:layout.status_off + 16].view(torch.int32), non_blocking=True)
        rec["status_ready"] = torch.cuda.Event()
        rec["status_ready"].record()
        if self.on_overflow == "retain" and self._lost(rec):
            rec["retained"] = True
            self.records.append(rec)
            return t
        self.records.append(rec)
        return _Saved(m, blob, layout, t.shape, numel, rec)

    @staticmethod
    def _lost(rec):
        """True when the blob of this record does not hold its tensor.  Waits for the status copy only."""
        rec["status_ready"].synchronize()
        st = rec["status"].tolist()
        return bool(st[1] or st[2])

    def _unpack(self, s):
        if isinstance(s, _SavedMask):
            out = torch.empty(s.shape, dtype=torch.bool, device=s.bits.device)
            ev = self._events(s.record, "decompress")
            mask_unpack(s.bits, out, s.numel)
            if ev:
                ev[1].record()
            return out
        if not isinstance(s, _Saved):
            return s
        if self._lost(s.record):
            m = s.method
            room = m.max_channels if isinstance(m, ChannelMethod) else m.max_outliers
            raise CompressedActivationLost(
                f"saved activation of shape {tuple(s.shape)}: {s.record['status'][0].item()} outliers found, the method "
                f"has room for {room}; raise max_outliers / max_channels or use on_overflow='retain'")
        out = torch.empty(s.shape, dtype=torch.float16 if s.method.dtype == DTYPE_F16 else torch.bfloat16,
                          device=s.blob.device)
        ev = self._events(s.record, "decompress")
        if isinstance(s.method, ChannelMethod):
            hidden = s.shape[-1]
            channel_decompress(s.method, s.blob, s.numel // hidden, hidden, out)
        else:
            decompress(s.method, s.blob, out)
        if ev:
            ev[1].record()
        return out

    def _events(self, rec, key):
        if not self.timing:
            return None
        ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        ev[0].record()
        rec["events"][key] = ev
        return ev

    # ---- the figures of Section 3.3 / 3.4, one entry per compressed tensor, in the order they were saved
    def report(self):
        """[{shape, numel, n_outliers, overflow, original_bytes, compressed_bytes, crate, tc_ms, tdc_ms}].
        crate = compressed / original bytes, the factor CRate_i multiplies M_i with in the memory
        constraint of Section 3.3.  Waits for the GPU."""
        torch.cuda.synchronize()
        rows = []
        for rec in self.records:
            m = rec["method"]
            if m == "mask":  # byte format -> bit format
                row = {"shape": rec["shape"], "numel": rec["numel"], "n_outliers": 0, "overflow": False,
                       "original_bytes": rec["numel"], "compressed_bytes": mask_packed_bytes(rec["numel"]),
                       "crate": mask_packed_bytes(rec["numel"]) / float(rec["numel"]), "tc_ms": None, "tdc_ms": None}
                for key, name in (("compress", "tc_ms"), ("decompress", "tdc_ms")):
                    ev = rec["events"].get(key)
                    if ev:
                        row[name] = ev[0].elapsed_time(ev[1])
                rows.append(row)
                continue
            st = rec["status"].tolist()
            if rec.get("retained"):
                comp = 2 * rec["numel"]
            elif isinstance(m, ChannelMethod):
                hidden = rec["shape"][-1]
                comp = channel_compressed_bytes(m, rec["numel"] // hidden, hidden, st[0])
            else:
                comp = compressed_bytes(m, rec["numel"], st[0])
            row = {"shape": rec["shape"], "numel": rec["numel"], "n_outliers": st[0], "overflow": bool(st[1] or st[2]),
                   "original_bytes": 2 * rec["numel"], "compressed_bytes": comp,
                   "crate": comp / (2.0 * rec["numel"]), "tc_ms": None, "tdc_ms": None}
            for key, name in (("compress", "tc_ms"), ("decompress", "tdc_ms")):
                ev = rec["events"].get(key)
                if ev:
                    row[name] = ev[0].elapsed_time(ev[1])
            rows.append(row)
        return rows
