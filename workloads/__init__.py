"""Seeded synthetic activations shaped like the five benchmark configurations, and the
method each configuration applies, as plain dictionaries.

This module serves both the CPU oracle's tests and the GPU library's tests / bench, so it
contains none of the compression arithmetic: it only draws random tensors (torch ops on
the requested device) and names parameters.  The tensors stand in for activations of GPT /
LLaMA training runs; no dataset or checkpoint is involved.

Every generator takes `rows` so that tests can draw a short tensor with the same
per-row distribution as the full-size one.
"""
import math

import torch

# ---------------------------------------------------------------------------- methods
# keys: bits, quant_group, asym, outlier_mode ('none' | 'abs' | 'std' | 'topk'), stat_group, thresh, topk,
#       outliers_per_row (upper bound used to size the outlier stream; None = not bounded by construction)
C1_METHOD = dict(bits=8, quant_group=1024, asym=0, outlier_mode="std", stat_group=1024, thresh=6.0, topk=0)
C2_METHOD = dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=2048, thresh=0.0, topk=2)
C3_METHOD = dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=8.0, topk=0)
C4_METHOD = dict(bits=8, quant_group=2048, asym=1, outlier_mode="abs", stat_group=0, thresh=0.05, topk=0)
# the five saved tensors of one LLaMA-7B-shaped layer (hidden 4096, MLP 11008)
C5_LAYER = (
    ("qkv_in", 4096, dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=4096, thresh=0.0, topk=4)),
    ("attn_out", 4096, dict(bits=4, quant_group=128, asym=0, outlier_mode="topk", stat_group=4096, thresh=0.0, topk=4)),
    ("mlp_up", 11008, dict(bits=8, quant_group=128, asym=0, outlier_mode="none", stat_group=0, thresh=0.0, topk=0)),
    ("silu_out", 11008, dict(bits=8, quant_group=64, asym=0, outlier_mode="std", stat_group=64, thresh=8.0, topk=0)),
    ("down_in", 11008, None),  # retained as it is (no-op)
)
C5_LAYERS = 32
C5_ROWS = 2 * 4096

SHAPES = {"c1": (4096, 1024), "c2": (16 * 2048, 2048), "c3": (8 * 2048, 16384), "c4": (4 * 32 * 2048, 2048)}
METHODS = {"c1": C1_METHOD, "c2": C2_METHOD, "c3": C3_METHOD, "c4": C4_METHOD}


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _normal(shape, std, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std


def _outlier_channels(x, n_ch, g, device):
    """Replace n_ch columns (chosen from the seed) by heavy-tailed Student-t(nu=2) * 20."""
    rows, hidden = x.shape
    ch = torch.randperm(hidden, generator=g, device=device)[:n_ch]
    z = torch.randn((rows, n_ch), generator=g, device=device)
    a = torch.randn((rows, n_ch), generator=g, device=device)
    b = torch.randn((rows, n_ch), generator=g, device=device)
    t = z / torch.sqrt((a * a + b * b) / 2.0)
    x[:, ch] = t * 20.0
    return x


def c1(device="cpu", rows=None, seed=1001):
    """[4096, 1024] N(0,1) with 4 fixed channels scaled by 40."""
    rows = rows or SHAPES["c1"][0]
    g = _gen(seed, device)
    x = _normal((rows, 1024), 1.0, g, device)
    ch = torch.randperm(1024, generator=g, device=device)[:4]
    x[:, ch] *= 40.0
    return x.to(torch.bfloat16)


def c2(device="cpu", rows=None, seed=1002, hidden=2048):
    """[32768, 2048] N(0,1); 0.5 % of the channels heavy-tailed."""
    rows = rows or SHAPES["c2"][0]
    g = _gen(seed, device)
    x = _normal((rows, hidden), 1.0, g, device)
    x = _outlier_channels(x, max(1, round(0.005 * hidden)), g, device)
    return x.to(torch.bfloat16)


def c3(device="cpu", rows=None, seed=1003, hidden=16384):
    """[16384, 16384] exact (erf) GELU of N(0, std 1.5) pre-activations."""
    rows = rows or SHAPES["c3"][0]
    g = _gen(seed, device)
    out = torch.empty((rows, hidden), dtype=torch.bfloat16, device=device)
    step = 2048
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        out[r0:r1] = torch.nn.functional.gelu(_normal((r1 - r0, hidden), 1.5, g, device)).to(torch.bfloat16)
    return out


def c4(device="cpu", rows=None, seed=1004, seq=2048):
    """[4*32*2048, 2048] causal softmax rows of N(0, std 2) logits (row r of a [seq, seq] block keeps
    columns <= r; masked entries are exactly 0).  rows must be a multiple of seq."""
    rows = rows or SHAPES["c4"][0]
    assert rows % seq == 0
    g = _gen(seed, device)
    out = torch.empty((rows, seq), dtype=torch.bfloat16, device=device)
    keep = torch.tril(torch.ones((seq, seq), dtype=torch.bool, device=device))
    for r0 in range(0, rows, seq):
        logits = _normal((seq, seq), 2.0, g, device)
        logits = logits.masked_fill(~keep, float("-inf"))
        out[r0:r0 + seq] = torch.softmax(logits, dim=-1).to(torch.bfloat16)
    return out


def c5_tensor(name, device="cpu", rows=None, seed=5000):
    """One saved tensor of a LLaMA-7B-shaped layer."""
    rows = rows or C5_ROWS
    g = _gen(seed, device)
    if name in ("qkv_in", "attn_out"):
        x = _normal((rows, 4096), 1.0, g, device)
        return _outlier_channels(x, max(1, round(0.005 * 4096)), g, device).to(torch.bfloat16)
    if name == "mlp_up":
        return _normal((rows, 11008), 1.5, g, device).to(torch.bfloat16)
    if name == "silu_out":
        return torch.nn.functional.silu(_normal((rows, 11008), 1.5, g, device)).to(torch.bfloat16)
    if name == "down_in":
        a = _normal((rows, 11008), 1.5, g, device)
        b = _normal((rows, 11008), 1.5, g, device)
        return (torch.nn.functional.silu(a) * b).to(torch.bfloat16)
    raise KeyError(name)


def c5(device="cpu", rows=None, layers=None):
    """List of (layer, name, tensor, method-dict-or-None) for the whole layer set."""
    out = []
    for layer in range(layers or C5_LAYERS):
        for t, (name, _hidden, method) in enumerate(C5_LAYER):
            out.append((layer, name, c5_tensor(name, device, rows, seed=5000 + 10 * layer + t), method))
    return out


def make(name, device="cpu", rows=None):
    return {"c1": c1, "c2": c2, "c3": c3, "c4": c4}[name](device=device, rows=rows)


def outlier_capacity(method, numel, hidden):
    """A capacity for the outlier stream that the configuration can not exceed by construction
    (or a generous bound where the count is data dependent)."""
    if method is None or method["outlier_mode"] == "none":
        return 0
    if method["outlier_mode"] == "topk":
        return method["topk"] * (numel // method["stat_group"]) + 1024
    if method["outlier_mode"] == "abs":
        # a softmax row sums to 1: fewer than 1/tau entries can exceed tau
        return (numel // hidden) * int(math.ceil(1.0 / method["thresh"])) if method["thresh"] > 0 else numel
    return max(4096, numel // 64)


def algorithmic_bytes(method, numel, n_out, n_tiles):
    """Bytes one direction of the path has to move for a tensor: the bf16 tensor once, the codes,
    the scales (and offsets), the outliers actually produced and one offset per tile."""
    if method is None:
        return 0
    groups = numel // method["quant_group"]
    b = 2 * numel + numel * method["bits"] // 8 + 4 * groups * (2 if method["asym"] else 1)
    if method["outlier_mode"] != "none":
        b += 6 * n_out + 4 * n_tiles
    return b
