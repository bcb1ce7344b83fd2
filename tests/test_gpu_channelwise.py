"""GPU parity for channel-wise symmetric quantisation (Section 3.2: the scheme for Query, Key and
Value): adacc_channelwise_* through the C ABI against the CPU oracle.  Bar: packed codes and scales
bit-exact; decompressed binary32 bit-equal (hence within 1e-6), bf16 equal."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_00806_amd as adacc
import workloads
from helpers import assert_bf16_matches, assert_f32_matches, bits_of, fmt_of, from_bits

pytestmark = pytest.mark.gpu


def run(x, bits, rule=0):
    tokens, hidden = x.shape
    xb = bits_of(x)
    fmt = fmt_of(x)
    codes, packed, scale = oracle.channelwise_compress(bits, xb, tokens, hidden, rule, fmt)
    blob, L, ws = adacc.alloc_channelwise(bits, tokens, hidden)
    blob.fill_(0xA5)
    adacc.channelwise_compress(bits, x.contiguous().cuda(), tokens, hidden, blob, ws, scale_rule=rule)
    n = tokens * hidden
    got_codes = blob[L.codes_off:L.codes_off + n * bits // 8].cpu().numpy()
    got_scale = blob[L.scales_off:L.scales_off + 4 * hidden].view(torch.float32).cpu().numpy()
    assert np.array_equal(got_scale.view(np.uint32), scale.view(np.uint32)), "scales differ"
    assert np.array_equal(got_codes, packed), "packed codes differ"
    of32, obf = oracle.channelwise_decompress(bits, packed, scale, tokens, hidden, fmt)
    d32 = torch.empty(n, dtype=torch.float32, device="cuda")
    dbf = torch.empty(n, dtype=x.dtype, device="cuda")
    adacc.channelwise_decompress(bits, blob, tokens, hidden, d32)
    adacc.channelwise_decompress(bits, blob, tokens, hidden, dbf)
    torch.cuda.synchronize()
    assert_f32_matches(d32.cpu().numpy(), of32)
    assert_bf16_matches(bits_of(dbf), obf, fmt)


def matrix(tokens, hidden, seed):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(tokens, hidden, generator=g) * torch.exp(torch.randn(hidden, generator=g) * 1.5)
    return x.to(torch.bfloat16)


@pytest.mark.parametrize("bits,rule", [(4, 0), (8, 0), (4, 1), (8, 1)])
def test_qkv_shaped_activation(bits, rule):
    """Channels of very different ranges (what makes one scale per channel worthwhile); 300 tokens:
    four whole chunks of 64 and a short one."""
    print(f"[channelwise] rows=300 hidden=2048 bits={bits} rule={rule}", flush=True)
    run(matrix(300, 2048, 51), bits, rule)


def test_shapes_and_tails():
    print("[channelwise] shapes", flush=True)
    run(matrix(37, 11008, 52), 8)      # hidden not a power of two, short last tile
    run(matrix(1000, 40, 53), 4)       # a tile spans 51 tokens
    run(matrix(1, 2048, 54), 8)        # one token: every code is +-max
    run(matrix(70, 8, 55), 4)          # the narrowest matrix
    run(matrix(5, 65536, 56), 8)       # the widest


def test_values_that_need_care():
    print("[channelwise] special values", flush=True)
    x = matrix(130, 256, 57)
    b = bits_of(x).reshape(130, 256).copy()
    b[5, 100] = 0x7F80    # +Inf counts as zero and does not enter the scale
    b[77, 100] = 0xFFC0   # NaN
    b[:, 7] = 0           # an empty channel: scale 0, codes 0
    b[:, 8] = 0x8000      # all -0
    b[3, 9] = 0x7F7F      # the largest finite value
    b[4, 9] = 0x0001      # the smallest denormal
    b[:, 10] = 0x0001     # a channel of denormals only: D / max overflows and is held at FLT_MAX
    run(from_bits(b.reshape(-1)).view(130, 256), 8)
    run(from_bits(b.reshape(-1)).view(130, 256), 4, rule=1)


def test_full_size_c2_shape():
    print("[channelwise] full C2 shape", flush=True)
    run(workloads.make("c2", "cpu"), 4)
