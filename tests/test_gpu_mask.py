"""GPU parity for the dropout-mask scheme (Section 3.2: byte format to bit format, lossless):
adacc_mask_pack / adacc_mask_unpack through the C ABI against the CPU oracle, byte for byte."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_00806_amd as adacc

pytestmark = pytest.mark.gpu


def roundtrip(mask_np):
    n = mask_np.size
    want = oracle.mask_pack(mask_np)
    m = torch.from_numpy(mask_np).cuda()
    bits = torch.full((max(adacc.mask_packed_bytes(n), 1) + 16,), 0xA5, dtype=torch.uint8, device="cuda")
    adacc.mask_pack(m, bits, n)
    got = bits.cpu().numpy()
    assert np.array_equal(got[:want.size], want), "packed bits differ"
    assert np.all(got[want.size:] == 0xA5), "wrote past the packed mask"
    back = torch.full((n + 16,), 7, dtype=torch.uint8, device="cuda")
    adacc.mask_unpack(bits, back, n)
    b = back.cpu().numpy()
    assert np.array_equal(b[:n], oracle.mask_unpack(want, n)), "unpacked mask differs"
    assert np.array_equal(b[:n], (mask_np != 0).astype(np.uint8)) and np.all(b[n:] == 7)


@pytest.mark.parametrize("n", [1, 7, 8, 31, 32, 33, 255, 1024, 4099, 32 * 256 * 4 + 17, 3_000_001])
def test_mask_sizes_and_tails(n):
    print(f"[mask] n={n}", flush=True)
    rng = np.random.default_rng(n)
    roundtrip((rng.random(n) < 0.9).astype(np.uint8))


def test_mask_bytes_other_than_one_count_as_kept_and_bool_tensors_work():
    print("[mask] byte values / bool", flush=True)
    rng = np.random.default_rng(5)
    roundtrip(rng.choice(np.array([0, 1, 2, 128, 255], dtype=np.uint8), size=100_003))
    roundtrip(np.zeros(5000, dtype=np.uint8))
    roundtrip(np.ones(5000, dtype=np.uint8))
    n = 70_001
    keep = torch.rand(n, device="cuda") < 0.9  # torch.bool: what a framework hands over
    bits = torch.empty(adacc.mask_packed_bytes(n), dtype=torch.uint8, device="cuda")
    adacc.mask_pack(keep, bits)
    assert np.array_equal(bits.cpu().numpy(), oracle.mask_pack(keep.cpu().numpy()))
    back = torch.empty(n, dtype=torch.bool, device="cuda")
    adacc.mask_unpack(bits, back)
    assert torch.equal(back, keep)


def test_mask_of_an_attention_layer_full_size():
    """[4, 32, 2048, 2048] mask bytes (the C4 shape), the launch the bench times; packed bits compared
    with the oracle in full."""
    print("[mask] full size", flush=True)
    n = 4 * 32 * 2048 * 2048
    g = torch.Generator(device="cuda").manual_seed(77)
    keep = (torch.rand(n, device="cuda", generator=g) < 0.9).to(torch.uint8)
    bits = torch.empty(adacc.mask_packed_bytes(n), dtype=torch.uint8, device="cuda")
    adacc.mask_pack(keep, bits)
    assert np.array_equal(bits.cpu().numpy(), oracle.mask_pack(keep.cpu().numpy()))
    back = torch.empty(n, dtype=torch.uint8, device="cuda")
    adacc.mask_unpack(bits, back)
    assert torch.equal(back, keep)
