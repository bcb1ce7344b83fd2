"""A real forward / backward pass with saved activations compressed by libadacc (Fig. 3(c): compress
in the forward pass, decompress in the backward pass), and the per-tensor figures of Section 3.3.
What the backward pass receives must be the oracle's reconstruction of what the forward pass saved,
bit for bit; the gradients are then those of the same graph fed with that reconstruction."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_00806_amd as adacc
from paper_2508_00806_amd.hooks import SavedActivationCompression
from helpers import bits_of, from_bits

pytestmark = pytest.mark.gpu


def oracle_roundtrip(x_cpu_bf16, method):
    xb = bits_of(x_cpu_bf16)
    if isinstance(method, adacc.ChannelMethod):
        tokens, hidden = x_cpu_bf16.numel() // x_cpu_bf16.shape[-1], x_cpu_bf16.shape[-1]
        om = oracle.Method(bits=method.bits, quant_group=method.quant_group, asym=method.asym)
        c = oracle.channel_compress(om, xb, tokens, hidden, method.z_thresh, cap=method.max_channels)
        return from_bits(oracle.channel_decompress(c)[1]).view(x_cpu_bf16.shape), c.n_ch
    om = oracle.Method(bits=method.bits, quant_group=method.quant_group, asym=method.asym,
                       outlier_mode=method.outlier_mode, stat_group=method.stat_group, thresh=method.thresh,
                       topk=method.topk)
    c = oracle.compress(om, xb, cap=method.max_outliers)
    return from_bits(oracle.decompress(c)[1]).view(x_cpu_bf16.shape), c.n_out


@pytest.mark.parametrize("kind", ["topk", "channel"])
def test_linear_layer_backward_uses_the_reconstruction(kind):
    print(f"[hooks] linear layer, {kind}", flush=True)
    torch.manual_seed(3)
    tokens, hidden, out = 96, 2048, 256
    x = torch.randn(tokens, hidden)
    x[:, [7, 900]] *= 40.0
    x = x.to(torch.bfloat16).cuda()
    w = (torch.randn(out, hidden) * 0.02).to(torch.bfloat16).cuda().requires_grad_(True)
    g = torch.randn(tokens, out).to(torch.bfloat16).cuda()
    if kind == "topk":
        m = adacc.Method(bits=4, quant_group=128, outlier_mode=adacc.OUTLIER_TOPK, stat_group=2048, topk=2,
                         max_outliers=2 * tokens)
    else:
        m = adacc.ChannelMethod(bits=4, quant_group=128, z_thresh=3.0, max_channels=16)
    ctx = SavedActivationCompression(lambda t: m if t.shape == x.shape else None)
    with ctx:
        y = torch.nn.functional.linear(x, w)
    y.backward(g)
    xhat, n_out = oracle_roundtrip(x.cpu(), m)
    want = g.t().float() @ xhat.cuda().float()          # dL/dW of y = x W^T with x replaced by its reconstruction
    got = w.grad.float()
    assert torch.allclose(got, want, rtol=2e-2, atol=2e-2 * float(want.abs().max()))
    exact = g.t().float() @ x.float()
    assert not torch.equal(got, exact.to(torch.bfloat16).float())  # the compressed activation really was used
    rep = ctx.report()
    assert len(rep) == 1 and rep[0]["shape"] == (tokens, hidden) and rep[0]["n_outliers"] == n_out
    assert not rep[0]["overflow"] and rep[0]["tc_ms"] > 0 and rep[0]["tdc_ms"] > 0
    n = tokens * hidden
    if kind == "topk":
        assert rep[0]["compressed_bytes"] == n // 2 + 4 * n // 128 + 6 * n_out + 4 * (tokens + 1)
    else:
        assert n_out == 2 and rep[0]["compressed_bytes"] == n // 2 + 4 * n // 128 + n_out * (2 * tokens + 4)
    assert abs(rep[0]["crate"] - rep[0]["compressed_bytes"] / (2 * n)) < 1e-12 and rep[0]["crate"] < 0.3


def test_unpacked_activation_is_the_oracle_reconstruction_bit_for_bit():
    """The hooks themselves, without autograd in between."""
    print("[hooks] pack / unpack", flush=True)
    torch.manual_seed(4)
    x = (torch.randn(64, 1024) * 1.5).to(torch.bfloat16)
    for m in (adacc.Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_STD, stat_group=64, thresh=3.0,
                           max_outliers=4096),
              adacc.Method(bits=4, quant_group=128),
              adacc.ChannelMethod(bits=8, quant_group=64, z_thresh=2.5, max_channels=64)):
        ctx = SavedActivationCompression(lambda t: m, timing=False)
        saved = ctx._pack(x.cuda())
        back = ctx._unpack(saved)
        want, _ = oracle_roundtrip(x, m)
        assert np.array_equal(bits_of(back), bits_of(want))
    # not offered to the policy: other dtypes, parameters, CPU tensors
    ctx = SavedActivationCompression(lambda t: pytest.fail("policy asked for an ineligible tensor"))
    for t in (torch.randn(8, 8).cuda(), torch.nn.Parameter(x.cuda()), x):
        assert ctx._pack(t) is t


def test_mlp_trains_one_step_with_compressed_activations():
    """Two linear layers and a GELU under the hooks: every saved bf16 activation goes through the
    library, the loss gradient stays close to the one of the uncompressed graph."""
    print("[hooks] mlp", flush=True)
    torch.manual_seed(5)
    mlp = torch.nn.Sequential(torch.nn.Linear(512, 2048), torch.nn.GELU(), torch.nn.Linear(2048, 512)).cuda().to(torch.bfloat16)
    x = torch.randn(128, 512).to(torch.bfloat16).cuda()
    ref = _grads(mlp, x, None)
    m8 = lambda t: adacc.Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_STD, stat_group=64, thresh=6.0,
                                max_outliers=t.numel() // 64)
    ctx = SavedActivationCompression(m8)
    got = _grads(mlp, x, ctx)
    rep = ctx.report()
    assert len(rep) >= 3 and all(0.5 < r["crate"] < 0.6 for r in rep)  # int8 + one scale per 64: 0.53
    for a, b in zip(got, ref):
        assert torch.isfinite(a).all()
        rel = (a.float() - b.float()).norm() / b.float().norm()
        assert rel < 0.05, float(rel)


def test_llama_shaped_mlp_with_whole_rows_as_groups():
    """A gated MLP with LLaMA's ratio of widths (344 = 11008 / 32 is no power of two): the policy keeps the
    4 largest values of every row exactly and gives the rest int8 in groups of 8 - group sizes that run in the
    fallback kernels, forward and backward, under the hooks."""
    print("[hooks] rows as groups", flush=True)
    torch.manual_seed(9)

    class Gated(torch.nn.Module):
        def __init__(self):
            super().__init__()
            self.up = torch.nn.Linear(128, 344)
            self.gate = torch.nn.Linear(128, 344)
            self.down = torch.nn.Linear(344, 128)

        def forward(self, x):
            return self.down(torch.nn.functional.silu(self.gate(x)) * self.up(x))

    mlp = Gated().cuda().to(torch.bfloat16)
    x = torch.randn(96, 128).to(torch.bfloat16).cuda()
    ref = _grads(mlp, x, None)

    def policy(t):
        if t.shape[-1] != 344:
            return None
        return adacc.Method(bits=8, quant_group=8, outlier_mode=adacc.OUTLIER_TOPK, stat_group=344, topk=4,
                            max_outliers=4 * (t.numel() // 344))
    ctx = SavedActivationCompression(policy)
    got = _grads(mlp, x, ctx)
    rep = ctx.report()
    assert len(rep) >= 3 and all(r["n_outliers"] == 4 * 96 and not r["overflow"] for r in rep), rep
    for a, b in zip(got, ref):
        assert torch.isfinite(a).all()
        rel = (a.float() - b.float()).norm() / b.float().norm()
        assert rel < 0.05, float(rel)


def _grads(model, x, ctx):
    """Detached copies of the parameter gradients of one forward / backward pass."""
    for p in model.parameters():
        p.grad = None
    if ctx is None:
        loss = model(x).float().pow(2).mean()
    else:
        with ctx:
            loss = model(x).float().pow(2).mean()
    loss.backward()
    return [p.grad.detach().clone() for p in model.parameters()]


def test_dropout_mask_is_saved_in_bit_format_without_loss():
    """Section 3.2: the dropout mask goes from byte format to bit format; the gradient is exactly the
    one of the unhooked graph, because nothing is lost."""
    print("[hooks] dropout mask", flush=True)
    x = torch.randn(64, 4096, device="cuda", dtype=torch.bfloat16).requires_grad_(True)
    torch.manual_seed(11)
    y = torch.nn.functional.dropout(x, 0.1, training=True)
    y.float().sum().backward()
    ref = x.grad.clone()
    x.grad = None
    ctx = SavedActivationCompression(lambda t: None)
    torch.manual_seed(11)
    with ctx:
        y = torch.nn.functional.dropout(x, 0.1, training=True)
    y.float().sum().backward()
    assert torch.equal(x.grad, ref)
    rep = ctx.report()
    masks = [r for r in rep if r["original_bytes"] == r["numel"]]
    assert len(masks) == 1 and masks[0]["shape"] == (64, 4096) and masks[0]["crate"] == 0.125
    # the hook's own round trip, against the oracle
    keep = torch.rand(1000, 37, device="cuda") < 0.9
    saved = ctx._pack(keep)
    assert np.array_equal(saved.bits.cpu().numpy(), oracle.mask_pack(keep.cpu().numpy()))
    assert torch.equal(ctx._unpack(saved), keep)


def linear_case(tokens=96, hidden=2048, out=64, seed=11):
    torch.manual_seed(seed)
    x = torch.randn(tokens, hidden)
    x[:, [7, 900]] *= 40.0
    x = x.to(torch.bfloat16).cuda()
    w = (torch.randn(out, hidden) * 0.02).to(torch.bfloat16).cuda().requires_grad_(True)
    g = torch.randn(tokens, out).to(torch.bfloat16).cuda()
    return x, w, g


@pytest.mark.parametrize("kind", ["abs", "channel"])
def test_a_blob_that_overflowed_stops_the_backward_pass(kind):
    """More outliers than the method has room for (Section 3.4: the number of outliers moves while
    training): the blob does not hold the tensor, and the backward pass must say so instead of
    handing a wrong activation to the gradient."""
    from paper_2508_00806_amd.hooks import CompressedActivationLost
    print(f"[hooks] overflow raises, {kind}", flush=True)
    x, w, g = linear_case()
    if kind == "abs":
        m = adacc.Method(bits=8, quant_group=128, outlier_mode=adacc.OUTLIER_ABS, thresh=3.0, max_outliers=8)
    else:
        m = adacc.ChannelMethod(bits=4, quant_group=128, z_thresh=3.0, max_channels=1)  # two channels stand out
    ctx = SavedActivationCompression(lambda t: m if t.shape == x.shape else None)
    with ctx:
        y = torch.nn.functional.linear(x, w)
    with pytest.raises(CompressedActivationLost):
        y.backward(g)
    rep = ctx.report()
    assert len(rep) == 1 and rep[0]["overflow"] and rep[0]["n_outliers"] > (8 if kind == "abs" else 1)


@pytest.mark.parametrize("kind", ["abs", "channel"])
def test_a_blob_that_overflowed_can_fall_back_to_the_tensor(kind):
    print(f"[hooks] overflow retains, {kind}", flush=True)
    x, w, g = linear_case()
    if kind == "abs":
        m = adacc.Method(bits=8, quant_group=128, outlier_mode=adacc.OUTLIER_ABS, thresh=3.0, max_outliers=8)
    else:
        m = adacc.ChannelMethod(bits=4, quant_group=128, z_thresh=3.0, max_channels=1)
    ctx = SavedActivationCompression(lambda t: m if t.shape == x.shape else None, on_overflow="retain")
    with ctx:
        y = torch.nn.functional.linear(x, w)
    y.backward(g)
    w2 = w.detach().clone().requires_grad_(True)
    torch.nn.functional.linear(x, w2).backward(g)
    assert torch.equal(w.grad, w2.grad)  # the activation itself was used
    rep = ctx.report()
    assert len(rep) == 1 and rep[0]["overflow"] and rep[0]["crate"] == 1.0 and rep[0]["tdc_ms"] is None


def test_tensors_the_library_does_not_take_are_saved_as_they_are():
    """A contiguous view at an address that is not a multiple of 16 bytes, and (outlier channels) a size
    the groups do not divide: no error in the forward pass, the tensor is retained."""
    print("[hooks] misaligned and indivisible tensors", flush=True)
    for tokens, hidden, offset, m in (
            (32, 256, 1, adacc.Method(bits=8, quant_group=64, outlier_mode=adacc.OUTLIER_STD, stat_group=64, thresh=6.0,
                                      max_outliers=4096)),
            (30, 104, 0, adacc.ChannelMethod(bits=4, quant_group=128, max_channels=8))):
        torch.manual_seed(5)
        buf = torch.randn(tokens * hidden + 8).to(torch.bfloat16).cuda()
        x = buf[offset:offset + tokens * hidden].view(tokens, hidden)
        assert x.is_contiguous() and (offset == 0 or x.data_ptr() % 16 != 0)
        w = (torch.randn(16, hidden) * 0.1).to(torch.bfloat16).cuda().requires_grad_(True)
        g = torch.randn(tokens, 16).to(torch.bfloat16).cuda()
        ctx = SavedActivationCompression(lambda t: m if t.shape == x.shape else None)
        with ctx:
            y = torch.nn.functional.linear(x, w)
        y.backward(g)
        w2 = w.detach().clone().requires_grad_(True)
        torch.nn.functional.linear(x, w2).backward(g)
        assert torch.equal(w.grad, w2.grad)
        assert ctx.report() == []
        assert (len(ctx.retained) == 1) == (offset == 0)  # the indivisible size was offered and turned down


def test_float16_activations_are_compressed_in_their_own_format():
    """The paper's own setting: an FP16 activation saved as INT4 with its outlier channels kept."""
    print("[hooks] float16", flush=True)
    torch.manual_seed(21)
    tokens, hidden, out = 96, 2048, 64
    x = torch.randn(tokens, hidden)
    x[:, [7, 900]] *= 40.0
    x = x.to(torch.float16).cuda()
    w = (torch.randn(out, hidden) * 0.02).to(torch.float16).cuda().requires_grad_(True)
    g = torch.randn(tokens, out).to(torch.float16).cuda()
    for m in (adacc.ChannelMethod(bits=4, quant_group=128, z_thresh=3.0, max_channels=16),
              adacc.Method(bits=4, quant_group=128, outlier_mode=adacc.OUTLIER_TOPK, stat_group=2048, topk=2,
                           max_outliers=2 * tokens)):
        w.grad = None
        ctx = SavedActivationCompression(lambda t: m if t.shape == x.shape else None)
        with ctx:
            y = torch.nn.functional.linear(x, w)
        y.backward(g)
        xb = bits_of(x)
        if isinstance(m, adacc.ChannelMethod):
            om = oracle.Method(bits=4, quant_group=128, dtype=oracle.DT_F16)
            c = oracle.channel_compress(om, xb, tokens, hidden, 3.0, cap=16)
            xhat = from_bits(oracle.channel_decompress(c)[1], dtype=torch.float16).view(tokens, hidden)
        else:
            om = oracle.Method(bits=4, quant_group=128, outlier_mode=oracle.OUT_TOPK, stat_group=2048, topk=2,
                               dtype=oracle.DT_F16)
            xhat = from_bits(oracle.decompress(oracle.compress(om, xb))[1], dtype=torch.float16).view(tokens, hidden)
        want = g.t().float() @ xhat.cuda().float()
        assert torch.allclose(w.grad.float(), want, rtol=2e-2, atol=2e-2 * float(want.abs().max()))
        rep = ctx.report()
        assert len(rep) == 1 and not rep[0]["overflow"] and rep[0]["crate"] < 0.3
