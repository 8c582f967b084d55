"""The autograd wrapper (paper_2505_14669_amd.nn) against the oracle, and a short training run.

The wrapper adds no arithmetic: its outputs must be the library's, i.e. the oracle's linear_fwd /
linear_bwd rounded to bf16, and a model built from it must train (Section 3: the backward pass is an
unbiased estimate of the gradient of the quantized forward pass)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_14669_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qnn():
    from paper_2505_14669_amd import nn as qnn
    return qnn


def _bf16_tensor(u16):
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).to("cuda:0")


def _to_f32(t):
    return t.detach().float().cpu().numpy()


def test_autograd_function_matches_oracle(qnn):
    x = synth.small_matrix(11, 96, 160, "heavy")
    w = synth.small_matrix(12, 224, 160, "normal", 0.02)
    dy = synth.small_matrix(13, 96, 224, "normal", 1e-3)
    seed = 2 ** 40 + 5
    xt = _bf16_tensor(x).requires_grad_(True)
    wt = _bf16_tensor(w).requires_grad_(True)
    y = qnn.QuartetLinearFunction.apply(xt, wt, seed, 0)
    y.backward(_bf16_tensor(dy))
    y_ref, ctx = oracle.linear_fwd(x, w)
    dx_ref, dw_ref = oracle.linear_bwd(dy, ctx, seed, 0)

    def bf16_close(got, want):
        # the library rounds its fp32 result to bf16 once; the oracle's fp64 sum rounded the same way may fall on
        # the neighbouring bf16 value when the two differ by 1e-5 relative: allow one bf16 step (2^-8 relative)
        # on a few elements, none further
        got, want = _to_f32(got), synth.bf16_to_f32(synth.f32_to_bf16(want.astype(np.float32)))
        err = np.abs(got - want)
        assert np.all(err <= np.abs(want) * 2.0 ** -7 + 1e-30)
        assert np.mean(err > 0) < 0.02

    bf16_close(y, y_ref)
    bf16_close(xt.grad, dx_ref)
    bf16_close(wt.grad, dw_ref)


def test_leading_dimensions_are_flattened(qnn):
    lin = qnn.QuartetLinear(64, 96, bias=True, seed=3)
    x = torch.randn(2, 16, 64, device="cuda:0").to(torch.bfloat16).requires_grad_(True)
    y = lin(x)
    assert y.shape == (2, 16, 96) and y.dtype == torch.bfloat16
    y.float().square().mean().backward()
    assert x.grad.shape == x.shape and lin.weight.grad.shape == lin.weight.shape and lin.bias.grad.shape == (96,)
    with pytest.raises(ValueError):
        lin(torch.randn(5, 64, device="cuda:0").to(torch.bfloat16))       # 5 tokens: not a multiple of 32


def _train(qnn, quantized, steps=150, lr=0.2):
    # regression onto a fixed random teacher; fp32 master weights, bf16 copies fed to the layers
    torch.manual_seed(0)
    d_in, d_hid, d_out, batch = 128, 256, 64, 512
    teacher1 = torch.randn(d_hid, d_in, device="cuda:0") / d_in ** 0.5
    teacher2 = torch.randn(d_out, d_hid, device="cuda:0") / d_hid ** 0.5
    w1 = (torch.randn(d_hid, d_in, device="cuda:0") / d_in ** 0.5).requires_grad_(True)
    w2 = (torch.randn(d_out, d_hid, device="cuda:0") / d_hid ** 0.5).requires_grad_(True)
    opt = torch.optim.SGD([w1, w2], lr=lr)
    losses = []
    for step in range(steps):
        x = torch.randn(batch, d_in, device="cuda:0")
        target = torch.relu(x @ teacher1.T) @ teacher2.T
        xb, w1b, w2b = x.to(torch.bfloat16), w1.to(torch.bfloat16), w2.to(torch.bfloat16)
        if quantized:
            h = torch.relu(qnn.QuartetLinearFunction.apply(xb, w1b, 2 * step, 0))
            out = qnn.QuartetLinearFunction.apply(h, w2b, 2 * step + 1, 0)
        else:
            out = torch.relu(xb @ w1b.T) @ w2b.T
        loss = (out.float() - target).square().mean()
        opt.zero_grad()
        loss.backward()
        opt.step()
        losses.append(loss.item())
    return float(np.mean(losses[:5])), float(np.mean(losses[-10:]))


def test_two_layer_mlp_trains_like_bf16(qnn):
    # Section 3's claim in miniature: with the unbiased backward pass the MXFP4 layers follow the bf16 run
    first_q, last_q = _train(qnn, True)
    first_b, last_b = _train(qnn, False)
    assert np.isfinite(last_q) and last_q < 0.5 * first_q, (first_q, last_q)
    assert last_q < 1.15 * last_b, (last_q, last_b)
