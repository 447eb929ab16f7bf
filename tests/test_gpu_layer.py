"""GPU: the TV layer (SoftPlus lambda, per-channel / shared, rows / columns / 2D, sharpening)
through torch autograd, against the oracle."""
import numpy as np
import pytest

import oracle
from gpuutil import lam_per_row, rows_view
from parity import check_batch

pytestmark = pytest.mark.gpu


def _softplus(v):
    return np.log1p(np.exp(v))


def _sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def _run_layer(layer, x, g):
    import torch
    xt = torch.from_numpy(x).cuda().requires_grad_(True)
    y = layer(xt)
    y.backward(torch.from_numpy(g).cuda())
    torch.cuda.synchronize()
    return y.detach().cpu().numpy(), xt.grad.cpu().numpy(), layer.raw_lambda.grad.cpu().numpy()


@pytest.mark.parametrize("mode,axis", [("rows", -1), ("cols", -2)])
def test_layer_1d_modes(mode, axis):
    import torch
    from paper_2204_03643_amd.layer import TVLayer
    rng = np.random.default_rng(81 + (axis == -2))
    B, C, H, W = 3, 5, 16, 32
    x = rng.normal(size=(B, C, H, W)).astype(np.float32)
    g = rng.normal(size=x.shape).astype(np.float32)
    raw = rng.uniform(-3.0, 1.0, size=C).astype(np.float32)
    out = {}
    for sharpen in (False, True):
        layer = TVLayer(C, mode=mode, sharpen=sharpen).cuda()
        with torch.no_grad():
            layer.raw_lambda.copy_(torch.from_numpy(raw))
        out[sharpen] = _run_layer(layer, x, g)
    # smoothing: prox, its gradient, and dL/dlam = dL/draw / SoftPlus'(raw) against the oracle
    y, gx, graw = out[False]
    lam = _softplus(raw.astype(np.float64))
    div = H if mode == "rows" else W
    xr, gr = rows_view(x, axis), rows_view(g, axis)
    lr = lam_per_row(lam, len(xr), div)
    gl = graw.astype(np.float64) / _sigmoid(raw.astype(np.float64))
    check_batch(xr, lr, gr, rows_view(y, axis), rows_view(gx, axis), gl_gpu=gl.astype(np.float32),
                lam_count=C, lam_div=div, label="layer %s" % mode)
    # sharpening is 2x - prox on the same kernels: the outputs and gradients must be those
    ys, gxs, graws = out[True]
    np.testing.assert_array_equal(ys, 2.0 * x - y)
    np.testing.assert_allclose(gxs, 2.0 * g - gx, rtol=0, atol=1e-6 * np.abs(g).max())
    np.testing.assert_allclose(graws, -graw, rtol=1e-6, atol=1e-7)


def test_layer_2d_shared_lambda_and_identity_limit():
    import torch
    from paper_2204_03643_amd.layer import TVLayer
    rng = np.random.default_rng(85)
    B, C, H, W = 2, 3, 32, 32
    x = rng.normal(size=(B, C, H, W)).astype(np.float32)
    g = rng.normal(size=x.shape).astype(np.float32)
    layer = TVLayer(C, mode="2d", shared_lambda=True, sweeps=3, init_lambda=0.3).cuda()
    assert abs(float(layer.lambdas().detach()[0]) - 0.3) < 1e-6
    y, gx, graw = _run_layer(layer, x, g)
    x_ref, saved = oracle.prox2d_fwd(x.astype(np.float64), np.array([0.3]), 3)
    assert np.abs(y - x_ref).max() <= 1e-4 * (1 + np.abs(x).max())
    gy_ref, gl_ref = oracle.prox2d_bwd(g.astype(np.float64), saved, 1, 3)
    close = np.abs(gx - gy_ref) <= 1e-3 * np.abs(gy_ref).max()
    assert close.mean() >= 0.9
    raw = float(layer.raw_lambda[0])
    assert abs(graw[0] / _sigmoid(raw) - gl_ref[0]) <= 0.05 * (abs(gl_ref[0]) + np.sqrt(x.size))
    # SoftPlus of a very negative parameter is ~0: smoothing and sharpening are both the identity
    for sharpen in (False, True):
        ident = TVLayer(C, mode="2d", sharpen=sharpen).cuda()
        with torch.no_grad():
            ident.raw_lambda.fill_(-40.0)
        y2, gx2, _ = _run_layer(ident, x, g)
        np.testing.assert_allclose(y2, x, atol=1e-6)
        np.testing.assert_allclose(gx2, g, atol=1e-6)


def test_lambda_of_any_shape_and_a_second_backward():
    """lambda handed over as [C, 1, 1]: its gradient comes back in that shape (1D and 2D), and the
    2D reverse sweep may run twice on one graph (it only reads what the forward pass saved)."""
    import torch

    from paper_2204_03643_amd.layer import tv_prox_1d, tv_prox_2d

    rng = np.random.default_rng(31)
    x = torch.from_numpy(rng.normal(size=(2, 3, 20, 24)).astype(np.float32)).cuda().requires_grad_(True)
    g = torch.from_numpy(rng.normal(size=(2, 3, 20, 24)).astype(np.float32)).cuda()
    lam = torch.tensor([0.2, 0.5, 1.0], device="cuda").reshape(3, 1, 1).requires_grad_(True)
    y = tv_prox_1d(x, lam, axis=-1, lam_div=20)
    gx, gl = torch.autograd.grad(y, (x, lam), g)
    assert gl.shape == (3, 1, 1)
    lam_flat = lam.detach().reshape(3).requires_grad_(True)
    gx2, gl2 = torch.autograd.grad(tv_prox_1d(x, lam_flat, axis=-1, lam_div=20), (x, lam_flat), g)
    assert torch.equal(gx, gx2) and torch.equal(gl.reshape(3), gl2)
    y = tv_prox_2d(x, lam, 3)
    gx, gl = torch.autograd.grad(y, (x, lam), g, retain_graph=True)
    assert gl.shape == (3, 1, 1)
    gx_again, gl_again = torch.autograd.grad(y, (x, lam), g)
    assert torch.equal(gx, gx_again) and torch.equal(gl, gl_again)


def test_bf16_feature_maps_through_the_layer():
    """bf16 feature maps (32 x 32, lambda fp32): the layer's 2D and row modes run on the library's
    bf16-storage kernels; outputs and input gradients are bf16 and equal the fp32 layer's on the
    same (widened) tensors up to bf16 rounding, the lambda gradient up to fp32 rounding order."""
    import torch

    from paper_2204_03643_amd.layer import TVLayer

    rng = np.random.default_rng(77)
    x32 = torch.from_numpy(rng.normal(size=(3, 4, 32, 32)).astype(np.float32)).cuda()
    g32 = torch.from_numpy(rng.normal(size=(3, 4, 32, 32)).astype(np.float32)).cuda()
    xb, gb = x32.to(torch.bfloat16), g32.to(torch.bfloat16)
    for mode in ("2d", "rows"):
        layer = TVLayer(4, mode=mode, sweeps=3).cuda()
        a = xb.clone().requires_grad_(True)
        ya = layer(a)
        assert ya.dtype == torch.bfloat16
        ga, gla = torch.autograd.grad(ya, (a, layer.raw_lambda), gb)
        assert ga.dtype == torch.bfloat16
        b = xb.float().requires_grad_(True)
        yb = layer(b)
        gbx, glb = torch.autograd.grad(yb, (b, layer.raw_lambda), gb.float())
        assert float((ya.float() - yb).abs().max()) <= 2.0 ** -7 * float(yb.abs().max())
        assert float((ga.float() - gbx).abs().max()) <= 2.0 ** -7 * float(gbx.abs().max())
        assert torch.allclose(gla, glb, rtol=1e-3, atol=1e-3)
    with pytest.raises(TypeError):
        TVLayer(4, mode="cols").cuda()(xb)
