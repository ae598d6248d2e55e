"""Pins for the oracle's elementary operations (CPU only).

Each operation is checked against something that is not the oracle itself: a
library routine with autograd (torch.nn.functional in float64), scipy, a closed
form, a brute-force loop on a tiny input, or an invariant of the mathematics.
"""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch
import torch.nn.functional as F

from oracle import ppll_oracle as O

RNG = np.random.default_rng(7)
T64 = dict(dtype=torch.float64)


def t(a, grad=False):
    x = torch.tensor(np.asarray(a), **T64)
    x.requires_grad_(grad)
    return x


def close(a, b, tol=1e-10):
    a = np.asarray(a, dtype=np.float64)
    b = b.detach().numpy() if isinstance(b, torch.Tensor) else np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    scale = max(1.0, np.abs(b).max())
    assert np.abs(a - b).max() <= tol * scale, np.abs(a - b).max()


# ---------------------------------------------------------------- linear
def test_linear_matches_torch_autograd():
    x, w, b = RNG.standard_normal((3, 5, 7)), RNG.standard_normal((7, 4)), RNG.standard_normal(4)
    dy = RNG.standard_normal((3, 5, 4))
    tx, tw, tb = t(x, True), t(w, True), t(b, True)
    ty = F.linear(tx, tw.T, tb)
    ty.backward(t(dy))
    close(O.linear_fwd(x, w, b), ty)
    dx, dw, db = O.linear_bwd(dy, x, w)
    close(dx, tx.grad); close(dw, tw.grad); close(db, tb.grad)


def test_linear_adjoint_identity():
    x, w = RNG.standard_normal((6, 7)), RNG.standard_normal((7, 4))
    y = RNG.standard_normal((6, 4))
    dx, _, _ = O.linear_bwd(y, x, w)
    assert abs(np.vdot(O.linear_fwd(x, w, 0.0), y) - np.vdot(x, dx)) < 1e-10


# ---------------------------------------------------------------- layernorm
def test_layernorm_matches_torch_autograd():
    x, g, b = RNG.standard_normal((4, 6, 16)) * 3 + 1, RNG.standard_normal(16), RNG.standard_normal(16)
    dy = RNG.standard_normal((4, 6, 16))
    tx, tg, tb = t(x, True), t(g, True), t(b, True)
    ty = F.layer_norm(tx, (16,), tg, tb, eps=1e-6)
    ty.backward(t(dy))
    y, cache = O.layernorm_fwd(x, g, b, 1e-6)
    close(y, ty)
    dx, dg, db = O.layernorm_bwd(dy, cache, g)
    close(dx, tx.grad); close(dg, tg.grad); close(db, tb.grad)


def test_layernorm_invariants():
    x = RNG.standard_normal((5, 32)) * 2 + 0.5
    y, cache = O.layernorm_fwd(x, np.ones(32), np.zeros(32), 1e-6)
    assert np.abs(y.mean(-1)).max() < 1e-12
    var = x.var(-1)
    np.testing.assert_allclose(y.var(-1), var / (var + 1e-6), rtol=1e-12)
    dx, _, _ = O.layernorm_bwd(RNG.standard_normal((5, 32)), cache, RNG.standard_normal(32))
    assert np.abs(dx.sum(-1)).max() < 1e-12              # rows of dx sum to 0
    # orthogonality to xhat is exact only for eps = 0 (mean(xhat^2) = var/(var+eps))
    _, cache0 = O.layernorm_fwd(x, np.ones(32), np.zeros(32), 0.0)
    dx0, _, _ = O.layernorm_bwd(RNG.standard_normal((5, 32)), cache0, RNG.standard_normal(32))
    assert np.abs((dx0 * cache0[0]).sum(-1)).max() < 1e-12


# ---------------------------------------------------------------- gelu
def test_gelu_matches_normal_cdf_and_torch():
    h = np.linspace(-6, 6, 241)
    close(O.gelu_fwd(h), h * scipy.stats.norm.cdf(h), 1e-13)
    th = t(h, True)
    tg = F.gelu(th)           # exact (erf) form
    dg = RNG.standard_normal(h.shape)
    tg.backward(t(dg))
    close(O.gelu_fwd(h), tg, 1e-13)
    close(O.gelu_bwd(dg, h), th.grad, 1e-12)


def test_gelu_closed_forms():
    assert O.gelu_fwd(np.array([0.0]))[0] == 0.0
    assert O.gelu_bwd(np.array([1.0]), np.array([0.0]))[0] == 0.5
    assert abs(O.gelu_fwd(np.array([30.0]))[0] - 30.0) < 1e-12
    assert abs(O.gelu_fwd(np.array([-30.0]))[0]) < 1e-12


# ---------------------------------------------------------------- softmax / CE
def test_softmax_matches_scipy_and_sums_to_one():
    s = RNG.standard_normal((3, 4, 9)) * 5
    p = O.softmax_rows(s)
    close(p, scipy.special.softmax(s, axis=-1), 1e-14)
    assert np.abs(p.sum(-1) - 1).max() < 1e-14
    big = np.array([[1000.0, 1001.0, 999.0]])   # max subtraction keeps this finite
    assert np.isfinite(O.softmax_rows(big)).all()


def test_cross_entropy_matches_torch():
    z = RNG.standard_normal((12, 10)) * 3
    y = RNG.integers(0, 10, 12)
    tz = t(z, True)
    tl = F.cross_entropy(tz, torch.tensor(y))
    tl.backward()
    loss, dz = O.cross_entropy(z, y)
    assert abs(loss - tl.item()) < 1e-12
    close(dz, tz.grad, 1e-13)


def test_cross_entropy_uniform_logits_is_ln10():
    y = RNG.integers(0, 10, 16)
    for c in (0.0, 3.7):                      # any constant row is uniform
        loss, dz = O.cross_entropy(np.full((16, 10), c), y)
        assert abs(loss - math.log(10.0)) < 1e-14
        expect = np.full((16, 10), 0.1)
        expect[np.arange(16), y] -= 1.0
        close(dz, expect / 16, 1e-14)
    assert np.abs(dz.sum(-1)).max() < 1e-15


# ---------------------------------------------------------------- attention
def _torch_attention(qkv, heads):
    B, T, D3 = qkv.shape
    D = D3 // 3
    q, k, v = (qkv[:, :, i * D:(i + 1) * D].reshape(B, T, heads, D // heads).transpose(1, 2)
               for i in range(3))
    o = F.scaled_dot_product_attention(q, k, v)       # scale 1/sqrt(dh), softmax over keys
    return o.transpose(1, 2).reshape(B, T, D)


def test_attention_matches_torch_sdpa_autograd():
    B, T, H, dh = 2, 7, 3, 4
    qkv = RNG.standard_normal((B, T, 3 * H * dh))
    dout = RNG.standard_normal((B, T, H * dh))
    tq = t(qkv, True)
    to = _torch_attention(tq, H)
    to.backward(t(dout))
    out, cache = O.attention_fwd(qkv, H)
    close(out, to, 1e-12)
    close(O.attention_bwd(dout, cache), tq.grad, 1e-12)
    p = cache[3]
    assert np.abs(p.sum(-1) - 1).max() < 1e-14


def test_attention_single_token_returns_v():
    qkv = RNG.standard_normal((3, 1, 3 * 8))
    out, _ = O.attention_fwd(qkv, 2)
    close(out, qkv[:, :, 16:], 1e-15)


def test_attention_zero_queries_average_values():
    B, T, D = 2, 6, 8
    qkv = RNG.standard_normal((B, T, 3 * D))
    qkv[:, :, :D] = 0.0                                # uniform attention
    out, _ = O.attention_fwd(qkv, 2)
    close(out, np.broadcast_to(qkv[:, :, 2 * D:].mean(axis=1, keepdims=True), (B, T, D)), 1e-14)


def test_attention_ds_rows_sum_to_zero():
    qkv = RNG.standard_normal((1, 5, 3 * 4))
    out, cache = O.attention_fwd(qkv, 1)
    q, k, v, p, scale = cache
    do = RNG.standard_normal((1, 1, 5, 4))
    dp = do @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(-1, keepdims=True))
    assert np.abs(ds.sum(-1)).max() < 1e-14


# ---------------------------------------------------------------- patchify
def test_patchify_brute_force():
    B, H, W, C, P = 2, 8, 12, 3, 4
    img = RNG.standard_normal((B, H, W, C))
    pt = O.patchify(img, P)
    assert pt.shape == (B, (H // P) * (W // P), P * P * C)
    for b in range(B):
        for gy in range(H // P):
            for gx in range(W // P):
                for r in range(P):
                    for c in range(P):
                        for ch in range(C):
                            assert pt[b, gy * (W // P) + gx, (r * P + c) * C + ch] == \
                                img[b, gy * P + r, gx * P + c, ch]


# ---------------------------------------------------------------- conv3x3
def _torch_conv(x, w, stride):
    # NHWC / [ky,kx,ci,co] -> NCHW / [co,ci,ky,kx]
    y = F.conv2d(x.permute(0, 3, 1, 2), w.permute(3, 2, 0, 1), stride=stride, padding=1)
    return y.permute(0, 2, 3, 1)


@pytest.mark.parametrize("stride,hw", [(1, (6, 5)), (2, (6, 6)), (2, (7, 5))])
def test_conv3x3_matches_torch_autograd(stride, hw):
    B, Ci, Co = 2, 3, 4
    x = RNG.standard_normal((B, *hw, Ci))
    w = RNG.standard_normal((3, 3, Ci, Co))
    tx, tw = t(x, True), t(w, True)
    ty = _torch_conv(tx, tw, stride)
    dy = RNG.standard_normal(tuple(ty.shape))
    ty.backward(t(dy))
    close(O.conv3x3_fwd(x, w, stride), ty, 1e-12)
    close(O.conv3x3_bwd_weight(dy, x, stride), tw.grad, 1e-12)
    close(O.conv3x3_bwd_input(dy, w, stride, x.shape), tx.grad, 1e-12)


@pytest.mark.parametrize("stride", [1, 2])
def test_conv3x3_brute_force(stride):
    B, H, W, Ci, Co = 1, 4, 5, 2, 3
    x = RNG.standard_normal((B, H, W, Ci))
    w = RNG.standard_normal((3, 3, Ci, Co))
    y = O.conv3x3_fwd(x, w, stride)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    assert y.shape == (B, Ho, Wo, Co)
    for oy in range(Ho):
        for ox in range(Wo):
            for co in range(Co):
                acc = 0.0
                for ky in range(3):
                    for kx in range(3):
                        iy, ix = oy * stride + ky - 1, ox * stride + kx - 1
                        if 0 <= iy < H and 0 <= ix < W:
                            for ci in range(Ci):
                                acc += x[0, iy, ix, ci] * w[ky, kx, ci, co]
                assert abs(y[0, oy, ox, co] - acc) < 1e-12


def test_conv3x3_centre_tap_is_identity_and_adjoint():
    x = RNG.standard_normal((2, 5, 5, 3))
    w = np.zeros((3, 3, 3, 3))
    w[1, 1] = np.eye(3)
    close(O.conv3x3_fwd(x, w, 1), x, 1e-15)
    for stride in (1, 2):
        w = RNG.standard_normal((3, 3, 3, 4))
        y = O.conv3x3_fwd(x, w, stride)
        dy = RNG.standard_normal(y.shape)
        lhs = np.vdot(y, dy)
        assert abs(lhs - np.vdot(x, O.conv3x3_bwd_input(dy, w, stride, x.shape))) < 1e-10
        assert abs(lhs - np.vdot(w, O.conv3x3_bwd_weight(dy, x, stride))) < 1e-10


# ---------------------------------------------------------------- parameter-free shortcut
def test_shortcut_is_identity_or_subsample_with_zero_channels():
    x = RNG.standard_normal((2, 6, 5, 3))
    assert O.shortcut_fwd(x, 3, 1) is x
    y = O.shortcut_fwd(x, 6, 2)
    assert y.shape == (2, 3, 3, 6)
    for b in range(2):
        for oy in range(3):
            for ox in range(3):
                for c in range(6):
                    assert y[b, oy, ox, c] == (x[b, 2 * oy, 2 * ox, c] if c < 3 else 0.0)
    # 1x1 stride-2 convolution with the [I | 0] matrix is the same map
    w = torch.zeros(6, 3, 1, 1, dtype=torch.float64)
    w[:3, :, 0, 0] = torch.eye(3, dtype=torch.float64)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), w, stride=2).permute(0, 2, 3, 1).numpy()
    close(y, ref, 1e-15)
    dy = RNG.standard_normal(y.shape)
    assert abs(np.vdot(y, dy) - np.vdot(x, O.shortcut_bwd(dy, x.shape, 2))) < 1e-12
    assert O.shortcut_bwd(dy, y.shape, 1) is dy


# ---------------------------------------------------------------- batchnorm
def test_batchnorm_matches_torch_autograd_and_invariants():
    x = RNG.standard_normal((3, 4, 5, 6)) * 2 + 1
    g, b = RNG.standard_normal(6), RNG.standard_normal(6)
    dy = RNG.standard_normal(x.shape)
    tx, tg, tb = t(x, True), t(g, True), t(b, True)
    ty = F.batch_norm(tx.permute(0, 3, 1, 2), None, None, tg, tb, training=True, eps=1e-5).permute(0, 2, 3, 1)
    ty.backward(t(dy))
    y, cache = O.batchnorm_fwd(x, g, b, 1e-5)
    close(y, ty, 1e-12)
    dx, dg, db = O.batchnorm_bwd(dy, cache, g)
    close(dx, tx.grad, 1e-12); close(dg, tg.grad, 1e-12); close(db, tb.grad, 1e-12)
    np.testing.assert_allclose(y.mean(axis=(0, 1, 2)), b, atol=1e-12)
    assert np.abs(dx.sum(axis=(0, 1, 2))).max() < 1e-12
    _, cache0 = O.batchnorm_fwd(x, g, b, 0.0)
    dx0, _, _ = O.batchnorm_bwd(dy, cache0, g)
    assert np.abs((dx0 * cache0[0]).sum(axis=(0, 1, 2))).max() < 1e-11


# ---------------------------------------------------------------- optimizers
@pytest.mark.parametrize("momentum,nesterov,wd", [(0.0, False, 0.0), (0.9, False, 1e-2), (0.9, True, 1e-4)])
def test_sgd_matches_torch_optim(momentum, nesterov, wd):
    p0 = RNG.standard_normal(11)
    grads = [RNG.standard_normal(11) for _ in range(4)]
    tp = t(p0, True)
    opt = torch.optim.SGD([tp], lr=0.05, momentum=momentum, nesterov=nesterov, weight_decay=wd)
    p, buf = p0.copy(), np.zeros(11)
    for i, g in enumerate(grads):
        tp.grad = t(g)
        opt.step()
        p, buf = O.sgd_update(p, g, buf, 0.05, momentum, nesterov, wd, i == 0)
        close(p, tp, 1e-13)


def test_adamw_matches_torch_optim():
    p0 = RNG.standard_normal(13)
    tp = t(p0, True)
    opt = torch.optim.AdamW([tp], lr=1e-2, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.05)
    p, m, v = p0.copy(), np.zeros(13), np.zeros(13)
    for i in range(5):
        g = RNG.standard_normal(13)
        tp.grad = t(g)
        opt.step()
        p, m, v = O.adamw_update(p, g, m, v, i + 1, 1e-2, 0.9, 0.999, 1e-8, 0.05)
        close(p, tp, 1e-12)


def test_optimizer_first_step_closed_forms():
    p, g = RNG.standard_normal(9), RNG.standard_normal(9)
    lr, mu, wd = 0.1, 0.9, 1e-4
    q, _ = O.sgd_update(p, g, np.zeros(9), lr, 0.0, False, 0.0, True)
    close(q, p - lr * g, 1e-15)
    q, buf = O.sgd_update(p, g, np.zeros(9), lr, mu, True, wd, True)
    close(q, p - lr * (1 + mu) * (g + wd * p), 1e-14)
    close(buf, g + wd * p, 1e-15)
    q, m, v = O.adamw_update(p, g, np.zeros(9), np.zeros(9), 1, lr, 0.9, 0.999, 1e-8, 0.01)
    close(q, p * (1 - lr * 0.01) - lr * g / (np.abs(g) + 1e-8), 1e-12)


# ---------------------------------------------------------------- bf16 storage emulation
def test_bf16_values_matches_torch_rounding_and_ties_to_even():
    a = (RNG.standard_normal(20000) * np.exp(RNG.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = O.bf16_values(a.astype(np.float64))
    assert np.array_equal(got, want.astype(np.float64))
    # ties: 1 + 2^-8 lies midway between 1 and 1 + 2^-7 -> even (1); 1 + 3*2^-8 -> 1 + 2^-6
    assert O.bf16_values(np.array([1 + 2.0 ** -8]))[0] == 1.0
    assert O.bf16_values(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6
    assert O.bf16_values(np.array([0.0, -0.0, np.inf]))[2] == np.inf
    x = O.bf16_values(RNG.standard_normal(1000))
    assert np.array_equal(O.bf16_values(x), x)            # idempotent
