"""Pins for the oracle's whole local-block step (CPU only).

The step is pinned by (i) central finite differences of the local loss in
float64, (ii) torch.autograd over library ops plus torch.optim for the update,
(iii) closed forms (zero head -> ln 10), (iv) the structural facts of
Algorithm 1: gradient isolation, the output being pre-update, and the
sequential chain that the pipeline must reproduce.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ppll_oracle as O
from paper_2411_12780_amd import synth
from helpers import oracle_cfg, rel_l2

TINY_VIT_IMG = dict(arch=0, input_kind=0, batch=2, num_classes=10, img_h=8, img_w=8, img_c=3,
                    patch=4, tokens=5, dim=8, heads=2, mlp_dim=16, depth=1, aux_depth=1,
                    optimizer=0, ln_eps=1e-6, precision=0)
TINY_VIT_ACT = dict(TINY_VIT_IMG, input_kind=1, depth=2, aux_depth=0)
TINY_RESNET = dict(arch=1, input_kind=1, batch=2, num_classes=10, channels=4, height=6, width=6,
                   n_basic_blocks=2, aux_channels=6, optimizer=0, momentum=0.9, nesterov=1,
                   weight_decay=1e-4, bn_eps=1e-5, bn_momentum=0.1, precision=0)
# basic block 1 of 3 halves the map and doubles the channels: the backward pass crosses its shortcut
TINY_RESNET_DOWN = dict(TINY_RESNET, channels=4, height=4, width=4, n_basic_blocks=3, transition_block=2)
# the network's first module: stem on the image, then basic blocks; the stem is trained, so the
# backward pass also crosses basic block 0
TINY_RESNET_STEM = dict(TINY_RESNET, input_kind=0, img_h=6, img_w=6, img_c=3)
TINY_RESNET_STEM_DOWN = dict(TINY_RESNET, input_kind=0, img_h=6, img_w=6, img_c=3, channels=4, height=3, width=3,
                             transition_block=1)
CASES = {"vit_img": TINY_VIT_IMG, "vit_act": TINY_VIT_ACT, "resnet": TINY_RESNET, "resnet_down": TINY_RESNET_DOWN,
         "resnet_stem": TINY_RESNET_STEM, "resnet_stem_down": TINY_RESNET_STEM_DOWN}


def make(wl, seed=0, dtype=np.float64):
    cfg = oracle_cfg(wl)
    flat = synth.make_params(O.param_spec(cfg), seed=seed, jitter=True).astype(np.float64)
    flat = flat + np.random.default_rng(seed + 99).standard_normal(flat.size) * 0.05  # livelier than the bench init
    st = O.block_init(cfg, flat, dtype)
    x, y = synth.make_batch(wl, seed=seed)
    return cfg, st, x.astype(np.float64), y


# ------------------------------------------------------------------ counts
def test_param_counts_of_the_named_workloads():
    assert O.param_count(oracle_cfg(synth.workload("vit_tiny_fp32"))) == 75082
    assert O.param_count(oracle_cfg(synth.workload("vit_stage_bf16"))) == 7146634
    assert O.param_count(oracle_cfg(synth.workload("vit_stage_act_bf16"))) == 7102474
    assert O.param_count(oracle_cfg(synth.workload("vit_large_image_bf16"))) == 7232650
    assert O.param_count(oracle_cfg(synth.workload("resnet_stage_bf16"))) == 112010


def test_parameter_table_reproduces_the_published_size_of_vit_base_patch16_224():
    # Section 4.1 names ViT-base-patch16-224.  Written as one block (12 encoder layers, no auxiliary layers, the
    # head's LayerNorm as the final norm, a 1000-class Linear head, 224 x 224 images) the parameter table must add
    # up to that model's published 86,567,656 parameters: 7,087,872 per encoder layer, 590,592 patch embedding,
    # 768 class token, 197 x 768 positions, 1,536 final norm, 769,000 classifier.
    cfg = O.BlockConfig(arch=O.ARCH_VIT, input_kind=O.IN_IMAGE, batch=1, num_classes=1000, img_h=224, img_w=224, img_c=3,
                        patch=16, tokens=197, dim=768, heads=12, mlp_dim=3072, depth=12, aux_depth=0)
    assert O.param_count(cfg) == 86567656
    layer = sum(int(np.prod(shape)) for name, shape in O.param_spec(cfg) if name.startswith("blk0."))
    assert layer == 7087872


# ------------------------------------------------------------------ finite differences
@pytest.mark.parametrize("case", list(CASES))
def test_gradients_match_central_finite_differences(case):
    cfg, st, x, y = make(CASES[case])
    O.block_step(st_copy := O.block_init(cfg, O.flatten(cfg, st.params)), x, y, 0.0)
    grads = st_copy.grads
    rng = np.random.default_rng(3)
    h = 1e-5
    for name, shape in O.param_spec(cfg):
        n = int(np.prod(shape))
        for idx in rng.choice(n, size=min(n, 20), replace=False):
            flat = st.params[name].reshape(-1)
            old = flat[idx]
            flat[idx] = old + h
            lp = O.local_loss(st, x, y)
            flat[idx] = old - h
            lm = O.local_loss(st, x, y)
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            an = grads[name].reshape(-1)[idx]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)) + 1e-9, (name, idx, fd, an)


# ------------------------------------------------------------------ torch autograd reference
def _t(a):
    return torch.tensor(np.asarray(a), dtype=torch.float64)


def _torch_encoder(x, p, pre, heads, eps):
    D = x.shape[-1]
    u = F.layer_norm(x, (D,), p[pre + ".ln1.g"], p[pre + ".ln1.b"], eps)
    qkv = F.linear(u, p[pre + ".qkv.w"].T, p[pre + ".qkv.b"])
    B, T, _ = qkv.shape
    q, k, v = (qkv[:, :, i * D:(i + 1) * D].reshape(B, T, heads, D // heads).transpose(1, 2) for i in range(3))
    o = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(B, T, D)
    x = x + F.linear(o, p[pre + ".proj.w"].T, p[pre + ".proj.b"])
    u = F.layer_norm(x, (D,), p[pre + ".ln2.g"], p[pre + ".ln2.b"], eps)
    h = F.gelu(F.linear(u, p[pre + ".fc1.w"].T, p[pre + ".fc1.b"]))
    return x + F.linear(h, p[pre + ".fc2.w"].T, p[pre + ".fc2.b"])


def _torch_vit(cfg, p, x):
    if cfg.input_kind == O.IN_IMAGE:
        P = cfg.patch
        # F.unfold yields (channel, row, col) order per patch; the block uses (row, col, channel)
        cols = F.unfold(x.permute(0, 3, 1, 2), kernel_size=P, stride=P)          # [B, C*P*P, N]
        B, _, N = cols.shape
        pt = cols.reshape(B, cfg.img_c, P, P, N).permute(0, 4, 2, 3, 1).reshape(B, N, P * P * cfg.img_c)
        e = F.linear(pt, p["pe.w"].T, p["pe.b"])
        x = torch.cat([p["cls"].expand(B, 1, -1), e], dim=1) + p["pos"]
    x = x.detach() if cfg.input_kind != O.IN_IMAGE else x
    for l in range(cfg.depth):
        x = _torch_encoder(x, p, f"blk{l}", cfg.heads, cfg.ln_eps)
    x_out = x
    for a in range(cfg.aux_depth):
        x = _torch_encoder(x, p, f"aux{a}", cfg.heads, cfg.ln_eps)
    z = F.layer_norm(x[:, 0, :], (cfg.dim,), p["head.ln.g"], p["head.ln.b"], cfg.ln_eps)
    return x_out, F.linear(z, p["head.w"].T, p["head.b"])


def _torch_conv(x, w, stride):
    return F.conv2d(x.permute(0, 3, 1, 2), w.permute(3, 2, 0, 1), stride=stride, padding=1).permute(0, 2, 3, 1)


def _torch_bn(x, g, b, eps, run):
    y = F.batch_norm(x.permute(0, 3, 1, 2), run[0], run[1], g, b, training=True, momentum=0.1, eps=eps)
    return y.permute(0, 2, 3, 1)


def _torch_resnet(cfg, p, x, run):
    if cfg.input_kind == O.IN_IMAGE:
        x = F.relu(_torch_bn(_torch_conv(x, p["stem.conv.w"], 1), p["stem.bn.g"], p["stem.bn.b"], cfg.bn_eps, run["stem.bn"]))
    for i in range(cfg.n_basic_blocks):
        pre = f"rb{i}"
        down = i == cfg.transition_block - 1
        y = F.relu(_torch_bn(_torch_conv(x, p[pre + ".conv1.w"], 2 if down else 1), p[pre + ".bn1.g"], p[pre + ".bn1.b"],
                             cfg.bn_eps, run[pre + ".bn1"]))
        y = _torch_bn(_torch_conv(y, p[pre + ".conv2.w"], 1), p[pre + ".bn2.g"], p[pre + ".bn2.b"], cfg.bn_eps, run[pre + ".bn2"])
        if down:   # every second pixel, as many zero channels appended as there are channels
            x = F.pad(x[:, ::2, ::2, :], (0, x.shape[-1]))
        x = F.relu(x + y)
    x_out = x
    a = F.relu(_torch_bn(_torch_conv(x, p["aux.conv.w"], 2), p["aux.bn.g"], p["aux.bn.b"], cfg.bn_eps, run["aux.bn"]))
    return x_out, F.linear(a.mean(dim=(1, 2)), p["head.w"].T, p["head.b"])


@pytest.mark.parametrize("case,opt", [("vit_img", "sgd"), ("vit_act", "adamw"), ("vit_img", "adamw"),
                                      ("resnet", "sgd_nesterov"), ("resnet_down", "sgd_nesterov"),
                                      ("resnet_stem", "sgd_nesterov"), ("resnet_stem_down", "sgd_nesterov")])
def test_three_steps_match_torch_autograd_and_optim(case, opt):
    wl = dict(CASES[case])
    if opt == "adamw":
        wl.update(optimizer=1, weight_decay=0.01, beta1=0.9, beta2=0.999, adam_eps=1e-8)
    elif opt == "sgd":
        wl.update(optimizer=0, momentum=0.0, nesterov=0, weight_decay=0.0)
    cfg, st, _, _ = make(wl)
    tp = {k: _t(v).requires_grad_(True) for k, v in st.params.items()}
    run = {n: (torch.zeros(c, dtype=torch.float64), torch.ones(c, dtype=torch.float64)) for n, c in O.bn_stat_spec(cfg)}
    lr = 0.05
    if opt == "adamw":
        topt = torch.optim.AdamW(tp.values(), lr=lr, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    elif opt == "sgd":
        topt = torch.optim.SGD(tp.values(), lr=lr)
    else:
        topt = torch.optim.SGD(tp.values(), lr=lr, momentum=0.9, nesterov=True, weight_decay=1e-4)
    for step in range(3):
        x, y = synth.make_batch(wl, seed=5, index=step)
        tx = _t(x)
        topt.zero_grad()
        if cfg.arch == O.ARCH_VIT:
            t_out, t_logits = _torch_vit(cfg, tp, tx)
        else:
            t_out, t_logits = _torch_resnet(cfg, tp, tx, run)
        t_loss = F.cross_entropy(t_logits, torch.tensor(y, dtype=torch.long))
        t_loss.backward()
        x_out, loss = O.block_step(st, x.astype(np.float64), y, lr)
        assert abs(loss - t_loss.item()) < 1e-10
        assert rel_l2(x_out, t_out.detach().numpy()) < 1e-10
        for name in tp:
            assert rel_l2(st.grads[name], tp[name].grad.numpy()) < 1e-8, (step, name)
        topt.step()
        for name in tp:
            assert rel_l2(st.params[name], tp[name].detach().numpy()) < 1e-10, (step, name)
    for n, _ in O.bn_stat_spec(cfg):
        assert rel_l2(st.bn_mean[n], run[n][0].numpy()) < 1e-10
        assert rel_l2(st.bn_var[n], run[n][1].numpy()) < 1e-10


# ------------------------------------------------------------------ evaluation-mode forward
@pytest.mark.parametrize("case", ["resnet", "resnet_down", "resnet_stem_down"])
def test_eval_forward_matches_torch_eval_mode_after_training_steps(case):
    """ResNet: after two training steps (which move the running statistics) the evaluation forward must
    equal torch's batch_norm(training=False) network on a fresh batch, and must leave the state alone."""
    wl = dict(CASES[case])
    cfg, st, _, _ = make(wl)
    for step in range(2):
        x, y = synth.make_batch(wl, seed=8, index=step)
        O.block_step(st, x.astype(np.float64), y, 0.05)
    before = ({k: v.copy() for k, v in st.params.items()}, {k: v.copy() for k, v in st.bn_mean.items()},
              {k: v.copy() for k, v in st.bn_var.items()})
    x, _ = synth.make_batch(wl, seed=8, index=7)
    x_out, logits = O.block_forward_eval(st, x.astype(np.float64))
    tp = {k: _t(v) for k, v in st.params.items()}

    def bn(t, name):
        y = F.batch_norm(t.permute(0, 3, 1, 2), _t(st.bn_mean[name]), _t(st.bn_var[name]), tp[name + ".g"], tp[name + ".b"],
                         training=False, eps=cfg.bn_eps)
        return y.permute(0, 2, 3, 1)

    t = _t(x.astype(np.float64))
    if cfg.input_kind == O.IN_IMAGE:
        t = F.relu(bn(_torch_conv(t, tp["stem.conv.w"], 1), "stem.bn"))
    for i in range(cfg.n_basic_blocks):
        pre = f"rb{i}"
        down = i == cfg.transition_block - 1
        h = F.relu(bn(_torch_conv(t, tp[pre + ".conv1.w"], 2 if down else 1), pre + ".bn1"))
        if down:
            t = F.pad(t[:, ::2, ::2, :], (0, t.shape[-1]))
        t = F.relu(t + bn(_torch_conv(h, tp[pre + ".conv2.w"], 1), pre + ".bn2"))
    a = F.relu(bn(_torch_conv(t, tp["aux.conv.w"], 2), "aux.bn"))
    t_logits = F.linear(a.mean(dim=(1, 2)), tp["head.w"].T, tp["head.b"])
    assert rel_l2(x_out, t.numpy()) < 1e-12
    assert rel_l2(logits, t_logits.numpy()) < 1e-12
    for k in st.params:
        assert np.array_equal(st.params[k], before[0][k])
    for k in st.bn_mean:
        assert np.array_equal(st.bn_mean[k], before[1][k]) and np.array_equal(st.bn_var[k], before[2][k])


def test_eval_batchnorm_with_the_batchs_own_statistics_is_training_batchnorm():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, 4, 5, 6)); g = rng.standard_normal(6); b = rng.standard_normal(6)
    y_train, (_, _, mu, var) = O.batchnorm_fwd(x, g, b, 1e-5)
    assert rel_l2(O.batchnorm_eval(x, g, b, mu, var, 1e-5), y_train) < 1e-13


@pytest.mark.parametrize("case", ["vit_img", "vit_act"])
def test_eval_forward_of_a_vit_block_is_its_training_forward(case):
    cfg, st, x, _ = make(CASES[case])
    x_out, logits = O.block_forward_eval(st, x)
    tp = {k: _t(v) for k, v in st.params.items()}
    t_out, t_logits = _torch_vit(cfg, tp, _t(x))
    assert rel_l2(x_out, t_out.numpy()) < 1e-12 and rel_l2(logits, t_logits.numpy()) < 1e-12


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("case", ["vit_img", "resnet"])
def test_zero_head_gives_ln10_and_no_upstream_gradient(case):
    cfg, st, x, y = make(CASES[case])
    st.params["head.w"][:] = 0.0
    st.params["head.b"][:] = 0.0
    _, loss = O.block_step(st, x, y, 0.0)
    assert abs(loss - math.log(10.0)) < 1e-14
    freq = np.bincount(y, minlength=10) / len(y)
    np.testing.assert_allclose(st.grads["head.b"], 0.1 - freq, atol=1e-15)
    for name, g in st.grads.items():
        if name not in ("head.w", "head.b"):
            assert np.abs(g).max() == 0.0, name


def test_fp32_oracle_tracks_fp64_oracle():
    wl = synth.workload("vit_tiny_fp32")
    cfg = oracle_cfg(wl)
    flat = synth.make_params(O.param_spec(cfg), seed=0, jitter=True)
    x, y = synth.make_batch(wl)
    s64, s32 = O.block_init(cfg, flat, np.float64), O.block_init(cfg, flat, np.float32)
    o64, l64 = O.block_step(s64, x, y, 0.01)
    o32, l32 = O.block_step(s32, x, y, 0.01)
    assert o32.dtype == np.float32
    assert abs(l32 - l64) < 1e-5 * abs(l64)
    assert rel_l2(o32, o64) < 1e-5
    for name in s64.grads:
        assert rel_l2(s32.grads[name], s64.grads[name]) < 1e-4, name


# ------------------------------------------------------------------ Algorithm 1 structure
def _two_block_chain(seed_b2=1, head_scale=1.0):
    wl1 = dict(TINY_VIT_IMG, aux_depth=0)
    wl2 = dict(TINY_VIT_ACT, depth=1, aux_depth=1)
    c1, s1, x, y = make(wl1, seed=0)
    c2, s2, _, _ = make(wl2, seed=seed_b2)
    s2.params["head.w"] *= head_scale
    return [s1, s2], x, y


def test_gradient_isolation_block_update_ignores_later_blocks():
    ref, x, y = _two_block_chain()
    alt, _, _ = _two_block_chain(seed_b2=2, head_scale=50.0)
    for _ in range(2):
        O.chain_step(ref, x, y, 0.1)
        O.chain_step(alt, x, y, 0.1)
    for name in ref[0].params:
        assert np.array_equal(ref[0].params[name], alt[0].params[name]), name
    assert not np.array_equal(ref[1].params["head.w"], alt[1].params["head.w"])


def test_block_gradient_is_of_its_own_local_loss_only():
    # block 1's analytic gradient equals the finite difference of block 1's loss,
    # and differs from the finite difference of block 2's loss through x_1
    states, x, y = _two_block_chain()
    s1, s2 = states
    snap = O.block_init(s1.cfg, O.flatten(s1.cfg, s1.params))
    O.block_step(snap, x, y, 0.0)
    name, idx, h = "blk0.fc2.w", 5, 1e-5
    flat = s1.params[name].reshape(-1)

    def losses():
        x1, _, _ = O.block_forward(s1, x)
        return O.local_loss(s1, x, y), O.local_loss(s2, x1, y)

    old = flat[idx]
    flat[idx] = old + h; a1, a2 = losses()
    flat[idx] = old - h; b1, b2 = losses()
    flat[idx] = old
    own, downstream = (a1 - b1) / (2 * h), (a2 - b2) / (2 * h)
    an = snap.grads[name].reshape(-1)[idx]
    assert abs(own - an) < 1e-7 * max(1, abs(own))
    assert abs(downstream) > 1e-6 and abs(downstream - an) > 1e-6


def test_output_is_computed_with_pre_update_parameters():
    cfg, st, x, y = make(TINY_VIT_IMG)
    before = O.block_init(cfg, O.flatten(cfg, st.params))
    x_out, _ = O.block_step(st, x, y, 0.5)
    pre, _, _ = O.block_forward(before, x)
    post, _, _ = O.block_forward(st, x)
    assert np.array_equal(x_out, pre)
    assert rel_l2(post, pre) > 1e-6


def test_chain_equals_blocks_called_in_order_and_labels_ride_along():
    a, x, y = _two_block_chain()
    b, _, _ = _two_block_chain()
    losses, outs = O.chain_step(a, x, y, 0.1)
    x1, l1 = O.block_step(b[0], x, y, 0.1)
    x2, l2 = O.block_step(b[1], x1, y, 0.1)
    assert losses == [l1, l2]
    assert np.array_equal(outs[0], x1) and np.array_equal(outs[1], x2)
    c, _, _ = _two_block_chain()
    y_other = (y + 1) % 10
    lo, _ = O.chain_step(c, x, y_other, 0.1)
    assert lo[1] != l2                        # block 2 sees the labels of its batch


def test_batch_permutation_leaves_loss_unchanged():
    for case in ("vit_img", "resnet"):
        cfg, st, x, y = make(CASES[case])
        perm = np.array([1, 0])
        assert abs(O.local_loss(st, x, y) - O.local_loss(st, x[perm], y[perm])) < 1e-12


def test_token_permutation_with_pos_rows_leaves_logits_unchanged():
    cfg, st, x, y = make(TINY_VIT_IMG)
    _, logits, _ = O.block_forward(st, x)
    # swap patches 0 and 3 of the 2x2 grid in the image and the matching pos rows (cls row 0 stays)
    P = cfg.patch
    x2 = x.copy()
    x2[:, :P, :P], x2[:, P:, P:] = x[:, P:, P:], x[:, :P, :P]
    pos = st.params["pos"].copy()
    st.params["pos"][1], st.params["pos"][4] = pos[4], pos[1]
    _, logits2, _ = O.block_forward(st, x2)
    assert rel_l2(logits2, logits) < 1e-12


@pytest.mark.parametrize("case", list(CASES))
def test_loss_decreases_when_overfitting_one_batch(case):
    cfg, st, x, y = make(CASES[case])
    first = None
    for i in range(20):
        _, loss = O.block_step(st, x, y, 0.05)
        first = loss if first is None else first
    assert loss < 0.8 * first


# ------------------------------------------------------------------ what bf16 storage alone does
def test_bf16_storage_alone_moves_relu_gradients_by_more_than_the_tolerance():
    """Oracle vs oracle: rounding stored activations and filters to bf16 (arithmetic still
    float64) flips the ReLU masks nearest zero, which moves the five-block ResNet stage's
    gradients by far more than 2e-2 while loss and output stay inside it.  This is why the GPU
    parity tests bound a ReLU network's bf16 gradients by this same oracle-vs-oracle distance,
    computed per tensor in the test itself, instead of a flat figure."""
    wl = synth.workload("resnet_stage_bf16", batch=32)
    cfg = oracle_cfg(wl)
    flat = synth.make_params(O.param_spec(cfg), seed=0, jitter=True)
    x, y = synth.make_batch(wl)
    a, b = O.block_init(cfg, flat), O.block_init(cfg, flat, storage="bf16")
    oa, la = O.block_step(a, x.astype(np.float64), y, 0.01)
    ob, lb = O.block_step(b, x.astype(np.float64), y, 0.01)
    assert abs(la - lb) < 2e-2 * la and rel_l2(ob, oa) < 2e-2
    worst = max(rel_l2(b.grads[n], a.grads[n]) for n in a.grads)
    assert 0.05 < worst < 0.3, worst


def test_storage_mode_is_refused_for_the_vit_block():
    """The ViT block takes no binary decision on a floating-point value, so its oracle has one mode: float64."""
    wl = synth.workload("vit_stage_bf16", batch=2, dim=32, heads=2, mlp_dim=64)
    cfg = oracle_cfg(wl)
    flat = synth.make_params(O.param_spec(cfg), seed=0)
    with pytest.raises(ValueError):
        O.block_init(cfg, flat, storage="bf16")
    with pytest.raises(ValueError):
        O.block_init(oracle_cfg(synth.workload("resnet_stage_bf16", batch=2)), None, storage="fp16")


def test_bf16_storage_rounds_what_passes_between_layers_and_nothing_else(monkeypatch):
    """What the storage emulation means, stated without reference to any implementation: one rounding for every
    tensor that one layer hands to the next, forward (convolution output, activation behind BatchNorm + ReLU, block
    output, pooled features) and backward (the gradient maps travelling the other way), one for every filter a
    convolution reads, and none anywhere else: statistics, the values inside a BatchNorm, logits, loss and every
    parameter gradient keep full precision.  Counted here on a stage of n = 3 basic blocks without a stem (the
    first block's input gradient is not formed): 4 n + 3 activations and 4 n + 3 gradient maps, 4 n + 1 filter reads;
    every rounded tensor is made of bfloat16 values; parameter gradients are not."""
    n = 3
    wl = synth.workload("resnet_stage_bf16", batch=4, channels=8, height=6, width=6, n_basic_blocks=n, aux_channels=8)
    cfg = oracle_cfg(wl)
    flat = synth.make_params(O.param_spec(cfg), seed=2, jitter=True)
    x, y = synth.make_batch(wl, seed=2)
    seen = {"act": [], "wmat": []}
    real_act, real_wmat = O.BlockState.act, O.BlockState.wmat

    def act(self, a):
        out = real_act(self, a)
        seen["act"].append(out)
        return out

    def wmat(self, w):
        out = real_wmat(self, w)
        seen["wmat"].append(out)
        return out

    monkeypatch.setattr(O.BlockState, "act", act)
    monkeypatch.setattr(O.BlockState, "wmat", wmat)
    st = O.block_init(cfg, flat, storage="bf16")
    O.block_step(st, x.astype(np.float64), y, 0.01)
    # forward: c1, y1, c2, out per block; aux conv output, aux activation, pooled.  backward: dpooled, its broadcast
    # map, the aux conv-output gradient, the block-output gradient; per block dc2, dy1, dc1 and (not for the first
    # block) the input gradient
    assert len(seen["act"]) == (4 * n + 3) + (4 + 4 * n - 1)
    assert len(seen["wmat"]) == (2 * n + 1) + (1 + n + (n - 1))

    def is_bf16(a):
        a32 = np.asarray(a, dtype=np.float32)
        return np.array_equal(a32.view(np.uint32) & 0xFFFF, np.zeros(a32.shape, np.uint32)) and np.array_equal(a32.astype(np.float64), a)

    assert all(is_bf16(a) for a in seen["act"]) and all(is_bf16(w) for w in seen["wmat"])
    assert not any(is_bf16(g) for k, g in st.grads.items() if g.size > 8), "parameter gradients keep full precision"
    # and with the emulation off nothing is rounded
    seen["act"].clear()
    st2 = O.block_init(cfg, flat)
    O.block_step(st2, x.astype(np.float64), y, 0.01)
    assert seen["act"] and not any(is_bf16(a) for a in seen["act"] if a.size > 8)
