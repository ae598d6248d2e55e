"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element on the same seeded inputs.

Tolerances: 1e-4 on the fp32 path, 2e-2 on the bf16 path, for the local loss
(|dloss|/|loss|), every parameter-gradient tensor and every updated parameter
tensor; the output activation is held to 1e-2 on the bf16 path.  A tensor passes
when its relative L2 error is within the tolerance, no single element is off by
more than MAX_ABS_FACTOR x tolerance x the largest reference magnitude, and (for
the output activation) every row, i.e. every token or pixel, is within 2e-2 /
1e-4 on its own (helpers.assert_close).

The reference is the float64 oracle, nothing else, for every ViT case: that
network takes no binary decision on a floating-point value.

ReLU networks.  A ReLU mask is such a decision, and its gradient is discontinuous
in the pre-activation: one element whose mask differs changes a gradient tensor
by that element's full magnitude.  The oracle is run up to three times, all on
the CPU:
  P    the float64 oracle (the definition);
  E    the float64 oracle deciding its masks on values of the path's precision:
       bf16 storage emulated on the bf16 path; on the fp32 path (only where a test
       asks for it: at small sizes that path meets 1e-4) the oracle in float32;
  E32  bf16 path only: E again with float32 arithmetic, i.e. a second evaluation
       that rounds to bf16 at the same places and differs from E in nothing but
       accumulation precision, which is how a correct GPU result differs from E.
Loss and output are held to the tolerance against P and against E.  A gradient
tensor is held
  against P to max(tolerance, FLOOR_FACTOR x d(E, P)):  the GPU result is one more
      evaluation in that precision, so it may stand as far from the definition as
      E does and not much further (one basic block at natural statistics already
      gives d(E, P) of 0.07 to 0.17: rounding the stored values to bf16 flips the
      masks nearest zero);
  against E to max(tolerance, FLOOR_FACTOR x d(E32, E)):  with one or two blocks
      this is the plain 2e-2; stored bf16 values decorrelate layer by layer, and
      at five blocks two evaluations that differ only in accumulation order stand
      0.1 to 0.15 apart.
Both distances are taken per tensor for the very case under test (depth, seed,
statistics), oracle against oracle; the largest-element criterion, and the
worst-row criterion of the output against P, are bounded the same way.  E rounds
every tensor that passes from one layer to the next, forward and backward, so a
cancelling sum over such a tensor (a weight gradient whose input carries a large
common offset) shows in d(E, P) with the noise it has in any bf16 evaluation.  The shift gradient of a BatchNorm is measured on the scale of the
(scale, shift) gradient pair of that layer: both are sums of the same terms with
weights of order one, and where everything behind the layer is invariant to a
shift (a channel whose ReLU is open everywhere, another BatchNorm further on) the
true shift gradient is a cancelling sum with no scale of its own.  Cases with wide
mask margins (_decisive_shifts) remove the mask flips altogether: there E32 and E
stand 1e-2 to 2e-2 apart at five blocks, and that is how close the GPU has to come
to E; the offsets that make the masks decisive also make every weight gradient
behind them a cancelling sum, so d(E, P) is not small in those cases.
"""
import numpy as np
import pytest

from oracle import ppll_oracle as O
from paper_2411_12780_amd import synth
from helpers import MAX_ABS_FACTOR, assert_close, closeness, oracle_cfg, rel_l2

pytestmark = pytest.mark.gpu

TOL = {synth.FP32: 1e-4, synth.BF16: 2e-2}
OUT_TOL = {synth.FP32: 1e-4, synth.BF16: 1e-2}     # whole output activation (ViT, and against E); its rows are held to TOL
FLOOR_FACTOR = 1.5        # a GPU tensor may stand this many times as far from a reference as the oracle's own runs do
FLOOR_FACTOR_MAX = 2.0    # the same for the largest single element error, which varies more from run to run than a norm


def run_case(wl, steps, seed=0, check_bn=False, tweak=None, precision_floor=False):
    """precision_floor: on the fp32 path of a ReLU network, also run the oracle in float32 and bound the
    gradients by its distance to the float64 oracle (the bf16 path of a ReLU network always does the same
    with bf16 storage emulated)."""
    from gpu_harness import GpuBlock
    from paper_2411_12780_amd import binding as P
    wl = {**dict(beta1=0.9, beta2=0.999, adam_eps=1e-8, momentum=0.0, nesterov=0, weight_decay=0.0), **wl}
    cfg = oracle_cfg(wl)
    flat = synth.make_params(O.param_spec(cfg), seed=seed, jitter=True)
    if tweak is not None:
        tensors = O.unflatten(cfg, flat, np.float32)
        tweak(tensors)
        flat = O.flatten(cfg, tensors).astype(np.float32)
    bf16 = wl["precision"] == synth.BF16
    relu_net = wl["arch"] == synth.RESNET
    pure = O.block_init(cfg, flat, np.float64)
    emul = emul32 = None
    if relu_net and bf16:
        emul = O.block_init(cfg, flat, np.float64, storage="bf16")
        emul32 = O.block_init(cfg, flat, np.float32, storage="bf16")
    elif relu_net and precision_floor:
        emul = O.block_init(cfg, flat, np.float32)
    st = emul if (relu_net and bf16) else pure     # the state that loss, output, parameters and statistics are held to
    gb = GpuBlock(wl, flat)
    assert gb.names == [n for n, _ in O.param_spec(cfg)]
    tol, out_tol = TOL[wl["precision"]], OUT_TOL[wl["precision"]]
    out_tol_pure = tol if relu_net else out_tol    # masks decided in bf16 put the ReLU network's output up to 1e-2 from P
    row_len = wl["dim"] if wl["arch"] == synth.VIT else wl["channels"]
    adamw = wl["optimizer"] == synth.ADAMW
    # AdamW moves a coordinate by about lr*sign(g) however small |g| is, so where the true
    # gradient is zero (key bias) or under the bf16 noise floor the end-to-end parameter is
    # noise-determined.  There the update is checked as arithmetic on the GPU's own gradient
    # (always done, tight tolerance) and end to end on coordinates with a resolvable gradient.
    masked = adamw and bf16
    worst = {}

    def note(key, c):
        for k, v in c.items():
            worst[f"{key}.{k}"] = max(worst.get(f"{key}.{k}", 0.0), v)

    try:
        for i in range(steps):
            x, y = synth.make_batch(wl, seed=seed, index=i)
            print(f"  step {i}: arch={wl['arch']} batch={wl['batch']}", flush=True)
            if masked and i > 0:
                # noise-determined AdamW coordinates make the two trajectories drift apart; each
                # further step is checked from the oracle's state (oracle -> GPU, never back)
                for idx, name in enumerate(gb.names):
                    P.ppll_block_write_tensor(gb.h, P.T_PARAM, idx, st.params[name])
                    P.ppll_block_write_tensor(gb.h, P.T_MOMENT1, idx, st.mom1[name])
                    P.ppll_block_write_tensor(gb.h, P.T_MOMENT2, idx, st.mom2[name])
            p_before, m_before = gb.tensors(P.T_PARAM), gb.tensors(P.T_MOMENT1)
            v_before = gb.tensors(P.T_MOMENT2) if adamw else None
            pure_out, pure_loss = O.block_step(pure, x.astype(np.float64), y, wl["lr"])
            if emul is not None:
                emul_out, emul_loss = O.block_step(emul, x.astype(emul.dtype), y, wl["lr"])
            if emul32 is not None:
                O.block_step(emul32, x.astype(np.float32), y, wl["lr"])
            out, loss = gb.step(x, y, wl["lr"])
            assert abs(loss - pure_loss) <= tol * abs(pure_loss), (i, "loss against the float64 oracle", loss, pure_loss)
            row_tol = max_tol = None
            if emul is not None:       # single pixels next to a flipped mask: bounded by what the precision alone does to them
                apart = closeness(emul_out, pure_out, row_len)
                row_tol = max(tol, FLOOR_FACTOR_MAX * apart["row"])
                max_tol = max(MAX_ABS_FACTOR * out_tol_pure, FLOOR_FACTOR_MAX * apart["max_abs"])
            note("x_out", assert_close(out, pure_out, out_tol_pure, f"step {i} x_out against the float64 oracle", row_len,
                                       row_tol if row_tol else tol, max_tol))
            if st is emul:
                assert abs(loss - emul_loss) <= tol * abs(emul_loss), (i, "loss against the oracle with bf16 masks", loss, emul_loss)
                note("x_out_E", assert_close(out, emul_out, out_tol, f"step {i} x_out against the oracle with bf16 masks",
                                             row_len, tol))
            grads, params = gb.tensors(P.T_GRAD), gb.tensors(P.T_PARAM)
            report = []
            for name, shape in O.param_spec(cfg):
                bound, max_bound = tol, None
                mate = name[:-2] + ".g" if relu_net and ".bn" in name and name.endswith(".b") else None
                if emul is not None:
                    floor = closeness(emul.grads[name], pure.grads[name], floor_ref=pure.grads[mate] if mate else None)
                    bound = max(tol, FLOOR_FACTOR * floor["rel_l2"])
                    max_bound = max(MAX_ABS_FACTOR * tol, FLOOR_FACTOR_MAX * floor["max_abs"])
                if emul32 is not None:
                    apart = closeness(emul32.grads[name], emul.grads[name], floor_ref=emul.grads[mate] if mate else None)
                    note("grad_E", assert_close(grads[name], emul.grads[name], max(tol, FLOOR_FACTOR * apart["rel_l2"]),
                                                f"step {i} grad {name} against the oracle with bf16 masks (float32 against "
                                                f"float64 arithmetic in that oracle: {apart['rel_l2']:.1e})",
                                                max_tol=max(MAX_ABS_FACTOR * tol, FLOOR_FACTOR_MAX * apart["max_abs"]),
                                                floor_ref=emul.grads[mate] if mate else None))
                c = assert_close(grads[name], pure.grads[name], bound, f"step {i} grad {name} against the float64 oracle",
                                 max_tol=max_bound, floor_ref=pure.grads[mate] if mate else None)
                note("grad", c)
                report.append((name, c["rel_l2"], bound))
                # update arithmetic: the oracle's rule applied to the GPU's own tensors
                if adamw:
                    want, _, _ = O.adamw_update(p_before[name], grads[name], m_before[name], v_before[name], i + 1,
                                                wl["lr"], wl["beta1"], wl["beta2"], wl["adam_eps"], wl["weight_decay"])
                else:
                    want, _ = O.sgd_update(p_before[name], grads[name], m_before[name], wl["lr"], wl["momentum"],
                                           bool(wl["nesterov"]), wl["weight_decay"], i == 0)
                e = rel_l2(params[name], want)
                assert e <= 1e-5, (i, "update", name, e)
                worst["update"] = max(worst.get("update", 0), e)
                g_ref = st.grads[name].reshape(-1)
                p_ref = st.params[name].reshape(-1)
                if masked:
                    keep = np.abs(g_ref) >= 0.05 * np.sqrt(np.mean(g_ref ** 2) + 1e-300)
                    if keep.any():
                        note("param", assert_close(params[name][keep], p_ref[keep], tol, f"step {i} param {name}"))
                else:
                    note("param", assert_close(params[name], p_ref, tol, f"step {i} param {name}"))
            top = sorted(report, key=lambda r: -r[1] / r[2])[:6]
            print("  gradient errors nearest their bounds:", [(n, f"{e:.2e}/{b:.2e}") for n, e, b in top], flush=True)
        if check_bn:
            mean, var = gb.bn(P.T_BN_MEAN), gb.bn(P.T_BN_VAR)
            for name, _ in O.bn_stat_spec(cfg):
                assert_close(mean[name], st.bn_mean[name], tol, f"running mean {name}")
                assert_close(var[name], st.bn_var[name], tol, f"running variance {name}")
    finally:
        gb.close()
    print("  worst:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    return worst


def _decisive_shifts(tensors):
    """BatchNorm shifts of +5 / -5 by channel parity: every ReLU decision has a margin of several standard
    deviations, so no mask depends on a rounding.  The second BatchNorm of a block feeds the skip sum: the first
    block lifts it to +5 and the later ones add little to it (scale 0.35, shift 0.5), which keeps that sum
    positive with the same margin without letting the stored values grow block by block (larger values cost
    bf16 its absolute precision)."""
    for name, v in tensors.items():
        if ".bn" in name and name.endswith(".b"):
            v[:] = np.where(np.arange(v.size) % 2 == 0, 5.0, -5.0)
        if name == "aux.bn.b" or name == "stem.bn.b":      # keep the pooled features and the first block's input alive
            v[:] = 5.0
        if name.endswith("bn2.b"):
            v[:] = 5.0 if name.startswith("rb0.") else 0.5
        if name.endswith("bn2.g") and not name.startswith("rb0."):
            v[:] = 0.35


# ------------------------------------------------------------------ fp32 path
def test_vit_tiny_fp32_one_sgd_step():
    run_case(synth.workload("vit_tiny_fp32"), steps=1)


def test_vit_tiny_fp32_three_steps():
    run_case(synth.workload("vit_tiny_fp32"), steps=3, seed=1)


def test_vit_fp32_ragged_activation_input_adamw():
    # sizes off every tile edge: 7 tokens, dim 24 (3 heads of 8), mlp 40, batch 3
    wl = synth.workload("vit_tiny_fp32", input_kind=synth.ACTIVATION, batch=3, tokens=7, dim=24, heads=3,
                        mlp_dim=40, depth=2, aux_depth=1, optimizer=synth.ADAMW, weight_decay=0.01, lr=1e-3)
    run_case(wl, steps=3)


def test_vit_fp32_single_token():
    wl = synth.workload("vit_tiny_fp32", input_kind=synth.ACTIVATION, batch=2, tokens=1, dim=16, heads=2,
                        mlp_dim=32, depth=1, aux_depth=1)
    run_case(wl, steps=2)


def test_vit_fp32_image_many_tokens():
    wl = synth.workload("vit_tiny_fp32", batch=2, img_h=40, img_w=48, patch=4, tokens=121, dim=32, heads=2,
                        mlp_dim=64, depth=1, aux_depth=1)
    run_case(wl, steps=2)


def test_resnet_fp32_small():
    wl = synth.workload("resnet_stage_bf16", precision=synth.FP32, batch=3, channels=8, height=6, width=10,
                        n_basic_blocks=2, aux_channels=12)
    run_case(wl, steps=3, check_bn=True)


def test_resnet_fp32_odd_spatial_plain_sgd():
    wl = synth.workload("resnet_stage_bf16", precision=synth.FP32, batch=2, channels=4, height=7, width=5,
                        n_basic_blocks=1, aux_channels=6, momentum=0.0, nesterov=0, weight_decay=0.0)
    run_case(wl, steps=2, check_bn=True)


def test_resnet_fp32_downsampling_block_in_the_middle():
    # basic block 1 of 3 halves a 10 x 12 map of 4 channels to 5 x 6 x 8: the backward pass crosses its
    # zero-padded, subsampled shortcut and its stride-2 input gradient
    wl = synth.workload("resnet_stage_bf16", precision=synth.FP32, batch=3, channels=8, height=5, width=6,
                        n_basic_blocks=3, transition_block=2, aux_channels=12)
    run_case(wl, steps=3, check_bn=True)


def test_resnet_fp32_stem_in_front_of_the_blocks():
    # first module of the network: the stem is trained, so the gradient also crosses basic block 0
    wl = synth.workload("resnet_stage_bf16", precision=synth.FP32, input_kind=synth.IMAGE, img_h=6, img_w=10, img_c=3,
                        batch=3, channels=8, height=6, width=10, n_basic_blocks=2, aux_channels=12)
    run_case(wl, steps=3, check_bn=True)


def test_resnet_fp32_stem_then_downsampling_first_block():
    wl = synth.workload("resnet_stage_bf16", precision=synth.FP32, input_kind=synth.IMAGE, img_h=14, img_w=10, img_c=3,
                        batch=2, channels=8, height=7, width=5, n_basic_blocks=2, transition_block=1, aux_channels=6)
    run_case(wl, steps=2, check_bn=True)


# ------------------------------------------------------------------ bf16 path
def test_vit_bf16_medium():
    wl = synth.workload("vit_stage_bf16", batch=8, dim=128, heads=2, mlp_dim=256, depth=2, aux_depth=1)
    run_case(wl, steps=2)


def test_vit_bf16_activation_input_ragged():
    wl = synth.workload("vit_stage_act_bf16", batch=5, tokens=37, dim=192, heads=3, mlp_dim=320, depth=1,
                        aux_depth=1)
    run_case(wl, steps=2)


@pytest.mark.parametrize("dim,heads", [(256, 4), (512, 8), (768, 12), (1024, 16)])
def test_vit_bf16_widths_of_the_fast_layernorm(dim, heads):
    # the LayerNorm kernels hold a row in 16, 32 or 64 lanes depending on the width (256: 16, 512 and 768: 32,
    # 1024: 64); 40 tokens leave a ragged last row group in every one of them
    wl = synth.workload("vit_stage_act_bf16", batch=3, tokens=40, dim=dim, heads=heads, mlp_dim=2 * dim, depth=1,
                        aux_depth=1)
    run_case(wl, steps=1)


def test_vit_bf16_deep_block_needs_two_grouped_weight_gradient_launches():
    # 7 encoder layers = 28 weight-gradient products (more than one grouped launch takes) with 336 output tiles
    wl = synth.workload("vit_stage_act_bf16", batch=4, tokens=32, dim=256, heads=4, mlp_dim=1024, depth=6, aux_depth=1)
    run_case(wl, steps=1)


@pytest.mark.parametrize("dim,heads,classes", [(128, 2, 200), (1024, 16, 1024)])
def test_vit_bf16_head_with_many_classes(dim, heads, classes):
    # 200 classes: more classes than lanes in the fused head kernel; 1024 x 1024: too large for its LDS,
    # so the head runs as separate LayerNorm / Linear / cross-entropy kernels
    wl = synth.workload("vit_stage_act_bf16", batch=5, tokens=8, dim=dim, heads=heads, mlp_dim=2 * dim, depth=1,
                        aux_depth=1, num_classes=classes)
    run_case(wl, steps=1)


def test_resnet_fp32_stage_full_size_decisive_masks():
    # not a named workload: fp32 at the full ResNet size.  Gradients pass 10 BatchNorm backward stages, each a
    # cancelling 32768-term reduction: the float32 oracle's own distance to the float64 one bounds them
    run_case(synth.workload("resnet_stage_bf16", precision=synth.FP32), steps=1, check_bn=True, tweak=_decisive_shifts,
             precision_floor=True)


def test_resnet_fp32_stage_full_size_natural_statistics():
    # a single flipped mask among ~1e6 elements moves a layer's gradient by ~1e-3: float32 arithmetic alone puts
    # the oracle 2e-3 to 5e-3 from its float64 self here, and that distance is the bound
    run_case(synth.workload("resnet_stage_bf16", precision=synth.FP32), steps=1, check_bn=True, precision_floor=True)


@pytest.mark.parametrize("tokens", [1, 32, 64, 256])
def test_vit_bf16_token_counts_at_tile_edges(tokens):
    # head dim 64: 1 token, exactly one / two 32-token tiles, and the 256-token maximum
    wl = synth.workload("vit_stage_act_bf16", batch=3, tokens=tokens, dim=128, heads=2, mlp_dim=256, depth=1,
                        aux_depth=1)
    run_case(wl, steps=1)


@pytest.mark.parametrize("tokens,dim,heads", [(20, 128, 4), (65, 96, 1)])
def test_vit_bf16_attention_shapes_outside_the_matrix_core_kernel(tokens, dim, heads):
    # a head dimension other than 64 (32, 96): the run-time-typed attention kernels on bf16 tensors
    wl = synth.workload("vit_stage_act_bf16", batch=2, tokens=tokens, dim=dim, heads=heads, mlp_dim=2 * dim, depth=1,
                        aux_depth=1)
    run_case(wl, steps=1)


def test_resnet_bf16_one_block_full_activation_size():
    run_case(synth.workload("resnet_stage_bf16", n_basic_blocks=1), steps=1, check_bn=True)


def test_resnet_bf16_two_narrow_blocks():
    # second block exercises the input-gradient + skip path; 8 channels keep the fan-out small
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=2, channels=8, aux_channels=16, batch=16)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_two_blocks_on_the_mfma_path():
    # 32 channels: matrix-core convolutions incl. the input gradient with the skip path
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=2)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_odd_sizes_on_the_mfma_path():
    # ragged pixel count (3*7*9 = 189, not a multiple of 32) and odd spatial size with the stride-2 aux conv
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=1, batch=3, height=7, width=9)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_weight_gradient_on_the_mfma_path_edges():
    # 16-pixel rows select the matrix-core weight gradient; 131 images over fewer workgroups make them loop
    # over images, 5 rows of 16 pixels leave the last 32-pixel reduction step of an image half empty
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=1, batch=131, height=5, width=16)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_downsampling_first_block_on_the_mfma_path():
    # 16 -> 32 channels with stride 2: matrix-core forward and the 16-input-channel weight gradient
    wl = synth.workload("resnet32_stage2_bf16", batch=8, n_basic_blocks=2)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_downsampling_block_behind_a_16_channel_block():
    # blocks 4 and 5 of ResNet-32: a 16-channel block on the 32 x 32 map, then the downsampling block
    wl = synth.workload("resnet32_stage2_bf16", batch=4, n_basic_blocks=2, transition_block=2)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_third_stage_64_channels():
    # 32 -> 64 downsampling block, then a 64-channel block on the 8 x 8 map: the filter of a 64 -> 64
    # convolution needs more LDS than a kernel gets without asking (73 KiB)
    wl = synth.workload("resnet32_stage2_bf16", batch=8, channels=64, height=8, width=8, n_basic_blocks=2)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_16_channels_ragged():
    # 16 produced channels fill half a matrix-core tile; 3*7*9 pixels leave a ragged last workgroup
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=2, batch=3, height=7, width=9, channels=16, aux_channels=32)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_48_channels():
    # 48 channels: three 16-channel reduction steps and one and a half 32-channel output tiles in the matrix-core
    # convolutions; BatchNorm and weight gradient take the run-time-typed kernels at this width
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=2, batch=6, height=8, width=8, channels=48, aux_channels=48)
    run_case(wl, steps=1, check_bn=True)


@pytest.mark.parametrize("channels,height,width,batch", [(32, 8, 8, 5), (32, 4, 32, 3), (16, 2, 16, 300), (64, 4, 8, 2)])
def test_resnet_bf16_tiled_weight_gradient_shapes(channels, height, width, batch):
    # the 16x16x32 matrix-core weight gradient: rows of 8, 16 and 32 pixels, 1 to 4 channel tiles, fewer
    # k-steps per image than waves (2 x 16 pixels), more images than workgroups (300)
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=1, batch=batch, height=height, width=width, channels=channels,
                        aux_channels=32)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_stride_2_weight_gradient_64_to_64():
    # the auxiliary convolution 64 -> 64 at stride 2 on a 16 x 16 map: odd / even column planes in the tiled weight
    # gradient, second k-split handed over through LDS
    wl = synth.workload("resnet_stage_bf16", n_basic_blocks=1, batch=3, height=16, width=16, channels=64, aux_channels=64)
    run_case(wl, steps=1, check_bn=True)


def test_resnet_bf16_stem_module():
    wl = synth.resnet32_modules(8, batch=4)[0]
    run_case(wl, steps=1, check_bn=True)


@pytest.mark.parametrize("name", ["resnet32_stage1_bf16", "resnet32_stage2_bf16", "resnet32_stage3_bf16"])
def test_resnet32_stages_at_their_full_shape(name):
    # the three stages of ResNet-32 at their real map and channel sizes (stem, both downsampling blocks, 16 / 32 /
    # 64 channels); batch 100 instead of 1024 keeps the float64 oracle to seconds and leaves ragged last tiles.
    # Five blocks of stored bf16 values decorrelate the masks: every gradient tensor is bounded by what bf16
    # storage alone does to it in the oracle.
    run_case(synth.workload(name, batch=100), steps=1, check_bn=True)


@pytest.mark.parametrize("name", ["resnet32_stage1_bf16", "resnet32_stage2_bf16", "resnet32_stage3_bf16"])
def test_resnet32_stages_at_their_full_shape_decisive_masks(name):
    # the same three stages with every ReLU decision several standard deviations from zero: GPU and oracle take
    # the same masks, so what is compared is the arithmetic of the five-block bf16 backward pass itself
    run_case(synth.workload(name, batch=100), steps=1, check_bn=True, tweak=_decisive_shifts)


def test_resnet_bf16_stage_full_size_natural_statistics():
    run_case(synth.workload("resnet_stage_bf16"), steps=2, check_bn=True)


def test_resnet_bf16_stage_full_size_decisive_masks():
    run_case(synth.workload("resnet_stage_bf16"), steps=2, check_bn=True, tweak=_decisive_shifts)


def test_vit_stage_bf16_full_size():
    run_case(synth.workload("vit_stage_bf16"), steps=3)


@pytest.mark.parametrize("batch,depth", [(37, 3), (50, 1)])
def test_vit_stage_bf16_divided_weight_gradient_tiles_with_a_ragged_reduction(batch, depth):
    # batch 37: 2405 token rows = 37 whole 64-row reduction steps and one of 37 rows, and 345 weight-gradient tiles, so
    # the grouped launch divides 89 of them along the token index and the last part ends in the ragged step; batch 50
    # with one module layer: 129 tiles with a long reduction, fewer than there are compute units, so every one of them is
    # summed from two parts (3250 rows = 50 steps + 50 rows), and 90 class-token tiles with a one-step reduction
    run_case(synth.workload("vit_stage_bf16", batch=batch, depth=depth), steps=1)


def test_vit_base_paper_shape_bf16_full_size():
    # the paper's ViT-Base stage: 640 rows of width 768, K = 768 patch embedding, 5-token attention, SGD Nesterov
    run_case(synth.workload("vit_base_paper_bf16"), steps=2)


def test_vit_base_224_shape_bf16():
    # the paper's ViT-Base at 224 x 224 (197 tokens of width 768: seven 32-token attention tiles, K = 768 and 3072
    # contractions); batch 8 instead of 128 keeps the float64 oracle to seconds
    run_case(synth.workload("vit_base_224_bf16", batch=8), steps=1)


def test_weight_gradients_on_the_side_stream_bf16():
    # 21 x 197 = 4137 rows of width 768: a layer's weight-gradient products have 432 output tiles and a reduction
    # over more than 4096 rows, so the auxiliary layer's run on the block's side stream beside the backward of the
    # module layer; two steps, so that the second forward and update also meet the first step's side work
    run_case(synth.workload("vit_base_224_bf16", batch=21, depth=1, aux_depth=1), steps=2)


def test_vit_large_image_bf16_full_size():
    run_case(synth.workload("vit_large_image_bf16"), steps=1)


# ------------------------------------------------------------------ error surfaced at sync
@pytest.mark.parametrize("name,kw", [
    ("vit_tiny_fp32", dict(aux_depth=1)),
    ("vit_stage_bf16", dict(batch=8)),
    ("resnet_stage_bf16", dict(precision=synth.FP32, batch=4, channels=8, height=8, width=8, n_basic_blocks=2, aux_channels=8)),
    ("resnet_stage_bf16", dict(batch=8, n_basic_blocks=1)),
    ("resnet_stage_bf16", dict(precision=synth.FP32, input_kind=synth.IMAGE, img_h=12, img_w=8, img_c=3, batch=3, channels=8,
                               height=6, width=4, n_basic_blocks=2, transition_block=2, aux_channels=8)),
    ("resnet32_stage2_bf16", dict(batch=8, n_basic_blocks=2)),
])
def test_eval_forward_matches_the_oracle_after_training_steps(name, kw):
    """Two training steps (they move parameters and BatchNorm running statistics), then the evaluation-mode
    forward on a fresh batch: block output and auxiliary class scores against the oracle, with and without
    the logits; parameters and running statistics must be untouched by it."""
    import torch
    from paper_2411_12780_amd import binding as P
    from gpu_harness import GpuBlock, to_device, DEV
    wl = synth.workload(name, **kw)
    bf16 = wl["precision"] == synth.BF16
    tol = 2e-2 if bf16 else 1e-4
    cfg = oracle_cfg(wl)
    flat = synth.make_params(O.param_spec(cfg), seed=13, jitter=True)
    st = O.block_init(cfg, flat, np.float64, storage="bf16" if bf16 and wl["arch"] == synth.RESNET else None)
    blk = GpuBlock(wl, flat)
    stream = torch.cuda.current_stream().cuda_stream
    for i in range(2):
        x, y = synth.make_batch(wl, seed=13, index=i)
        O.block_step(st, x.astype(np.float64), y, float(wl["lr"]))
        P.ppll_block_step(blk.h, to_device(x, wl), torch.from_numpy(y.astype(np.int32)).to(DEV), float(wl["lr"]),
                          blk.x_out, blk.loss, stream)
        P.ppll_block_sync(blk.h)
    # start the evaluation from the oracle's state, so that the comparison is of the forward alone
    for i, (pname, _) in enumerate(O.param_spec(cfg)):
        P.ppll_block_write_tensor(blk.h, P.T_PARAM, i, st.params[pname].astype(np.float32))
    for i, (bname, _) in enumerate(O.bn_stat_spec(cfg)):
        P.ppll_block_write_tensor(blk.h, P.T_BN_MEAN, i, st.bn_mean[bname].astype(np.float32))
        P.ppll_block_write_tensor(blk.h, P.T_BN_VAR, i, st.bn_var[bname].astype(np.float32))
    params_before = [P.ppll_block_read_tensor(blk.h, P.T_PARAM, i) for i in range(len(blk.names))]
    x, _ = synth.make_batch(wl, seed=13, index=9)
    want_out, want_logits = O.block_forward_eval(st, x.astype(np.float64))
    logits = torch.full((wl["batch"], wl["num_classes"]), float("nan"), dtype=torch.float32, device=DEV)
    out2 = torch.empty_like(blk.x_out)
    P.ppll_block_forward_eval(blk.h, to_device(x, wl), blk.x_out, logits, stream)
    P.ppll_block_forward_eval(blk.h, to_device(x, wl), out2, None, stream)
    torch.cuda.synchronize()
    got_out = blk.x_out.float().cpu().numpy().reshape(want_out.shape)
    assert_close(got_out, want_out, OUT_TOL[wl["precision"]], "evaluation output", wl["dim"] if wl["arch"] == synth.VIT else wl["channels"], tol)
    assert_close(logits.cpu().numpy(), want_logits, tol, "evaluation logits")
    assert torch.equal(out2, blk.x_out)
    for i, b in enumerate(params_before):
        assert np.array_equal(P.ppll_block_read_tensor(blk.h, P.T_PARAM, i), b)
    for i, (bname, _) in enumerate(O.bn_stat_spec(cfg)):
        assert np.array_equal(P.ppll_block_read_tensor(blk.h, P.T_BN_MEAN, i), st.bn_mean[bname].astype(np.float32))
    blk.close()


def test_phase_timers_split_a_step_into_the_papers_four_terms():
    """f_1, f_a1, B_a1, U_a1 of Section 3.3: four positive durations that add up to about the step time, leave
    the step's results untouched, and are refused while the timers are off."""
    import time
    import torch
    from paper_2411_12780_amd import binding as P
    from gpu_harness import GpuBlock, to_device
    wl = synth.workload("vit_stage_bf16", batch=16)
    flat = synth.make_params(O.param_spec(oracle_cfg(wl)), seed=11, jitter=True)
    x, y = synth.make_batch(wl, seed=11, index=0)
    results = []
    for timers in (False, True):
        blk = GpuBlock(wl, flat)
        xd, yd = to_device(x, wl), torch.from_numpy(y.astype(np.int32)).to("cuda:0")
        stream = torch.cuda.current_stream().cuda_stream
        if timers:
            P.ppll_block_phase_timers(blk.h, True)
        else:
            with pytest.raises(RuntimeError):
                P.ppll_block_phase_times(blk.h)
        for _ in range(3):
            P.ppll_block_step(blk.h, xd, yd, 1e-3, blk.x_out, blk.loss, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        P.ppll_block_step(blk.h, xd, yd, 1e-3, blk.x_out, blk.loss, stream)
        loss = P.ppll_block_sync(blk.h)
        wall_ms = 1e3 * (time.perf_counter() - t0)
        if timers:
            ms = P.ppll_block_phase_times(blk.h)
            assert len(ms) == 4 and all(v > 0 for v in ms), ms
            assert sum(ms) <= wall_ms * 1.05, (ms, wall_ms)
        results.append((loss, [P.ppll_block_read_tensor(blk.h, P.T_PARAM, i) for i in range(len(blk.names))]))
        blk.close()
    assert results[0][0] == results[1][0]
    for a, b in zip(results[0][1], results[1][1]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("name,kw", [
    ("vit_stage_bf16", dict(batch=16)),
    ("resnet_stage_bf16", dict(batch=16, n_basic_blocks=2)),
    ("resnet32_stage1_bf16", dict(batch=8, n_basic_blocks=1)),
])
def test_two_runs_from_the_same_state_are_bit_identical(name, kw):
    """Every reduction on the path is ordered (two-stage partial sums, no floating-point atomics): the same
    inputs give the same bits, run after run, which is what lets the pipeline tests demand equality."""
    from gpu_harness import GpuBlock
    from paper_2411_12780_amd import binding as P
    wl = synth.workload(name, **kw)
    flat = synth.make_params(O.param_spec(oracle_cfg(wl)), seed=21, jitter=True)
    runs = []
    for _ in range(2):
        gb = GpuBlock(wl, flat)
        outs = []
        for i in range(3):
            x, y = synth.make_batch(wl, seed=21, index=i)
            out, loss = gb.step(x, y, float(wl["lr"]))
            outs.append((out.copy(), loss))
        runs.append((outs, [P.ppll_block_read_tensor(gb.h, P.T_PARAM, i) for i in range(len(gb.names))]))
        gb.close()
    for (oa, la), (ob, lb) in zip(runs[0][0], runs[1][0]):
        assert la == lb and np.array_equal(oa, ob)
    for a, b in zip(runs[0][1], runs[1][1]):
        assert np.array_equal(a, b)


def test_zero_learning_rate_leaves_parameters_alone_but_not_the_moments():
    from gpu_harness import GpuBlock
    from paper_2411_12780_amd import binding as P
    for wl in (synth.workload("vit_stage_bf16", batch=4, weight_decay=0.0), synth.workload("resnet_stage_bf16", batch=4, n_basic_blocks=1)):
        flat = synth.make_params(O.param_spec(oracle_cfg(wl)), seed=5, jitter=True)
        gb = GpuBlock(wl, flat)
        before = [P.ppll_block_read_tensor(gb.h, P.T_PARAM, i) for i in range(len(gb.names))]
        x, y = synth.make_batch(wl, seed=5)
        gb.step(x, y, 0.0)
        after = [P.ppll_block_read_tensor(gb.h, P.T_PARAM, i) for i in range(len(gb.names))]
        for a, b in zip(before, after):
            assert np.array_equal(a, b)
        m1 = [P.ppll_block_read_tensor(gb.h, P.T_MOMENT1, i) for i in range(len(gb.names))]
        assert any(np.abs(m).max() > 0 for m in m1)
        gb.close()


def test_resnet_downsampling_block_as_the_last_of_the_module_and_batch_of_one():
    # the module's output comes straight out of the downsampling block; one image still gives BatchNorm its rows
    wl = synth.workload("resnet_stage_bf16", precision=synth.FP32, batch=1, channels=8, height=4, width=6, n_basic_blocks=2,
                        transition_block=2, aux_channels=8)
    run_case(wl, steps=2, check_bn=True)


def test_vit_batch_of_one():
    run_case(synth.workload("vit_stage_bf16", batch=1, depth=1, aux_depth=1), steps=1)


def test_launch_brackets_count_the_contraction_kernels_and_their_work():
    """The measurement aid behind bench.py's roofline: with brackets on for a block, its ViT step reports its
    matrix-core GEMM launches with 2 M N K flops each, a ResNet block's step its convolution launches with their
    algorithmic bytes; the setting belongs to the block (a second block stepped in between reports nothing) and
    the step's results do not change."""
    from paper_2411_12780_amd import binding as P
    from gpu_harness import GpuBlock
    vit = synth.workload("vit_stage_act_bf16", batch=8, depth=2, aux_depth=0)
    res = synth.workload("resnet_stage_bf16", batch=4, n_basic_blocks=1)
    losses = {}
    for on in (False, True):
        for name, wl in (("vit", vit), ("resnet", res)):
            flat = synth.make_params(O.param_spec(oracle_cfg(wl)), seed=3, jitter=True)
            gb, other = GpuBlock(wl, flat), GpuBlock(wl, flat)
            P.ppll_block_profile_enable(gb.h, on)
            x, y = synth.make_batch(wl, seed=3)
            _, loss = gb.step(x, y, float(wl["lr"]))
            other.step(x, y, float(wl["lr"]))            # not timed: the switch is per block
            losses[(name, on)] = loss
            gemm_ms, gemm_flops, gemm_n = P.ppll_block_profile_read(gb.h)
            conv_ms, conv_bytes, conv_n = P.ppll_block_profile_read_conv(gb.h)
            assert P.ppll_block_profile_read(other.h)[2] == 0 and P.ppll_block_profile_read_conv(other.h)[2] == 0
            if not on:
                assert gemm_n == 0 and conv_n == 0
            elif name == "vit":
                # two encoder layers: forward, input gradient and weight gradient of QKV, proj, fc1, fc2 each (the first
                # layer's QKV input gradient too: LayerNorm 1 needs it for its scale and shift), however they are grouped
                M, D, F = 8 * vit["tokens"], vit["dim"], vit["mlp_dim"]
                fwd = 2.0 * M * (D * 3 * D + D * D + 2 * D * F)
                assert gemm_n >= 16 and gemm_ms > 0 and conv_n == 0
                assert P.ppll_block_profile_read_small(gb.h)[2] == 0      # no product with fewer than 256 rows here
                assert abs(gemm_flops - 2 * 3 * fwd) <= 1e-6 * gemm_flops
            else:
                # one basic block + auxiliary convolution: 3 forward launches, conv2's and the auxiliary input gradient
                px, C, A = 4 * 16 * 16, 32, 64
                f_block = 2.0 * (2 * px * C + 9 * C * C)
                f_aux = 2.0 * (px * C + (px // 4) * A + 9 * C * A)
                assert conv_n == 5 and conv_ms > 0 and gemm_n == 0
                assert abs(conv_bytes - (3 * f_block + 2 * f_aux)) <= 1e-6 * conv_bytes
            # a second read finds nothing new
            assert P.ppll_block_profile_read(gb.h)[2] == 0 and P.ppll_block_profile_read_conv(gb.h)[2] == 0
            gb.close(); other.close()
    assert losses[("vit", False)] == losses[("vit", True)] and losses[("resnet", False)] == losses[("resnet", True)]


def test_out_of_range_label_is_reported_at_sync():
    from gpu_harness import GpuBlock
    from paper_2411_12780_amd import binding as P
    wl = synth.workload("vit_tiny_fp32")
    cfg = oracle_cfg(wl)
    gb = GpuBlock(wl, synth.make_params(O.param_spec(cfg), seed=0))
    x, y = synth.make_batch(wl)
    y = y.copy()
    y[3] = 10
    with pytest.raises(P.PpllError) as e:
        gb.step(x, y, 0.01)
    assert e.value.status == 6
    y[3] = 9
    gb.step(x, y, 0.01)                 # flag is cleared by the failed sync
    gb.close()
    with pytest.raises(P.PpllError) as e:
        P.ppll_block_sync(gb.h)         # use after destroy is an error, not a crash
    assert e.value.status == 7
