"""ppll_block_forward_eval_noalloc (the evaluation forward whose activation scratch is the library's built-in device
buffer) against ppll_block_forward_eval, through the C ABI: bit-identical outputs, on calls in a row that share
the buffer, the later ones with smaller inputs; a block that does not fit is refused before anything runs."""
import numpy as np
import pytest

from oracle import ppll_oracle as O
from paper_2411_12780_amd import synth
from helpers import oracle_cfg

pytestmark = pytest.mark.gpu


def _block(name, seed, **kw):
    from gpu_harness import GpuBlock
    wl = synth.workload(name, **kw)
    flat = synth.make_params(O.param_spec(oracle_cfg(wl)), seed=seed, jitter=True)
    return wl, GpuBlock(wl, flat)


def _both_ways(wl, blk, seed):
    """(x_out, logits) of the existing entry point and of the one under test, on the same fresh input."""
    import torch
    from paper_2411_12780_amd import binding as P
    from gpu_harness import to_device, DEV
    stream = torch.cuda.current_stream().cuda_stream
    x, _ = synth.make_batch(wl, seed=seed, index=3)
    xd = to_device(x, wl)
    want_out = torch.full_like(blk.x_out, float("nan"))
    got_out = torch.full_like(blk.x_out, float("nan"))
    want_logits = torch.full((wl["batch"], wl["num_classes"]), float("nan"), dtype=torch.float32, device=DEV)
    got_logits = torch.full_like(want_logits, float("nan"))
    P.ppll_block_forward_eval(blk.h, xd, want_out, want_logits, stream)
    P.ppll_block_forward_eval_noalloc(blk.h, xd, got_out, got_logits, stream)
    torch.cuda.synchronize()
    return want_out, want_logits, got_out, got_logits


@pytest.mark.parametrize("cases", [
    # a ViT stage at batch 32 (29 MB of the 64 MiB buffer), then smaller ones: fewer images, then an activation-input block
    [("vit_stage_bf16", dict(batch=32)), ("vit_stage_bf16", dict(batch=8)), ("vit_stage_act_bf16", dict(batch=3, tokens=37))],
    # ResNet stages: five blocks at batch 64, then a stem + downsampling module at batch 8, then the fp32 path
    [("resnet_stage_bf16", dict(batch=64)),
     ("resnet32_stage2_bf16", dict(batch=8, n_basic_blocks=2)),
     ("resnet_stage_bf16", dict(precision=synth.FP32, input_kind=synth.IMAGE, img_h=12, img_w=8, img_c=3, batch=3, channels=8,
                                height=6, width=4, n_basic_blocks=2, transition_block=2, aux_channels=8))],
    # tiny fp32 ViT after a large bf16 one
    [("vit_stage_bf16", dict(batch=64)), ("vit_tiny_fp32", dict(aux_depth=1))],
])
def test_noalloc_eval_equals_the_workspace_eval_on_calls_in_a_row(cases):
    import torch
    from paper_2411_12780_amd import binding as P
    from gpu_harness import to_device, DEV
    blocks = [_block(name, 50 + i, **kw) for i, (name, kw) in enumerate(cases)]
    try:
        # one training step each, so that parameters, BatchNorm running statistics and saved activations are those of a run
        for wl, blk in blocks:
            x, y = synth.make_batch(wl, seed=77)
            blk.step(x, y, float(wl["lr"]))
        for i, (wl, blk) in enumerate(blocks):
            print(f"  call {i}: arch={wl['arch']} batch={wl['batch']}", flush=True)
            want_out, want_logits, got_out, got_logits = _both_ways(wl, blk, seed=60 + i)
            assert not torch.isnan(want_out.float()).any() and not torch.isnan(want_logits).any()
            assert torch.equal(got_out, want_out), i
            assert torch.equal(got_logits, want_logits), i
        # and once more in reverse order (larger after smaller), without the logits
        stream = torch.cuda.current_stream().cuda_stream
        for i, (wl, blk) in reversed(list(enumerate(blocks))):
            x, _ = synth.make_batch(wl, seed=90 + i)
            xd = to_device(x, wl)
            want = torch.empty_like(blk.x_out)
            got = torch.empty_like(blk.x_out)
            P.ppll_block_forward_eval(blk.h, xd, want, None, stream)
            P.ppll_block_forward_eval_noalloc(blk.h, xd, got, None, stream)
            torch.cuda.synchronize()
            assert torch.equal(got, want), i
    finally:
        for _, blk in blocks:
            blk.close()


def test_noalloc_eval_leaves_the_training_state_of_the_block_alone():
    """A step, the no-alloc evaluation, a second step: the second step's results equal those of two steps with no
    evaluation in between (the evaluation touches neither parameters nor statistics)."""
    import torch
    from paper_2411_12780_amd import binding as P
    from gpu_harness import to_device
    results = []
    for evaluate in (False, True):
        wl, blk = _block("resnet_stage_bf16", 5, batch=16, n_basic_blocks=2)
        stream = torch.cuda.current_stream().cuda_stream
        x0, y0 = synth.make_batch(wl, seed=5, index=0)
        x1, y1 = synth.make_batch(wl, seed=5, index=1)
        blk.step(x0, y0, 0.01)
        if evaluate:
            out = torch.empty_like(blk.x_out)
            P.ppll_block_forward_eval_noalloc(blk.h, to_device(x1, wl), out, None, stream)
            torch.cuda.synchronize()
        _, loss = blk.step(x1, y1, 0.01)
        results.append((loss, [P.ppll_block_read_tensor(blk.h, P.T_PARAM, i) for i in range(len(blk.names))],
                        blk.bn(P.T_BN_MEAN)))
        blk.close()
    assert results[0][0] == results[1][0]
    for a, b in zip(results[0][1], results[1][1]):
        assert np.array_equal(a, b)
    for k in results[0][2]:
        assert np.array_equal(results[0][2][k], results[1][2][k])


def test_noalloc_eval_refuses_a_block_that_does_not_fit_and_enqueues_nothing():
    import torch
    from paper_2411_12780_amd import binding as P
    from gpu_harness import to_device
    wl, blk = _block("vit_stage_bf16", 1)          # batch 128: 115 MB of activations, the buffer holds 64 MiB
    try:
        x, _ = synth.make_batch(wl)
        out = torch.full_like(blk.x_out, 7.0)
        with pytest.raises(P.PpllError) as e:
            P.ppll_block_forward_eval_noalloc(blk.h, to_device(x, wl), out, None, torch.cuda.current_stream().cuda_stream)
        assert e.value.status == 4 and "scratch" in str(e.value)
        torch.cuda.synchronize()
        assert bool((out == 7.0).all())
        with pytest.raises(P.PpllError) as e:      # argument errors as in the existing entry point
            P.ppll_block_forward_eval_noalloc(blk.h, None, out, None, None)
        assert e.value.status == 1
    finally:
        blk.close()
    with pytest.raises(P.PpllError) as e:
        P.ppll_block_forward_eval_noalloc(blk.h, out, out, None, None)
    assert e.value.status == 7
