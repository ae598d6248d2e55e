"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, answers size queries and rejects bad
configurations before touching the device."""
import os
import re

import numpy as np
import pytest

from paper_2411_12780_amd import binding as P
from paper_2411_12780_amd import synth
from oracle import ppll_oracle as O
from helpers import oracle_cfg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ppll.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ppll_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = P.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(P.EXPORTS)


@pytest.mark.parametrize("name", list(synth.WORKLOADS))
def test_size_queries_match_the_workload(name):
    wl = synth.workload(name)
    cfg = P.make_config(wl)
    esz = 2 if wl["precision"] == synth.BF16 else 4
    assert P.ppll_block_param_bytes(cfg) == 4 * O.param_count(oracle_cfg(wl))
    n_in = 1
    for d in synth.input_shape(wl):
        n_in *= d
    n_out = 1
    for d in synth.output_shape(wl):
        n_out *= d
    assert P.ppll_block_in_bytes(cfg) == n_in * esz
    assert P.ppll_block_out_bytes(cfg) == n_out * esz
    ws = P.ppll_block_workspace_bytes(cfg)
    assert ws % 256 == 0 and ws > 4 * P.ppll_block_param_bytes(cfg) // 2


def test_bad_configurations_are_rejected_on_the_host():
    good = synth.workload("vit_tiny_fp32")
    for bad in (dict(tokens=64), dict(heads=5), dict(precision=7), dict(arch=3), dict(batch=0),
                dict(optimizer=9), dict(depth=0), dict(patch=5), dict(tokens=300, img_h=68, img_w=68, patch=4)):
        cfg = P.make_config(dict(good, **bad))
        with pytest.raises(P.PpllError) as e:
            P.ppll_block_workspace_bytes(cfg)
        assert e.value.status == 2, bad
        assert P.ppll_last_error()
    cfg = P.make_config(good)
    cfg.struct_size = 12
    with pytest.raises(P.PpllError):
        P.ppll_block_workspace_bytes(cfg)
    res = synth.workload("resnet_stage_bf16")
    # a stem keeps the image size, a downsampling block needs an index inside the module and even channels
    for bad in (dict(input_kind=synth.IMAGE, img_h=32, img_w=32, img_c=3), dict(transition_block=6),
                dict(transition_block=-1), dict(transition_block=1, channels=31),
                dict(input_kind=synth.IMAGE, transition_block=1, img_h=16, img_w=16, img_c=3)):
        with pytest.raises(P.PpllError) as e:
            P.ppll_block_workspace_bytes(P.make_config(dict(res, **bad)))
        assert e.value.status == 2, bad


def test_library_and_published_size_of_vit_base_patch16_224_agree():
    # the library's own parameter table for ViT-base-patch16-224 as one block: the published 86,567,656 parameters
    wl = dict(synth.workload("vit_base_paper_bf16"), img_h=224, img_w=224, tokens=197, depth=12, aux_depth=0, num_classes=1000,
              batch=1)
    assert P.ppll_block_param_bytes(P.make_config(wl)) == 4 * 86567656


def test_size_queries_of_every_resnet32_module():
    wls = synth.resnet32_modules(8)
    for wl in wls:
        cfg = P.make_config(wl)
        assert P.ppll_block_param_bytes(cfg) == 4 * O.param_count(oracle_cfg(wl))
        assert P.ppll_block_in_bytes(cfg) == 2 * int(np.prod(synth.input_shape(wl)))
        assert P.ppll_block_out_bytes(cfg) == 2 * int(np.prod(synth.output_shape(wl)))
    # the chain of modules is accepted as a pipeline
    assert P.ppll_pipeline_workspace_bytes([P.make_config(w) for w in wls], 2) > 0


def test_null_and_misaligned_arguments():
    cfg = P.make_config(synth.workload("vit_tiny_fp32"))
    with pytest.raises(P.PpllError) as e:
        P.ppll_block_init(cfg, None, 1 << 20, None)
    assert e.value.status == 1
    with pytest.raises(P.PpllError) as e:
        P.ppll_block_init(cfg, 0x1008, 1 << 20, None)       # not 16-byte aligned: rejected before any use
    assert e.value.status == 4
    with pytest.raises(P.PpllError) as e:
        P.ppll_block_step(None, 16, 16, 0.1, 16)
    assert e.value.status == 1
    # the entry points added for evaluation and timing reject a null handle the same way
    for call in (lambda: P.ppll_block_forward_eval(None, 16, 16), lambda: P.ppll_block_phase_timers(None, True),
                 lambda: P.ppll_block_phase_times(None)):
        with pytest.raises(P.PpllError) as e:
            call()
        assert e.value.status == 1


def test_pipeline_shape_chain_is_checked():
    a = P.make_config(synth.workload("vit_stage_bf16"))
    b = P.make_config(synth.workload("vit_stage_act_bf16"))
    assert P.ppll_pipeline_workspace_bytes([a, b, b, b], 2) > 4 * P.ppll_block_workspace_bytes(b)
    with pytest.raises(P.PpllError) as e:
        P.ppll_pipeline_workspace_bytes([a, a], 2)          # second block wants images
    assert e.value.status == 3
    with pytest.raises(P.PpllError):
        P.ppll_pipeline_workspace_bytes([a, b], 0)
    small = P.make_config(synth.workload("vit_stage_act_bf16", batch=64))
    with pytest.raises(P.PpllError):
        P.ppll_pipeline_workspace_bytes([a, small], 2)
