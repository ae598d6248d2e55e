"""Workload tables: the auxiliary-depth heuristic, the finest ViT partition built from it, and the
partition of ResNet-32 into local modules."""
import pytest

from oracle import ppll_oracle as O
from paper_2411_12780_amd import synth
from helpers import oracle_cfg


def test_aux_depth_schedule_follows_the_papers_formula():
    # N_l = d' - floor(l / 3) for the 12 local blocks of the ViT (Section 4.2); written out by hand
    assert synth.aux_depth_schedule(4) == [4, 4, 4, 3, 3, 3, 2, 2, 2, 1, 1, 1]
    assert synth.aux_depth_schedule(3) == [3, 3, 3, 2, 2, 2, 1, 1, 1, 0, 0, 0]
    # d' = 2 would give -1 for l >= 9: floored at zero auxiliary layers
    assert synth.aux_depth_schedule(2) == [2, 2, 2, 1, 1, 1, 0, 0, 0, 0, 0, 0]
    # every entry equals the formula wherever the formula is non-negative
    for d in (2, 3, 4):
        for l, got in enumerate(synth.aux_depth_schedule(d)):
            assert got == max(0, d - l // 3)


def test_lpp_workloads_are_one_layer_blocks_chained_by_activations():
    wls = synth.lpp_workloads(4)
    assert len(wls) == 12
    assert wls[0]["input_kind"] == synth.IMAGE and all(w["input_kind"] == synth.ACTIVATION for w in wls[1:])
    assert all(w["depth"] == 1 for w in wls)
    assert [w["aux_depth"] for w in wls] == synth.aux_depth_schedule(4)
    # consecutive blocks agree on the activation they exchange
    for a, b in zip(wls, wls[1:]):
        assert synth.output_shape(a) == synth.input_shape(b)


@pytest.mark.parametrize("k", [2, 3, 4, 8, 15])
def test_resnet32_modules_add_up_to_resnet32(k):
    wls = synth.resnet32_modules(k)
    assert len(wls) == k and sum(w["n_basic_blocks"] for w in wls) == 15
    assert wls[0]["input_kind"] == synth.IMAGE and synth.input_shape(wls[0]) == (1024, 32, 32, 3)
    for a, b in zip(wls, wls[1:]):
        assert synth.output_shape(a) == synth.input_shape(b)
    assert synth.output_shape(wls[-1]) == (1024, 8, 8, 64)
    # the module parameters (everything but the auxiliary heads) are those of ResNet-32 without its
    # classifier: the published 464,154 parameters less the 64 x 10 + 10 of the final Linear layer
    theta = 0
    for w in wls:
        for name, shape in O.param_spec(oracle_cfg(w)):
            if not name.startswith(("aux.", "head.")):
                n = 1
                for d in shape:
                    n *= d
                theta += n
    assert theta == 464154 - 650
    # exactly two modules hold a downsampling block, at basic blocks 5 and 10 of the network
    first, found = 0, []
    for w in wls:
        if w["transition_block"]:
            found.append(first + w["transition_block"] - 1)
        first += w["n_basic_blocks"]
    assert found == [5, 10]


def test_resnet32_partitions_outside_the_supported_range_are_refused():
    for k in (0, 16):
        with pytest.raises(ValueError):
            synth.resnet32_modules(k)
    with pytest.raises(ValueError):
        synth.resnet32_modules(1)     # one module would hold both downsampling blocks


def test_cosine_schedule_endpoints_midpoint_and_symmetry():
    T = 400
    assert synth.cosine_lr(0, T) == 0.01
    assert abs(synth.cosine_lr(T // 2, T) - 0.005) < 1e-15
    assert abs(synth.cosine_lr(T, T)) < 1e-15
    rates = [synth.cosine_lr(t, T) for t in range(T + 1)]
    assert all(a > b for a, b in zip(rates, rates[1:]))
    # lr(t) + lr(T - t) = lr0: the curve is point-symmetric about its midpoint
    assert all(abs(rates[t] + rates[T - t] - 0.01) < 1e-15 for t in range(T + 1))
