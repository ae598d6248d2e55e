"""Workload tables: the auxiliary-depth heuristic and the finest partition built from it."""
from paper_2411_12780_amd import synth


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
