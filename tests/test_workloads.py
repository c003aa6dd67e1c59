"""The seeded synthetic workloads: shapes, determinism, zero fractions and the chained network's
consistency.  They are inputs only; these checks keep the recipe the documentation states."""
import numpy as np
import pytest

import oracle
from paper_2104_08314_amd import workloads


def test_layer_table_matches_the_five_workloads():
    specs = workloads.all_layers()
    assert len(specs) == 22 and len({s.name for s in specs}) == 22
    by = {s.name: s for s in specs}
    assert by["cfg1.16@28"].shape_tuple == (16, 28, 28, 16, 3, 3, 1, 1)
    assert by["cfg2.128@56"].shape_tuple == (128, 56, 56, 128, 3, 3, 1, 1)
    assert by["cfg3.256@14"].shape_tuple == (256, 14, 14, 256, 3, 3, 1, 1)
    assert by["cfg4a.5x5.64@27"].shape_tuple == (64, 27, 27, 192, 5, 5, 1, 2)
    assert by["cfg4b.3x3s2.128@56"].shape_tuple == (128, 56, 56, 256, 3, 3, 2, 1)
    assert by["cfg5.stem7x7s2"].shape_tuple == (3, 224, 224, 64, 7, 7, 2, 3)
    assert [s.C for s in workloads.layers(5)[1:]] == [64] * 3 + [128] * 4 + [256] * 6 + [512] * 3


def test_line_layers_keep_their_map_size():
    specs = workloads.line_layers()
    assert len(specs) == 8 and len({s.name for s in specs}) == 8
    for s in specs:
        assert (s.kh == 1) != (s.kw == 1) and s.stride == 1
        assert (s.Oh, s.Ow) == (s.H, s.W)                     # padded in the kernel's direction only
        assert s.shape_tuple[7:] == (s.kh // 2, s.kw // 2)
        act = workloads.make_activation(s)
        assert act.shape == (s.C, s.H, s.W) and (act >= 0).all()
        assert abs(float((act == 0).mean()) - (s.zero_frac + 0.05 * (1 - s.zero_frac))) < 0.03


@pytest.mark.parametrize("name,lo,hi", [("cfg1.16@28", 0.52, 0.60), ("cfg2.128@56", 0.59, 0.61),
                                        ("cfg3.256@14", 0.70, 0.76), ("cfg4a.5x5.64@27", 0.49, 0.51),
                                        ("cfg4b.3x3s2.128@56", 0.63, 0.67), ("cfg5.l16.512@7s1", 0.84, 0.88)])
def test_zero_fractions_of_the_recipe(name, lo, hi):
    spec = {s.name: s for s in workloads.all_layers()}[name]
    act = workloads.make_activation(spec)
    assert act.dtype == np.float32 and act.shape == (spec.C, spec.H, spec.W) and act.flags["C_CONTIGUOUS"]
    assert (act >= 0).all()                                   # post-ReLU maps
    assert lo <= float((act == 0).mean()) <= hi
    dead = int((act.reshape(spec.C, -1) == 0).all(axis=1).sum())
    assert dead >= spec.zero_channels


def test_generators_are_deterministic_and_inputs_differ():
    spec = workloads.layers(3)[0]
    a0, a0b, a1 = workloads.make_activation(spec), workloads.make_activation(spec), workloads.make_activation(spec, 1)
    assert np.array_equal(a0, a0b) and not np.array_equal(a0, a1)
    w0, w0b = workloads.make_weights(spec), workloads.make_weights(spec)
    assert np.array_equal(w0, w0b) and w0.shape == (spec.K, spec.C, spec.kh, spec.kw)
    sigma = np.sqrt(2.0 / (spec.C * spec.kh * spec.kw))
    assert abs(float(w0.std()) / sigma - 1.0) < 0.02          # He-normal


def test_chained_network_fits_together():
    specs = workloads.chain_specs()
    assert len(specs) == 16
    for prev, cur in zip(specs, specs[1:]):
        assert (cur.C, cur.H, cur.W) == (prev.K, prev.Oh, prev.Ow)
    assert (specs[0].C, specs[0].H) == (64, 56) and (specs[-1].K, specs[-1].Oh) == (512, 7)
    act, ws, bs = workloads.make_chain()
    assert act.shape == (64, 56, 56) and bs[0] is None
    assert all(w.shape == (s.K, s.C, 3, 3) for w, s in zip(ws, specs))
    assert all(b.shape == (s.C,) and b.dtype == np.float32 for b, s in zip(bs[1:], specs[1:]))


def test_chained_network_reaches_the_intended_sparsity():
    """The biases are set from a closed-form estimate of every layer's output spread; what the
    network really produces (oracle, first six layers) must stay near the targeted zero fractions
    and keep dead channels dead."""
    specs = workloads.chain_specs()[:6]
    act, ws, bs = workloads.make_chain()
    outs = oracle.chain_forward(act, [(s.shape_tuple, w, b, b is not None) for s, w, b in zip(specs, ws, bs)])
    for i in range(1, 6):
        a = oracle.bias_relu(outs[i - 1], bs[i])
        z = float((a == 0).mean())
        assert abs(z - specs[i].zero_frac) < 0.07, (i, z, specs[i].zero_frac)
        dead = int((a.reshape(a.shape[0], -1) == 0).all(axis=1).sum())
        assert dead >= specs[i].zero_channels
