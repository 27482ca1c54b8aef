"""The workload description against the paper's Table I and known ResNet-50 sizes."""
import os

import numpy as np

from paper_1808_05567_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_resnet50_layers.txt")


def test_table1_matches_fixture():
    rows = [tuple(int(t) for t in ln.split()) for ln in open(GOLDEN)
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 20
    for row, l in zip(rows, inputs.TABLE_I):
        assert row == (l.id, l.C, l.K, l.H, l.W, l.R, l.S, l.stride)


def test_output_sizes_are_resnet50():
    want = {1: 112, 4: 56, 6: 28, 7: 28, 8: 28, 11: 14, 12: 14, 13: 14, 16: 7, 17: 7, 18: 7, 20: 7}
    for lid, p in want.items():
        l = inputs.layer(lid)
        assert (l.P, l.Q) == (p, p)
    for l in inputs.TABLE_I:
        assert l.pad == {7: 3, 3: 1, 1: 0}[l.R]


def test_flop_total_per_pass():
    tot = sum(l.flops(256) for l in inputs.TABLE_I)
    assert abs(tot / 1e9 - 711.5) < 0.5
    assert inputs.layer(4).flops(256) == 2 * 256 * 64 * 64 * 56 * 56 * 9


def test_generators_are_seeded_and_distributed():
    a = inputs.gen_input(2, 8, 14, 14, layer_id=4)
    b = inputs.gen_input(2, 8, 14, 14, layer_id=4)
    assert a.dtype == np.float32 and np.array_equal(a, b)
    assert a.min() >= -1.0 and a.max() < 1.0 and abs(a.mean()) < 0.05
    assert not np.array_equal(a, inputs.gen_input(2, 8, 14, 14, layer_id=4, seed=1))
    w = inputs.gen_weights(64, 64, 3, 3, layer_id=4)
    assert abs(w.std() / np.sqrt(2.0 / (64 * 9)) - 1.0) < 0.03
    g = inputs.gen_outgrad(2, 8, 14, 14, layer_id=4)
    assert not np.array_equal(a, g)


def test_bf16_rounding_is_nearest_even():
    import torch
    x = np.concatenate([inputs.gen_input(1, 4, 16, 16).ravel(),
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e-39], np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(inputs.round_to_bf16(x), ref)
