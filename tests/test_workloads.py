"""Host-side checks of the seeded input generators: the shapes the benchmark spec names, the
layer layouts whose sizes add up to the models' parameter counts (ResNet-18 on CIFAR-10:
11,173,962, the figure of Sec. 4.1), reproducibility (the oracle and the GPU must get
the same bytes), and the statistical structure each workload promises."""
import json
import os

import numpy as np
import pytest
import torch

from paper_2011_06495_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_layouts_add_up_to_the_parameter_counts():
    r18, r50 = W.resnet18_cifar_blocks(), W.resnet50_imagenet_blocks()
    assert len(r18) == 62 and sum(r18) == 11_173_962          # Sec. 4.1
    assert len(r50) == 161 and sum(r50) == 25_557_032
    assert r18[0] == 3 * 3 * 3 * 64 and r18[-1] == 10 and r50[-1] == 1000


def test_shapes_are_those_of_the_baseline_configs():
    cfgs = json.load(open(os.path.join(ROOT, "BASELINE.json")))["configs"]
    assert len(cfgs) == 5
    want = {"C1": (4, 1 << 20, 10486, "f32"), "C2": (10, 11_173_962, 11_174, "f32"),
            "C3": (16, 11_173_962, 2_793, "f32"), "C4": (16, 11_173_962, 11_174, "f32"),
            "C5": (32, 25_557_032, 25_557, "bf16")}
    for name, (N, d, K, dt) in want.items():
        w = W.WORKLOADS[name]
        assert (w.N, w.d, w.K, w.grad_dtype) == (N, d, K, dt)
        assert ("N=%d workers" % N) in cfgs[w.index]
        if w.blocks:
            assert sum(w.blocks) == d
    assert W.C3.steps == 20 and W.C4.steps == 5 and W.C5.steps == 10


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_same_seed_same_bytes_and_rows_are_independent_streams(name):
    w = W.WORKLOADS[name].with_size(50_003, N=4)
    a = W.gradients(w, 3)
    b = W.gradients(w, 3, threads=4)
    assert a.dtype == (np.uint16 if w.grad_dtype == "bf16" else np.float32)
    assert np.array_equal(a, b)
    assert np.array_equal(a[2], W.gradient_row(w, 3, 2))
    assert not np.array_equal(a, W.gradients(w, 4))
    assert not np.array_equal(a[0], a[1])
    assert np.array_equal(W.selection_clocks(w, 3), W.selection_clocks(w, 3))
    assert not np.array_equal(W.selection_clocks(w, 3), W.selection_clocks(w, 4))


def test_reduced_sizes_keep_the_sparsity_and_the_layout():
    w = W.C2.with_size(300_007, N=10)
    assert w.K == round(W.C2.phi * 300_007) and sum(w.blocks) == 300_007 and len(w.blocks) <= 62
    assert W.C2.with_size(W.C2.d, K=111_740).K == 111_740 and W.C2.with_size(W.C2.d).blocks == W.C2.blocks
    assert np.all(W.zero_error(w) == 0) and W.zero_error(w).shape == (10, 300_007)


def test_workers_share_a_common_component():
    # C2: correlation 0.5 between two workers' rows before the block scaling
    w = W.C2.with_size(400_009, N=3)
    g = W.gradients(w, 0).astype(np.float64) / W.coordinate_scale(w)
    c = np.corrcoef(g[0], g[1])[0, 1]
    assert abs(c - 0.5) < 0.01
    assert abs(g[0].std() - 1.0) < 0.01
    # C1: weights 0.5 and 0.866, correlation 0.25
    w1 = W.C1.with_size(400_009)
    g1 = W.gradients(w1, 0).astype(np.float64) / W.coordinate_scale(w1)
    assert abs(np.corrcoef(g1[0], g1[1])[0, 1] - 0.25) < 0.01


def test_block_scales_span_the_stated_decades():
    w = W.C2.with_size(300_007, N=2)
    s = W.coordinate_scale(w)
    assert s.dtype == np.float32 and s.shape == (300_007,)
    assert 1e-3 <= s.min() and s.max() <= 1e-1
    edges = np.cumsum(w.blocks)[:-1]
    assert np.count_nonzero(np.diff(s) != 0) <= len(w.blocks) - 1      # constant inside a block
    assert np.all(np.isin(np.flatnonzero(np.diff(s) != 0) + 1, edges))
    s5 = W.coordinate_scale(W.C5.with_size(300_007, N=2))
    assert 1e-4 <= s5.min() and s5.max() <= 1e-1


def test_lattice_workload_stays_on_its_lattice():
    w = W.C4.with_size(200_003, N=4, lattice_shift=6)
    g = W.gradients(w, 0)
    level = np.abs(g) * 2.0 ** 6
    assert np.array_equal(level, np.rint(level)) and level.max() <= 255
    # sums of a few rows are still exact lattice values: ties persist under error feedback
    s = (g[0] + g[1]) + g[2]
    assert np.array_equal(s * 2.0 ** 6, np.rint(s * 2.0 ** 6))
    # heavy ties: far fewer distinct magnitudes than coordinates
    assert np.unique(np.abs(g[0])).size <= 256


def test_bf16_gradients_are_round_to_nearest_even_of_fp32_draws():
    w = W.C5.with_size(100_003, N=2)
    bits = W.gradient_row(w, 0, 1)
    assert bits.dtype == np.uint16
    # the generator's own conversion against torch's
    x = np.random.default_rng(1).standard_normal(100_000).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]              # two exact ties: to even
    ours = W._to_bf16_bits(x)
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, theirs)
    assert ours[2] == 0x3F80 and ours[3] == 0x3F82


def test_heavy_tailed_workload_and_selection_clocks():
    w = W.C3.with_size(400_009, N=2)
    g = W.gradients(w, 0).astype(np.float64) / W.coordinate_scale(w)
    k = ((g[0] - g[0].mean()) ** 4).mean() / g[0].var() ** 2
    assert k > 6.0                                   # Student-t(3): far heavier than a normal's 3
    r = W.selection_clocks(w, 0)
    assert r.dtype == np.float32 and r.shape == (w.d,) and np.all(r >= 0) and np.all(np.isfinite(r))
    assert abs(r.mean() - 1.0) < 0.01 and abs(np.median(r) - np.log(2.0)) < 0.01
