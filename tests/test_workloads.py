"""The synthetic input recipe: shapes of the benchmark configurations and the
statistics of the seeded generators (CPU only)."""
import math

import torch

from paper_2605_26842_amd import workloads as wl


def test_config_sizes():
    assert wl.WORKLOADS["single_256x512"].num_elements() == 131072
    assert wl.WORKLOADS["dense_block_h2048"].num_elements() == 4 * 2048 * 2048 + 2 * 2048 * 8192
    bank = wl.WORKLOADS["moe_bank_e64"]
    assert len(bank.shapes()) == 192 and bank.num_elements() == 192 * 2048 * 1024
    layer = wl.WORKLOADS["moe_layer_h4096_e128"]
    assert len(layer.shapes()) == 4 + 384
    assert layer.num_elements() == 4 * 4096 * 4096 + 384 * 4096 * 1536
    assert abs(layer.ns_flops_dense(5) - 96.4e12) < 0.1e12
    stack = wl.WORKLOADS["moe_stack_l24"]
    assert len(stack.shapes()) == 24 * (388 + 2)
    assert len(stack.names()) == len(stack.shapes())
    assert wl.CONFIG_ORDER[3] == "moe_layer_h4096_e128"


def test_generators_are_seeded_and_have_the_stated_statistics():
    shape = (256, 512)
    w1 = wl.draw_weight(shape, 7, torch.float32)
    w2 = wl.draw_weight(shape, 7, torch.float32)
    assert torch.equal(w1, w2)
    assert abs(w1.std().item() - 0.02) < 5e-4
    s1, s2 = wl.GradientStream(shape, 9), wl.GradientStream(shape, 9)
    a = [s1.next() for _ in range(4)]
    b = [s2.next() for _ in range(4)]
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert a[0].dtype == torch.float32
    for g in a:
        assert abs(g.std().item() - 1e-3) < 3e-5          # stationary
    # lag-1 correlation 0.9
    corr = (a[2] * a[3]).mean().item() / (a[2].std().item() * a[3].std().item())
    assert abs(corr - 0.9) < 0.02
    d = a[3] - a[2]
    assert abs(d.std().item() - 1e-3 * math.sqrt(0.2)) < 3e-5


def test_make_inputs_layout():
    w, g = wl.make_inputs(wl.WORKLOADS["ragged_mix"], 6, steps=2)
    shapes = wl.WORKLOADS["ragged_mix"].shapes()
    assert [tuple(x.shape) for x in w] == shapes
    assert len(g) == 2 and [tuple(x.shape) for x in g[1]] == shapes
    assert not torch.equal(g[0][0], g[1][0])


def test_in_place_gradient_stream():
    """`advance` overwrites the previous gradient: same draws as `next`, same AR(1) recurrence up to the
    order of rounding."""
    shape = (64, 96)
    a, b = wl.GradientStream(shape, 11), wl.GradientStream(shape, 11)
    g = torch.empty(shape)
    for k in range(4):
        want = a.next()
        b.advance(g)
        assert torch.allclose(g, want, rtol=1e-5, atol=1e-9)
        if k == 0:
            assert torch.equal(g, want)
    paper = wl.WORKLOADS["paper_moe_68b"]
    assert len(paper.shapes()) == 512 and paper.shapes()[0] == (3072, 1024) and paper.shapes()[-1] == (1024, 3072)
