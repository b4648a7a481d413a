"""GPU parity of the AdamW step for non-matrix parameters (Sec. 4.1) against the float64 oracle,
through the C ABI.  Tolerances: moments relative max error <= 1e-6 (fp32 recurrences); fp32
parameters |w - w_oracle| <= 2e-6 max|w| after each step from the GPU's own previous w (division and
square root are correctly rounded, the error is a few fp32 roundings of an O(eta) step); bf16
parameters within one bf16 ulp of the rounded float64 result."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import adamw_oracle as ao
from oracle import mona_oracle as orc
from paper_2605_26842_amd import binding as B

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def f64(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_max(x, ref):
    s = np.abs(ref).max()
    return float(np.abs(x - ref).max() / s) if s > 0 else float(np.abs(x - ref).max())


def draw(shapes, seed, dtype, scale):
    g = torch.Generator().manual_seed(seed)
    return [(torch.randn(s, generator=g) * scale).to(dtype) for s in shapes]


def run_case(shapes, w_dtype, g_dtype, hp, steps, seed, grad_scales=None):
    params = draw(shapes, seed, w_dtype, 0.5)
    dev = [p.to("cuda:0").contiguous() for p in params]
    opt = B.AdamWOptimizer(dev, g_dtype=g_dtype)
    ohp = ao.AdamWHParams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay).f32()
    oracles = [ao.AdamWOracle(tuple(s)) for s in shapes]
    for k in range(steps):
        scale = 1e-2 if grad_scales is None else grad_scales[k]
        grads = draw(shapes, seed + 100 + k, g_dtype, scale)
        before = [f64(d) for d in dev]
        opt.step([g.to("cuda:0") for g in grads], hp)
        torch.cuda.synchronize()
        for i, o in enumerate(oracles):
            want = o.step(before[i], f64(grads[i]), ohp)      # from the exact values the GPU started from
            got = f64(dev[i])
            tag = f"step {k + 1} tensor {i} {tuple(shapes[i])}"
            assert rel_max(f64(opt.exp_avg(i)), o.m) <= 1e-6, tag
            assert rel_max(f64(opt.exp_avg_sq(i)), o.v) <= 1e-6, tag
            if w_dtype == torch.float32:
                assert np.abs(got - want).max() <= 2e-6 * np.abs(want).max(), tag
            else:
                ulp = np.maximum(np.abs(want), 2.0 ** -126) * 2.0 ** -7
                assert (np.abs(got - orc.round_to_bf16(want)) <= ulp).all(), tag
                assert (got != orc.round_to_bf16(want)).mean() <= 2e-3, tag
    assert opt.step_count() == steps
    return opt, dev


@pytest.mark.parametrize("w_dtype,g_dtype", [(torch.float32, torch.float32), (torch.bfloat16, torch.float32),
                                              (torch.bfloat16, torch.bfloat16), (torch.float32, torch.bfloat16)])
def test_adamw_matches_oracle(w_dtype, g_dtype):
    say("[case] adamw", w_dtype, g_dtype)
    # sizes: below one quad, ragged tails, exactly one chunk, several chunks plus a tail, 2-D
    shapes = [(1,), (3,), (4,), (4095,), (4096,), (4097,), (3 * 4096 + 5,), (64, 129), (513, 32)]
    hp = B.mona_adamw_hparams(1e-2, 0.9, 0.95, 1e-8, 0.1)
    run_case(shapes, w_dtype, g_dtype, hp, steps=5, seed=7)


def test_adamw_other_hyperparameters_and_gradient_scales():
    say("[case] adamw hyper-parameters")
    shapes = [(1000,), (77, 33)]
    for hp in (B.mona_adamw_hparams(3e-2, 0.8, 0.999, 1e-6, 0.0), B.mona_adamw_hparams(1e-3, 0.0, 0.5, 1e-3, 0.5)):
        run_case(shapes, torch.float32, torch.float32, hp, steps=6, seed=11,
                 grad_scales=[1.0, 1e-6, 1e3, 1e-3, 0.0, 1e-2])


def test_adamw_mixed_dtypes_in_one_list_and_checkpoint():
    say("[case] adamw mixed list, checkpoint")
    hp = B.mona_adamw_hparams(1e-2, 0.9, 0.95, 1e-8, 0.1)
    shapes = [(5000,), (300,), (4096 * 2,)]
    g = torch.Generator().manual_seed(3)
    params = [torch.randn(shapes[0], generator=g), torch.randn(shapes[1], generator=g).bfloat16(),
              torch.randn(shapes[2], generator=g).bfloat16()]
    grads = [[torch.randn(s, generator=g) * 1e-2 for s in shapes] for _ in range(4)]
    grads = [[gs[0], gs[1], gs[2].bfloat16()] for gs in grads]

    dev_full = [p.to("cuda:0").contiguous() for p in params]
    opt_full = B.AdamWOptimizer(dev_full)
    with pytest.raises(B.MonaError) as ei:        # built for fp32 gradients: a bf16 one is a dtype change
        opt_full.step([x.to("cuda:0") for x in grads[0]], hp)
    assert ei.value.code == B.MONA_ESHAPE and opt_full.step_count() == 0
    # per-tensor gradient dtypes: build the descriptors from example gradients
    lib = B.load_library()

    def build(dev, ex):
        vec = B.make_vectors(dev, ex)
        nbytes = B.mona_adamw_state_size(vec, len(dev))
        arena = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        h = C.c_void_p(0)
        assert lib.mona_adamw_init_state(vec, len(dev), arena.data_ptr(), nbytes, 0, C.byref(h)) == B.MONA_OK
        return h.value, arena

    def steps(handle, dev, ks):
        for k in ks:
            gd = [x.to("cuda:0") for x in grads[k]]
            B.mona_adamw_step(handle, B.make_vectors(dev, gd), len(dev), hp, 0)
            torch.cuda.synchronize()

    ex = [x.to("cuda:0") for x in grads[0]]
    h_full, arena_full = build(dev_full, ex)
    steps(h_full, dev_full, range(4))
    # oracle on each tensor
    ohp = ao.AdamWHParams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay).f32()
    for i in range(3):
        o = ao.AdamWOracle(shapes[i])
        w = f64(params[i])
        for k in range(4):
            w = o.step(w, f64(grads[k][i]), ohp)
            if params[i].dtype == torch.bfloat16:
                w = orc.round_to_bf16(w)
        got = f64(dev_full[i])
        if params[i].dtype == torch.float32:
            assert np.abs(got - w).max() <= 1e-5 * np.abs(w).max()
        else:
            assert (np.abs(got - w) <= np.abs(w) * 2.0 ** -6 + 1e-30).all()     # a few ulps over 4 rounded steps
    # two steps, export, import into a fresh state, two more: bit-identical
    dev_a = [p.to("cuda:0").contiguous() for p in params]
    h_a, arena_a = build(dev_a, ex)
    steps(h_a, dev_a, range(2))
    n = C.c_size_t(0)
    assert lib.mona_adamw_state_export_size(h_a, C.byref(n)) == B.MONA_OK
    blob = torch.empty(n.value, dtype=torch.uint8, device="cuda:0")
    assert lib.mona_adamw_state_export(h_a, blob.data_ptr(), n.value, 0) == B.MONA_OK
    torch.cuda.synchronize()
    dev_b = [t.clone() for t in dev_a]
    h_b, arena_b = build(dev_b, ex)
    assert lib.mona_adamw_state_import(h_b, blob.data_ptr(), n.value, 2, 0) == B.MONA_OK
    steps(h_b, dev_b, (2, 3))
    for i in range(3):
        assert torch.equal(dev_b[i], dev_full[i]), f"tensor {i} differs after resume"
    t = C.c_int64(0)
    assert lib.mona_adamw_state_step_count(h_b, C.byref(t)) == B.MONA_OK and t.value == 4
    assert lib.mona_adamw_state_import(h_b, blob.data_ptr(), n.value - 256, 2, 0) == B.MONA_ESHAPE
    for h in (h_full, h_a, h_b):
        assert lib.mona_adamw_free_state(h) == B.MONA_OK
