"""GPU tests of the cases a long training run meets sooner or later: gradients of extreme scale, a matrix
that stops receiving gradients, a NaN step followed by a restored checkpoint, memory next to the arena."""
import ctypes as C
import dataclasses

import numpy as np
import pytest
import torch

from oracle import mona_oracle as orc
from paper_2605_26842_amd import binding as B
from paper_2605_26842_amd import workloads as wl
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("scale", [1e-25, 1e-14, 1e-9, 1e15, 1e30])
def test_gradient_scale_does_not_matter(scale):
    """X_0 = M / ||M||_F (Sec. 3.2) is scale-free: gradients of any magnitude the fp32 state can hold must give
    the oracle's O.  (The products accumulate the unscaled working copy in fp32; outside the safe window of
    the norm the copy is rescaled by a power of two first.)"""
    say(f"[case] gradient scale {scale:g}")
    shapes = [(256, 512), (300, 100), (40, 64), (512, 1536)]
    weights = [wl.draw_weight(s, 5000 + i, torch.float32) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 5100 + i, sigma=scale) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(2)]
    hp = wl.HParams()
    opt, _, hist = H.run_gpu(weights, grads, hp, 0)
    worst = H.check_history(weights, grads, hp, hist, range(len(shapes)), H.TOL_NS_BF16, label=f"scale {scale:g}")
    say("[worst]", worst)
    st = opt.status()
    for i, s in enumerate(st):
        norm = float(np.sqrt((hist[-1][i].M ** 2).sum()))
        assert ((s & B.MONA_STATUS_RESCALED) != 0) == (not 2.0 ** -40 <= norm <= 2.0 ** 40), (i, s, norm)
        assert (s & 3) == 0
    assert any(s & B.MONA_STATUS_RESCALED for s in st) == (scale != 1e-9)


def test_matrix_without_gradients_decays_to_zero_cleanly():
    """A matrix that receives exactly zero gradients (a dead expert): M decays as mu^k, G~ = alpha A decays
    as beta_a^k.  O must follow the oracle all the way down, through the rescaled range, until M is exactly
    zero, where only weight decay is left."""
    say("[case] zero gradients from step 2 on")
    shape = (192, 320)
    dev = "cuda:0"
    w = wl.draw_weight(shape, 5200, torch.float32, dev)
    g1 = wl.GradientStream(shape, 5201, dev).next()
    zero = torch.zeros(shape, device=dev)
    hp = wl.HParams(momentum=0.5, beta_a=0.5, alpha=-1.0, flags=B.MONA_FLAG_KEEP_O)
    ohp = H.oracle_hp(hp)
    opt = B.MonaOptimizer([w])
    o = orc.MonaOracle(shape)
    seen_rescaled = seen_zero = False
    for k in range(200):
        g = g1 if k == 0 else zero
        opt.step([g], hp)
        M = o.elementwise(H.f64(g), ohp)
        st = opt.status()[0]
        m_gpu = H.f64(opt.momentum(0))
        if not m_gpu.any():
            seen_zero = True
            assert st == B.MONA_STATUS_ZERO_NORM
            assert not H.f64(opt.last_o(0)).any()
            break
        if k % 8 == 0 or (st & B.MONA_STATUS_RESCALED):
            # fp32 state: compare O against the oracle's Newton-Schulz of the GPU's own M (the state arrays
            # leave the oracle's float64 trajectory once they reach fp32 subnormals)
            O_ref = orc.newton_schulz(m_gpu, ohp.ns_steps, ohp.ns_a, ohp.ns_b, ohp.ns_c, ohp.ns_eps)
            e = H.rel_fro(H.f64(opt.last_o(0)), O_ref)
            nrm = float(np.sqrt((m_gpu ** 2).sum()))
            assert e <= H.TOL_NS_BF16, f"step {k + 1}: ||M|| = {nrm:.3e}, O rel Fro err {e:.3e}"
            assert abs(float(opt.norm(0).item()) - nrm) <= 1e-6 * nrm + 2.0 ** -149    # the norm is reported in fp32
            if st & B.MONA_STATUS_RESCALED:
                seen_rescaled = True
                assert nrm < 2.0 ** -40
    assert seen_rescaled and seen_zero
    assert torch.isfinite(w).all()


def test_nan_step_then_restored_checkpoint_on_a_ragged_shape():
    """A NaN gradient must not outlive the step it came in: the parameter is left alone, and once the caller
    restores the previous checkpoint the following clean step is the oracle's (no NaN may have reached the
    zero padding of the working matrices, which a 333 x 130 matrix has on every side)."""
    say("[case] NaN step, import, clean step")
    shapes = [(333, 130), (100, 300), (512, 1536)]
    dev = "cuda:0"
    weights = [wl.draw_weight(s, 5300 + i, torch.float32) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 5310 + i) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(3)]
    hp = wl.HParams()
    dev_w = [w.to(dev) for w in weights]
    opt = B.MonaOptimizer(dev_w)
    hpk = dataclasses.replace(hp, flags=B.MONA_FLAG_KEEP_O)
    opt.step([g.to(dev) for g in grads[0]], hpk)
    ckpt = opt.export_state().clone()
    w_before = [w.clone() for w in dev_w]
    bad = [g.clone() for g in grads[1]]
    for b in bad:
        b[7, 9] = float("nan")
    opt.step([g.to(dev) for g in bad], hpk)
    assert all(s & B.MONA_STATUS_NONFINITE for s in opt.status())
    for w0, w1 in zip(w_before, dev_w):
        assert torch.equal(w0, w1)
    opt.import_state(ckpt, 1)
    opt.step([g.to(dev) for g in grads[1]], hpk)
    torch.cuda.synchronize()
    assert opt.status() == [0, 0, 0]
    ref = H.run_oracle_for(weights, grads[:2], hp, range(3))
    for i in range(3):
        assert H.rel_max(H.f64(opt.momentum(i)), ref[i][1]["M"]) <= H.TOL_STATE
        e = H.rel_fro(H.f64(opt.last_o(i)), ref[i][1]["O"])
        assert e <= H.TOL_NS_BF16, (i, e)
        assert torch.isfinite(dev_w[i]).all()
    # also without the import: the NaN momentum stays flagged, and a repaired M gives a clean step
    opt2 = B.MonaOptimizer([w.to(dev) for w in weights])
    opt2.step([g.to(dev) for g in bad], hpk)
    for i in range(3):
        opt2.momentum(i).zero_(); opt2.accel(i).zero_(); opt2.g_prev(i).zero_()
    opt2.step([g.to(dev) for g in grads[0]], hpk)
    torch.cuda.synchronize()
    assert opt2.status() == [0, 0, 0]
    for i in range(3):
        e = H.rel_fro(H.f64(opt2.last_o(i)), ref[i][0]["O"])
        assert e <= H.TOL_NS_BF16, (i, e)


def test_nothing_is_written_outside_the_arena():
    """Canary words on both sides of the arena survive init, steps of every kernel kind and a checkpoint
    round trip."""
    say("[case] arena canaries")
    dev = "cuda:0"
    shapes = [(512, 1536)] * 12 + [(333, 130), (100, 300), (40, 64), (257, 257)]
    weights = [wl.draw_weight(s, 5400 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
    grads = [wl.GradientStream(s, 5410 + i, dev).next() for i, s in enumerate(shapes)]
    mats = B.make_matrices(weights, None)
    need = B.mona_state_size(mats, len(shapes))
    guard = 1 << 20
    buf = torch.full((need + 2 * guard,), 0xA5, dtype=torch.uint8, device=dev)
    arena = buf[guard: guard + need]
    assert arena.data_ptr() % 256 == 0
    s = torch.cuda.current_stream().cuda_stream
    state = B.mona_init_state(mats, len(shapes), None, arena, s)
    for T in (5, 0):
        hp = B.make_hparams(wl.HParams(ns_steps=T, flags=B.MONA_FLAG_KEEP_O))
        B.mona_step(state, B.make_matrices(weights, grads), len(shapes), hp, s)
    torch.cuda.synchronize()
    B.mona_free_state(state)
    assert bool((buf[:guard] == 0xA5).all()) and bool((buf[guard + need:] == 0xA5).all())


def test_alpha_outside_the_theorems_range_is_noted_not_refused():
    say("[case] alpha warning")
    dev = "cuda:0"
    w = [wl.draw_weight((64, 96), 5500, torch.float32, dev)]
    g = [wl.GradientStream((64, 96), 5501, dev).next()]
    opt = B.MonaOptimizer(w)
    lib = B.load_library()
    opt.step(g, wl.HParams(beta_a=0.9, alpha=-5.0))
    assert lib.mona_last_error() == b""
    opt.step(g, wl.HParams(beta_a=0.9, alpha=-10.0))          # |alpha| = 1 / (1 - beta_a): not below it
    msg = lib.mona_last_error().decode()
    assert msg.startswith("warning") and "1 / (1 - beta_a)" in msg
    assert opt.step_count() == 2
    opt.step(g, wl.HParams(beta_a=0.9, alpha=-10.0, flags=B.MONA_FLAG_MUON_ONLY))   # alpha is ignored there
    assert lib.mona_last_error() == b""
    torch.cuda.synchronize()
