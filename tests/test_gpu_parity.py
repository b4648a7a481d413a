"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same
seeded inputs, element by element.  Tolerances: fp32 elementwise state relative max error
<= 1e-6; bf16 Newton-Schulz output and update relative Frobenius error <= 2e-2; fp32-class
variant <= 1e-4."""
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


def inputs(name, steps=None, g_dtype=torch.float32):
    w = wl.WORKLOADS[name]
    idx = list(wl.WORKLOADS).index(name)
    return w, *wl.make_inputs(w, idx, "cpu", steps, g_dtype)


# --------------------------------------------------------------------------------------------
# configs[0]: one fp32 256 x 512 matrix, 3 steps -- every output, every step
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("ns_precision,tol", [(0, H.TOL_NS_BF16), (1, H.TOL_NS_F32)])
def test_single_matrix_three_steps(ns_precision, tol):
    say(f"[case] single_256x512 ns_precision={ns_precision}")
    w, weights, grads = inputs("single_256x512")
    hp = wl.HParams()
    _, _, hist = H.run_gpu(weights, grads, hp, ns_precision)
    worst = H.check_history(weights, grads, hp, hist, [0], tol, label="single")
    say("[worst]", worst)
    assert worst["ns"] > 0      # the comparison is not vacuous


# --------------------------------------------------------------------------------------------
# ragged shapes: nothing is a multiple of a tile; tall, wide, square, vectors, a 3-member group
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("ns_precision,tol", [(0, H.TOL_NS_BF16), (1, H.TOL_NS_F32)])
def test_ragged_shapes(ns_precision, tol):
    say(f"[case] ragged_mix ns_precision={ns_precision}")
    w, weights, grads = inputs("ragged_mix", steps=2)
    hp = wl.HParams()
    _, _, hist = H.run_gpu(weights, grads, hp, ns_precision)
    worst = H.check_history(weights, grads, hp, hist, range(len(weights)), tol, label="ragged")
    say("[worst]", worst)


@pytest.mark.parametrize("beta_a,alpha", [(0.99, -50.0), (0.98, -25.0), (0.975, -20.0), (0.9, 0.0)])
def test_paper_hyperparameter_pairs_and_plain_muon(beta_a, alpha):
    """The (beta_a, alpha) pairs of the Limitations section, and alpha = 0 (plain Muon)."""
    say(f"[case] pairs beta_a={beta_a} alpha={alpha}")
    shapes = [(192, 320), (320, 192)]
    weights = [wl.draw_weight(s, 11 + i, torch.float32) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 21 + i) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(3)]
    hp = wl.HParams(beta_a=beta_a, alpha=alpha)
    _, _, hist = H.run_gpu(weights, grads, hp, 0)
    H.check_history(weights, grads, hp, hist, [0, 1], H.TOL_NS_BF16, label="pairs")
    if alpha == 0.0:
        # momentum is Muon's: M_k = mu M_{k-1} + G_k, bit for bit in fp32
        m = torch.zeros(shapes[0])
        for k in range(3):
            m = torch.tensor(0.95, dtype=torch.float32) * m + grads[k][0]
        got = hist[-1][0].M
        assert H.rel_max(got, m.double().numpy()) <= 1e-6


def test_ns_steps_zero_and_other_counts():
    for T in (0, 1, 2, 4):
        say(f"[case] ns_steps={T}")
        shapes = [(130, 260), (260, 130)]
        weights = [wl.draw_weight(s, 31 + i, torch.float32) for i, s in enumerate(shapes)]
        streams = [wl.GradientStream(s, 41 + i) for i, s in enumerate(shapes)]
        grads = [[st.next() for st in streams] for _ in range(2)]
        hp = wl.HParams(ns_steps=T)
        _, _, hist = H.run_gpu(weights, grads, hp, 0)
        H.check_history(weights, grads, hp, hist, [0, 1], H.TOL_NS_BF16, label=f"T={T}")


def test_first_diff_zero_flag_and_constant_gradient():
    say("[case] constant gradient")
    shape = (64, 96)
    g = wl.GradientStream(shape, 5).next()
    w0 = wl.draw_weight(shape, 6, torch.float32)
    # Alg. 1 literally: A_1 = (1 - beta) g, then pure decay because D_k is exactly 0
    hp = wl.HParams()
    opt, _, hist = H.run_gpu([w0], [[g]] * 4, hp, 0)
    for k in range(1, 4):
        a_prev, a_now = hist[k - 1][0].A, hist[k][0].A
        want = (np.float32(0.9) * a_prev.astype(np.float32)).astype(np.float64)
        assert np.array_equal(a_now, want)
    # with the flag the acceleration buffer stays exactly 0 and MONA is Muon
    hp2 = wl.HParams(flags=B.MONA_FLAG_FIRST_DIFF_ZERO)
    _, _, hist2 = H.run_gpu([w0], [[g]] * 3, hp2, 0)
    for snap in hist2:
        assert not snap[0].A.any()
    hp3 = wl.HParams(alpha=0.0)
    _, _, hist3 = H.run_gpu([w0], [[g]] * 3, hp3, 0)
    assert np.array_equal(hist2[-1][0].M, hist3[-1][0].M)
    assert np.array_equal(hist2[-1][0].W, hist3[-1][0].W)


def test_plain_muon_flag():
    """MONA_FLAG_MUON_ONLY: Eqs. muon_momentum / muon_ns / muon_update, acceleration buffers untouched."""
    say("[case] muon-only flag")
    shapes = [(160, 288), (288, 160)]
    weights = [wl.draw_weight(s, 101 + i, torch.float32) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 111 + i) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(3)]
    hp = wl.HParams(flags=B.MONA_FLAG_MUON_ONLY)        # alpha = -5 is ignored
    _, _, hist = H.run_gpu(weights, grads, hp, 0)
    for snap in hist:
        for i in (0, 1):
            assert not snap[i].A.any() and not snap[i].G_prev.any()
    # the oracle with alpha = 0 is Muon; compare M, O and the update, not A / G_prev
    hp0 = wl.HParams(alpha=0.0)
    ref = H.run_oracle_for(weights, grads, hp0, [0, 1])
    for k, snap in enumerate(hist):
        for i in (0, 1):
            assert H.rel_max(snap[i].M, ref[i][k]["M"]) <= H.TOL_STATE
            assert H.rel_fro(snap[i].O, ref[i][k]["O"]) <= H.TOL_NS_BF16
            want = H.expected_update(snap[i].W_before, ref[i][k]["O"], hp0, False)
            assert H.rel_fro(snap[i].W - snap[i].W_before, want - snap[i].W_before) <= H.TOL_NS_BF16


def test_zero_and_nonfinite_gradients():
    say("[case] zero / nan gradients")
    shapes = [(40, 72), (72, 40), (33, 33)]
    weights = [wl.draw_weight(s, 51 + i, torch.float32) for i, s in enumerate(shapes)]
    g_ok = wl.GradientStream(shapes[2], 9).next()
    g_nan = torch.zeros(shapes[1])
    g_nan[3, 4] = float("nan")
    grads = [[torch.zeros(shapes[0]), g_nan, g_ok]]
    hp = wl.HParams()
    opt, dev_w, hist = H.run_gpu(weights, grads, hp, 0)
    st = opt.status()
    assert st == [B.MONA_STATUS_ZERO_NORM, B.MONA_STATUS_NONFINITE, 0]
    # zero momentum: O = 0, only the decoupled decay acts
    want = H.f64(weights[0]) * (1.0 - float(np.float32(hp.lr)) * float(np.float32(hp.weight_decay)))
    assert H.rel_max(hist[0][0].W, want) <= 1e-6
    assert not hist[0][0].O.any()
    # non-finite norm: the parameter is left untouched
    assert np.array_equal(hist[0][1].W, H.f64(weights[1]))
    # the healthy matrix is unaffected by its neighbours
    H.check_history(weights, grads, hp, hist, [2], H.TOL_NS_BF16, label="healthy")


def test_bf16_parameters_and_bf16_gradients():
    say("[case] bf16 params / grads")
    shapes = [(256, 384), (384, 256), (256, 384)]
    weights = [wl.draw_weight(s, 61 + i, torch.bfloat16) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 71 + i) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(3)]
    hp = wl.HParams()
    _, _, hist = H.run_gpu(weights, grads, hp, 0)
    H.check_history(weights, grads, hp, hist, [0, 1, 2], H.TOL_NS_BF16, label="bf16 W")
    grads16 = [[g.to(torch.bfloat16) for g in gs] for gs in grads]
    _, _, hist16 = H.run_gpu(weights, grads16, hp, 0)
    H.check_history(weights, grads16, hp, hist16, [0, 1, 2], H.TOL_NS_BF16, label="bf16 W+G")


def test_low_precision_state_variant():
    """Stored G_{k-1} and A_k in bf16 (Sec. 6.3, MONA-Lite): same recurrence, the stored values
    rounded to nearest even after each step."""
    say("[case] bf16 state")
    shapes = [(128, 200), (200, 128)]
    weights = [wl.draw_weight(s, 81 + i, torch.float32) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 91 + i) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(4)]
    hp = wl.HParams()
    _, _, hist = H.run_gpu(weights, grads, hp, 0, state_dtype=torch.bfloat16)
    # a bf16 rounding boundary can fall between the fp32 and the float64 value of A, so the
    # stored state may differ by one bf16 ulp on a few elements
    worst = H.check_history(weights, grads, hp, hist, [0, 1], H.TOL_NS_BF16, state_tol=2.0 ** -7,
                            state_dtype="bf16", label="lite")
    say("[worst]", worst)
    ref = H.run_oracle_for(weights, grads, hp, [0], "bf16")[0][-1]
    frac = (hist[-1][0].A != ref["A"]).mean()
    assert frac < 5e-3, f"{frac:.2e} of the stored A values differ from the oracle's bf16 values"


@pytest.mark.parametrize("state_dtype", [torch.float32, torch.bfloat16])
def test_one_buffer_form_of_the_acceleration_term(state_dtype):
    """No stored G_{k-1}: C_{k+1} = beta_a A_k - (1 - beta_a) G_k is carried and A_k = C_k + (1 - beta_a) G_k.
    Checked against the oracle's own one-buffer recurrence (which is pinned to Alg. 1), and against
    the two-buffer GPU path."""
    lite = state_dtype == torch.bfloat16
    say("[case] one-buffer form, state", state_dtype)
    w, weights, grads = inputs("ragged_mix", steps=4)
    hp = wl.HParams()
    watch = list(range(len(weights)))
    opt, _, hist = H.run_gpu(weights, grads, hp, 0, state_dtype=state_dtype, accel_form=B.MONA_ACCEL_ONE_BUFFER)
    worst = H.check_history(weights, grads, hp, hist, watch, H.TOL_NS_BF16, state_tol=2.0 ** -7 if lite else H.TOL_STATE,
                            state_dtype="bf16" if lite else "f32", label="one-buffer", accel_form="one_buffer")
    say("[worst]", worst)
    # the views of the arrays this form does not store say so
    for kind in (B.MONA_VIEW_G_PREV, B.MONA_VIEW_A):
        with pytest.raises(B.MonaError) as ei:
            opt.view(0, kind)
        assert ei.value.code == B.MONA_EUNSUPPORTED
    if not lite:
        # same M_k as Alg. 1's two-buffer form on the GPU (the two differ in rounding order only),
        # and as the float64 oracle of Alg. 1 itself
        opt2, _, hist2 = H.run_gpu(weights, grads, hp, 0)
        ref = H.run_oracle_for(weights, grads, hp, watch)
        beta = float(np.float32(hp.beta_a))
        for i in watch:
            assert H.rel_max(hist[-1][i].M, hist2[-1][i].M) <= 2 * H.TOL_STATE
            assert H.rel_max(hist[-1][i].M, ref[i][-1]["M"]) <= H.TOL_STATE
            # the carried bracket is beta_a A_k - (1 - beta_a) G_k of Alg. 1's own A_k
            want_c = beta * ref[i][-1]["A"] - (1 - beta) * H.f64(grads[-1][i])
            assert H.rel_max(hist[-1][i].C, want_c) <= H.TOL_STATE
        with pytest.raises(B.MonaError) as ei:
            opt2.view(0, B.MONA_VIEW_C)
        assert ei.value.code == B.MONA_EUNSUPPORTED
    # beta_a must not change between steps in this form
    dev_g = [g.to("cuda:0") for g in grads[0]]
    with pytest.raises(B.MonaError) as ei:
        opt.step(dev_g, dataclasses.replace(hp, beta_a=0.95))
    assert ei.value.code == B.MONA_EINVAL and opt.step_count() == 4


@pytest.mark.parametrize("state_dtype", [torch.float32, torch.bfloat16])
def test_streaming_gradient_with_caller_kept_slots(state_dtype):
    """Sec. 6.3's streaming variant: the library holds no G_{k-1}; it differences against the slot the
    caller keeps and leaves G_k there.  Same arithmetic as Alg. 1, so the oracle of Alg. 1 is the
    reference, and the stored-G_{k-1} GPU path must agree bit for bit."""
    lite = state_dtype == torch.bfloat16
    say("[case] streaming gradient, caller-kept slots, state", state_dtype)
    w, weights, grads = inputs("ragged_mix", steps=4)
    hp = dataclasses.replace(wl.HParams(), flags=B.MONA_FLAG_KEEP_O)
    watch = list(range(len(weights)))
    dev_w = [x.to("cuda:0").contiguous() for x in weights]
    opt = B.MonaOptimizer(dev_w, state_dtype=state_dtype, g_dtype=grads[0][0].dtype,
                          accel_form=B.MONA_ACCEL_CALLER_SLOT)
    slots = [torch.zeros(x.shape, dtype=state_dtype, device="cuda:0") for x in weights]
    hist = []
    for gk in grads:
        dev_g = [g.to("cuda:0").contiguous() for g in gk]
        before = {i: H.f64(dev_w[i]) for i in watch}
        opt.step(dev_g, hp, slots=slots)
        torch.cuda.synchronize()
        hist.append({i: H.Snapshot(H.f64(slots[i]), H.f64(opt.accel(i)), None, H.f64(opt.momentum(i)),
                                   float(opt.norm(i).item()), H.f64(opt.last_o(i)), H.f64(dev_w[i]), before[i])
                     for i in watch})
    worst = H.check_history(weights, grads, hp, hist, watch, H.TOL_NS_BF16,
                            state_tol=2.0 ** -7 if lite else H.TOL_STATE,
                            state_dtype="bf16" if lite else "f32", label="caller-slot")
    say("[worst]", worst)
    # bit-identical to the path that stores G_{k-1} itself
    opt2, dev_w2, hist2 = H.run_gpu(weights, grads, hp, 0, state_dtype=state_dtype)
    for i in watch:
        assert torch.equal(dev_w[i], dev_w2[i])
        assert torch.equal(opt.momentum(i), opt2.momentum(i)) and torch.equal(opt.accel(i), opt2.accel(i))
        assert torch.equal(slots[i], opt2.g_prev(i))
    assert opt2.arena_bytes - opt.arena_bytes >= sum(x.numel() for x in weights) * slots[0].element_size()
    # the array the caller keeps has no view; the plain entry point refuses such a state, and
    # the streaming one refuses a state that stores G_{k-1} itself
    with pytest.raises(B.MonaError) as ei:
        opt.view(0, B.MONA_VIEW_G_PREV)
    assert ei.value.code == B.MONA_EUNSUPPORTED
    dev_g = [g.to("cuda:0") for g in grads[0]]
    with pytest.raises(B.MonaError) as ei:
        opt.step(dev_g, hp)
    assert ei.value.code == B.MONA_EINVAL
    with pytest.raises(B.MonaError) as ei:
        opt2.step(dev_g, hp, slots=slots)
    assert ei.value.code == B.MONA_EINVAL
    with pytest.raises(ValueError):
        opt.step(dev_g, hp, slots=[s.t() for s in slots])
    assert opt.step_count() == 4 and opt2.step_count() == 4


def test_one_buffer_form_first_difference_flag_and_checkpoint():
    say("[case] one-buffer form: constant gradient with the first-difference flag; checkpoint")
    shapes = [(96, 160), (160, 96)]
    weights = [wl.draw_weight(s, 201 + i, torch.float32) for i, s in enumerate(shapes)]
    g = [wl.GradientStream(s, 211 + i).next() for i, s in enumerate(shapes)]
    hp = wl.HParams(flags=B.MONA_FLAG_FIRST_DIFF_ZERO)
    grads = [g, g, g]
    _, w_one, hist = H.run_gpu(weights, grads, hp, 0, accel_form=B.MONA_ACCEL_ONE_BUFFER)
    # A_k = 0 at every step: the momentum is plain Muon's, M_k = sum_j mu^(k-j) g
    mu = float(np.float32(hp.momentum))
    for i in range(2):
        want = (1 + mu + mu * mu) * H.f64(g[i])
        assert H.rel_max(hist[-1][i].M, want) <= H.TOL_STATE
        # and the carried bracket sits at its fixed point -(1 - beta_a) g
        beta = float(np.float32(hp.beta_a))
        assert H.rel_max(hist[-1][i].C, -(1 - beta) * H.f64(g[i])) <= H.TOL_STATE
    # checkpoint: {C, M} travels, the run continues bit-identically
    w, weights, grads = inputs("ragged_mix", steps=4)
    hp = wl.HParams()
    _, w_full, hist_full = H.run_gpu(weights, grads, hp, 0, accel_form=B.MONA_ACCEL_ONE_BUFFER)
    opt_a, w_a, _ = H.run_gpu(weights, grads[:2], hp, 0, accel_form=B.MONA_ACCEL_ONE_BUFFER)
    blob = opt_a.export_state()
    torch.cuda.synchronize()
    w_b = [t.clone() for t in w_a]
    opt_b = B.MonaOptimizer(w_b, accel_form=B.MONA_ACCEL_ONE_BUFFER)
    opt_b.import_state(blob, 2)
    for k in (2, 3):
        opt_b.step([x.to("cuda:0") for x in grads[k]], hp)
    torch.cuda.synchronize()
    for i in range(len(weights)):
        assert torch.equal(w_b[i], w_full[i]), f"matrix {i} differs after resume"
        assert torch.equal(opt_b.carry(i), torch.from_numpy(hist_full[-1][i].C).float().cuda())
    # a two-buffer checkpoint does not fit a one-buffer state
    opt_two = B.MonaOptimizer([t.clone() for t in w_a])
    with pytest.raises(B.MonaError) as ei:
        opt_b.import_state(opt_two.export_state(), 0)
    assert ei.value.code == B.MONA_ESHAPE


def test_checkpoint_round_trip_and_determinism():
    say("[case] checkpoint / determinism")
    w, weights, grads = inputs("ragged_mix", steps=4)
    hp = wl.HParams()
    # uninterrupted run
    _, w_full, hist_full = H.run_gpu(weights, grads, hp, 0)
    # second identical run: bitwise the same (no atomics, fixed reduction order)
    _, w_again, hist_again = H.run_gpu(weights, grads, hp, 0)
    for i in range(len(weights)):
        assert torch.equal(w_full[i], w_again[i])
        assert np.array_equal(hist_full[-1][i].M, hist_again[-1][i].M)
        assert hist_full[-1][i].norm == hist_again[-1][i].norm
    # two steps, export, import into a fresh state, two more steps
    opt_a, w_a, _ = H.run_gpu(weights, grads[:2], hp, 0)
    blob = opt_a.export_state()
    torch.cuda.synchronize()
    assert opt_a.step_count() == 2
    w_b = [t.clone() for t in w_a]
    opt_b = B.MonaOptimizer(w_b)
    opt_b.import_state(blob, 2)
    hp_keep = dataclasses.replace(hp, flags=B.MONA_FLAG_KEEP_O)
    for k in (2, 3):
        opt_b.step([g.to("cuda:0") for g in grads[k]], hp_keep)
    torch.cuda.synchronize()
    assert opt_b.step_count() == 4
    for i in range(len(weights)):
        assert torch.equal(w_b[i], w_full[i]), f"matrix {i} differs after resume"
        assert torch.equal(opt_b.momentum(i), torch.from_numpy(hist_full[-1][i].M).float().cuda())


def test_step_captured_in_a_hip_graph_replays_like_eager_steps():
    """mona_step records kernel launches only (no memset, no event, no table upload when the pointers are
    those of the previous call), so a caller may capture it; every replay must equal the eager step."""
    say("[case] HIP graph capture")
    w, weights, grads = inputs("ragged_mix", steps=6)
    hp = wl.HParams()
    dev = "cuda:0"
    w_eager = [t.to(dev).contiguous() for t in weights]
    opt_e = B.MonaOptimizer(w_eager)
    w_graph = [t.to(dev).contiguous() for t in weights]
    opt_g = B.MonaOptimizer(w_graph)
    static = [g.to(dev).contiguous() for g in grads[0]]
    # step 1 eagerly on both (uploads the graph optimizer's pointer table)
    opt_e.step([g.to(dev) for g in grads[0]], hp)
    opt_g.step(static, hp)
    torch.cuda.synchronize()
    # capture one step reading the static gradient buffers; capture only records, nothing runs
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        opt_g.step(static, hp)
    torch.cuda.synchronize()
    assert opt_g.step_count() == 2          # the host-side counter counts calls, not replays
    for k in range(1, 6):
        for dst, src in zip(static, grads[k]):
            dst.copy_(src)                      # eager work between the replays
        opt_e.step([g.to(dev) for g in grads[k]], hp)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(len(weights)):
            assert torch.equal(w_graph[i], w_eager[i]), f"replay {k}, matrix {i}: parameters differ"
            assert torch.equal(opt_g.momentum(i), opt_e.momentum(i)), f"replay {k}, matrix {i}: M differs"
            assert torch.equal(opt_g.accel(i), opt_e.accel(i)), f"replay {k}, matrix {i}: A differs"
            assert torch.equal(opt_g.g_prev(i), opt_e.g_prev(i)), f"replay {k}, matrix {i}: G_prev differs"


def test_step_rejects_changed_matrix_list():
    w = [torch.zeros(64, 64, device="cuda:0"), torch.zeros(64, 32, device="cuda:0")]
    opt = B.MonaOptimizer(w)
    hp = B.make_hparams(wl.HParams())
    g = [torch.zeros_like(x) for x in w]
    bad = B.make_matrices([w[1], w[0]], [g[1], g[0]])
    with pytest.raises(B.MonaError) as ei:
        B.mona_step(opt.state, bad, 2, hp, 0)
    assert ei.value.code == B.MONA_ESHAPE
    with pytest.raises(B.MonaError) as ei:
        B.mona_step(opt.state, B.make_matrices(w[:1], g[:1]), 1, hp, 0)
    assert ei.value.code == B.MONA_ESHAPE
    hp_bad = B.make_hparams(wl.HParams(momentum=1.0))
    with pytest.raises(B.MonaError) as ei:
        B.mona_step(opt.state, B.make_matrices(w, g), 2, hp_bad, 0)
    assert ei.value.code == B.MONA_EINVAL
    mis = B.make_matrices(w, g)
    mis[0].g = g[0].data_ptr() + 4
    with pytest.raises(B.MonaError) as ei:
        B.mona_step(opt.state, mis, 2, hp, 0)
    assert ei.value.code == B.MONA_EINVAL
    assert opt.step_count() == 0


# --------------------------------------------------------------------------------------------
# (configs[1..4] at full size and their stated step counts: tests/test_gpu_full_size.py)
# --------------------------------------------------------------------------------------------
def test_square_4096_against_the_svd_closed_form():
    """The largest short side of the BASELINE shapes, 4096 x 4096, is beyond a float64 Newton-Schulz on
    the host.  What the iteration computes has a closed form, though: O = U diag(p^T(sigma_i / ||M||_F)) V^T
    with p(s) = a s + b s^3 + c s^5 applied T times to the singular values of M (the oracle itself is pinned
    to it on small matrices).  M_1 comes from the oracle's elementwise step on the host; the eigendecomposition
    of M M^T is a library routine run in float64 (on the GPU, as a fast LAPACK); nothing expected here comes
    from the HIP path."""
    say("[case] 4096 x 4096 against the SVD closed form")
    dev = "cuda:0"
    shape = (4096, 4096)
    # four of them, as in configs[3], so that the products run on the large-tile kernel
    weights = [wl.draw_weight(shape, 7100 + i, torch.bfloat16, dev) for i in range(4)]
    grads = [wl.GradientStream(shape, 7200 + i, dev).next() for i in range(4)]
    hp = dataclasses.replace(wl.HParams(), flags=B.MONA_FLAG_KEEP_O)
    opt = B.MonaOptimizer(weights)
    opt.step(grads, hp)
    torch.cuda.synchronize()
    ohp = H.oracle_hp(hp)
    for i in (0, 3):
        o = orc.MonaOracle(shape)
        o.elementwise(H.f64(grads[i]), ohp)
        assert H.rel_max(H.f64(opt.momentum(i)), o.M) <= H.TOL_STATE
        M = torch.from_numpy(o.M).to(dev)                       # float64
        fro = torch.linalg.norm(M)
        lam, U = torch.linalg.eigh(M @ M.T)
        sigma = lam.clamp_min(0).sqrt() / fro                   # singular values of X_0
        s = sigma.clone()
        for _ in range(ohp.ns_steps):
            s = ohp.ns_a * s + ohp.ns_b * s ** 3 + ohp.ns_c * s ** 5
        # O = U diag(p^T(sigma)) V^T with V^T = diag(1 / (sigma fro)) U^T M
        O_ref = (U * (s / (sigma * fro))) @ (U.T @ M)
        O = opt.last_o(i).double()
        err = float(torch.linalg.norm(O - O_ref) / torch.linalg.norm(O_ref))
        say(f"[closed form] matrix {i}: sigma in [{float(sigma.min()):.3e}, {float(sigma.max()):.3e}], "
            f"p^T(sigma) in [{float(s.min()):.4f}, {float(s.max()):.4f}], O rel Fro err {err:.3e}")
        assert float(sigma.min()) > 1e-7                        # the closed form divides by sigma
        assert err <= H.TOL_NS_BF16
        # and the parameter moved by -eta (gamma O + lambda W) from the value it had
        W0 = wl.draw_weight(shape, 7100 + i, torch.bfloat16, dev).double()
        gamma = ohp.gamma_coeff * float(np.sqrt(max(shape)))
        dW_ref = -ohp.lr * (gamma * O_ref + ohp.weight_decay * W0)
        dW = weights[i].double() - W0
        # the stored parameter is bf16: its rounding (half an ulp of values around 0.02) is part of dW
        rounding = float(torch.linalg.norm((W0 + dW_ref).to(torch.bfloat16).double() - (W0 + dW_ref)) /
                         torch.linalg.norm(dW_ref))
        e_upd = float(torch.linalg.norm(dW - dW_ref) / torch.linalg.norm(dW_ref))
        say(f"[closed form] matrix {i}: update rel Fro err {e_upd:.3e} (bf16 rounding of W alone {rounding:.3e})")
        assert e_upd <= H.TOL_NS_BF16          # no allowance for the parameter's own rounding


def test_mixed_large_and_small_groups_on_several_streams():
    """One group whose launches cover the chip twice over (it stays on the caller's stream) next to small
    groups that run on the side streams, some with the large-tile kernel, some with the 128-tile and fp32
    kernels: every lane's result against the oracle, and the same bits as a single-stream run."""
    say("[case] mixed lanes")
    dev = "cuda:0"
    shapes = [(1024, 2048)] * 156 + [(512, 4096)] * 2 + [(768, 768)] + [(4096, 512)] * 2 + [(100, 300), (40, 64)]
    big = 156           # 156 x 10 Gram tiles = 1560: a group that keeps the caller's stream to itself
    sample = [3, big, big + 2, big + 3, big + 5, big + 6]
    weights = [wl.draw_weight(s, 9000 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
    grads = [[wl.GradientStream(s, 9500 + i, dev).next() for i, s in enumerate(shapes)] for _ in range(2)]
    hp = wl.HParams()
    w_cpu = [x.cpu() if i in sample else x for i, x in enumerate(weights)]
    opt, dev_w, hist = H.run_gpu(weights, grads, hp, 0, watch=sample)
    worst = H.check_history(w_cpu, grads, hp, hist, sample, H.TOL_NS_BF16, label="mixed lanes")
    say("[worst]", worst)
    assert opt.status() == [0] * len(shapes)
    # the same run on the caller's stream alone: the lanes change when kernels run, never what they
    # compute.  (The small groups may pick a different tile size without company, so compare against
    # the oracle-checked run through the parameters only where the plan is the same: the large group.)
    w1 = [wl.draw_weight(s, 9000 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
    opt1 = B.MonaOptimizer(w1, max_streams=1)
    for gs in grads:
        opt1.step(gs, hp)
    torch.cuda.synchronize()
    for i in range(big):
        assert torch.equal(w1[i], dev_w[i]), f"matrix {i}: one stream and several streams disagree"
    for i in range(big, len(shapes)):
        d = (w1[i].float() - dev_w[i].float()).norm() / (dev_w[i].float().norm() + 1e-30)
        assert float(d) <= 1e-3, (i, float(d))


def test_profiling_and_plan_reports():
    """The timing hooks the benchmark relies on: phase events, per-launch events, plan figures."""
    say("[case] profiling hooks")
    w = wl.WORKLOADS["moe_bank_e64"]
    shapes = w.shapes()[:6] + w.shapes()[-6:]          # 6 tall + 6 wide 2048x1024 matrices
    dev = "cuda:0"
    weights = [wl.draw_weight(s, 500 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
    grads = [wl.GradientStream(s, 600 + i, dev).next() for i, s in enumerate(shapes)]
    hp = wl.HParams()
    # the fused schedule: per group Gram + 9 p x p products + apply for
    # the chunk of three iterations, Gram + 5 + apply for the chunk of two; fewer flop than the literal one
    fused = B.MonaOptimizer(weights, ns_schedule=B.MONA_NS_SCHEDULE_FUSED).plan_info(hp.ns_steps)
    assert fused["ns_launches"] == 2 * (11 + 7)
    opt = B.MonaOptimizer(weights, ns_schedule=B.MONA_NS_SCHEDULE_LITERAL)
    plan = opt.plan_info(hp.ns_steps)
    assert plan["ns_launches"] == 2 * 3 * hp.ns_steps            # two shape groups
    assert fused["ns_flops_issued"] < plan["ns_flops_issued"]
    n_elem = sum(a * b for a, b in shapes)
    assert plan["elementwise_bytes"] == n_elem * 30
    sym = sum(hp.ns_steps * (3.0 * min(s) ** 2 * max(s) + min(s) ** 3) for s in shapes)
    dense = sum(hp.ns_steps * (4.0 * min(s) ** 2 * max(s) + 2.0 * min(s) ** 3) for s in shapes)
    assert sym <= plan["ns_flops_issued"] <= dense               # triangle plus full diagonal tiles
    with pytest.raises(B.MonaError):
        opt.last_step_times()                                    # nothing profiled yet
    opt.set_profiling(2)
    opt.step(grads, hp)
    t = opt.last_step_times()
    assert all(x >= 0 for x in t) and t[3] > 0 and abs(t[0] + t[1] + t[2] - t[3]) < 0.05 * t[3] + 0.05
    recs = opt.last_step_launches()
    assert len(recs) == plan["ns_launches"]
    assert sorted({r["kind"] for r in recs}) == [0, 1, 2]
    assert abs(sum(r["flops"] for r in recs) - plan["ns_flops_issued"]) < 1e-6 * plan["ns_flops_issued"]
    assert all(r["ms"] > 0 for r in recs)
    # the mean over the steps profiled since set_profiling: more steps than the library keeps marks for
    opt.set_profiling(1)
    with pytest.raises(B.MonaError):
        opt.mean_step_times()
    singles = []
    for _ in range(40):
        opt.step(grads, hp)
        singles.append(opt.last_step_times())
    mean, n = opt.mean_step_times()
    assert n == 32
    for i in range(4):
        want = sum(x[i] for x in singles[-32:]) / 32
        assert abs(mean[i] - want) <= 1e-3 * want + 1e-4
    opt.set_profiling(0)
    opt.step(grads, hp)
    torch.cuda.synchronize()
    assert opt.step_count() == 42
