"""GPU parity of the two layouts of the Newton-Schulz iterations (Eq. newton_schulz): the literal one
(Gram, poly, apply per iteration) and the fused one (chunks of iterations advanced on the p x p side).
Both compute the same polynomial of X_0; each is held to the same bound against the float64 oracle."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2605_26842_amd import binding as B
from paper_2605_26842_amd import workloads as wl
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("schedule", [B.MONA_NS_SCHEDULE_LITERAL, B.MONA_NS_SCHEDULE_FUSED, B.MONA_NS_SCHEDULE_PAIRS])
@pytest.mark.parametrize("T", [2, 3, 4, 5])
def test_both_schedules_against_the_oracle(schedule, T):
    """Shapes that take every kernel: 256 x 256 tiles (12 x 512 x 1536 wide and tall), 128 x 128 tiles
    (ragged 300 x 900, one 640 x 1280), and a square.  Forcing the fused schedule on a square saves nothing and
    costs accuracy (a square Gaussian matrix has singular values down to zero, the case in which advancing the
    Gram matrix on its own is least accurate: measured 3.1e-2), which is why the automatic choice never does
    it; there the test only demands the right matrix to a looser bound."""
    say(f"[case] schedule={schedule} T={T}")
    shapes = [(512, 1536)] * 12 + [(1536, 512)] * 12 + [(300, 900), (900, 300), (640, 1280), (384, 384)]
    sample = [0, 11, 12, 23, 24, 25, 26, 27]
    dev = "cuda:0"
    weights = [wl.draw_weight(s, 3000 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 3100 + i, dev) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(2)]
    hp = wl.HParams(ns_steps=T)
    w_cpu = [x.cpu() if i in sample else x for i, x in enumerate(weights)]
    opt, _, hist = H.run_gpu(weights, grads, hp, 0, watch=sample, ns_schedule=schedule)
    strict = sample if schedule == B.MONA_NS_SCHEDULE_LITERAL else sample[:-1]
    worst = H.check_history(w_cpu, grads, hp, hist, strict, H.TOL_NS_BF16, label=f"schedule {schedule} T {T}")
    say("[worst]", worst)
    if schedule != B.MONA_NS_SCHEDULE_LITERAL:
        ref = H.run_oracle_for(w_cpu, grads, hp, [27])[27]
        for k in range(2):
            e = H.rel_fro(hist[k][27].O, ref[k]["O"])
            say(f"[square, fused] step {k + 1}: O rel Fro err {e:.3e}")
            assert e <= 5e-2
    assert opt.status() == [0] * len(shapes)


def test_fused_schedule_on_ill_conditioned_momentum():
    """A momentum matrix with a steep spectrum (rank-deficient part plus noise five orders of magnitude
    smaller), where the bf16 products are least accurate.  No fixed bound holds here for either layout
    (the literal one is itself several per cent off the float64 oracle on such input); the fused layout
    must stay within a factor of the literal one's error."""
    say("[case] ill-conditioned input, both schedules")
    dev = "cuda:0"
    p, q, rk = 512, 1536, 128
    gen = torch.Generator(device="cpu").manual_seed(77)
    g = (torch.randn(p, rk, generator=gen) @ torch.randn(rk, q, generator=gen)) * (1e-3 / np.sqrt(rk)) \
        + torch.randn(p, q, generator=gen) * 1e-8
    shapes = [(p, q)] * 12
    errs = {}
    for schedule in (B.MONA_NS_SCHEDULE_LITERAL, B.MONA_NS_SCHEDULE_FUSED):
        weights = [wl.draw_weight(s, 3300 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
        grads = [[g.clone().to(dev) for _ in shapes]]
        hp = wl.HParams(alpha=0.0)
        opt, _, hist = H.run_gpu(weights, grads, hp, 0, watch=[5], ns_schedule=schedule)
        ref = H.run_oracle_for([w.cpu() for w in weights], grads, hp, [5])[5][0]
        errs[schedule] = H.rel_fro(hist[0][5].O, ref["O"])
    say("[ill-conditioned] O rel Fro err: literal %.3e, fused %.3e" % (errs[1], errs[2]))
    assert errs[2] <= 2.0 * errs[1] + 1e-2


def test_late_group_overlap_changes_timing_not_results():
    """mona_options.overlap = MONA_OVERLAP_LATE_GROUP: the elementwise pass of the group with the most elements
    runs on a CU-masked stream beside the products of the other group.  Same kernels on the same data, so
    every output must be bit-identical to the run without it; and the pass must really have left the common
    elementwise phase (its share of the step's first interval is gone)."""
    say("[case] late-group overlap")
    dev = "cuda:0"
    shapes = [(1024, 1024)] * 200 + [(512, 1536)] * 400
    run_stream = torch.cuda.Stream(dev)          # not the null stream: it would serialise the two passes
    results = {}
    with torch.cuda.stream(run_stream):
        grads = [[wl.GradientStream(s, 3500 + i, dev).next() for i, s in enumerate(shapes)] for _ in range(2)]
        for mode in (B.MONA_OVERLAP_OFF, B.MONA_OVERLAP_LATE_GROUP):
            weights = [wl.draw_weight(s, 3400 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
            opt = B.MonaOptimizer(weights, overlap=mode)
            opt.set_profiling(1)
            hp = wl.HParams()
            first = []
            for gs in grads + grads:
                opt.step(gs, hp)
                first.append(opt.last_step_times()[0])
            run_stream.synchronize()
            results[mode] = (weights, [opt.momentum(i).clone() for i in (0, 199, 200, 599)],
                             [opt.accel(i).clone() for i in (0, 199, 200, 599)], min(first[1:]), opt.status())
            del opt
    w0, m0, a0, t0, s0 = results[B.MONA_OVERLAP_OFF]
    w1, m1, a1, t1, s1 = results[B.MONA_OVERLAP_LATE_GROUP]
    say(f"[late-group overlap] elementwise interval before the products: {t0:.3f} ms without, {t1:.3f} ms with")
    assert s0 == s1 == [0] * len(shapes)
    for i in range(len(shapes)):
        assert torch.equal(w0[i], w1[i]), f"matrix {i}: parameters differ with the late-group overlap"
    for x, y in zip(m0 + a0, m1 + a1):
        assert torch.equal(x, y)
    assert t1 < 0.8 * t0


def test_the_papers_own_expert_shapes():
    """One matrix of each expert shape of the paper's three models (Sec. 6 model descriptions: hidden 768 with FFN
    256, hidden 1536 with FFN 1024, hidden 3072 with FFN 1024), tall and wide, in groups large enough for the
    large-tile kernel, three steps, against the oracle."""
    say("[case] the paper's expert shapes")
    dev = "cuda:0"
    base = [(768, 256), (256, 768), (1536, 1024), (1024, 1536), (3072, 1024), (1024, 3072)]
    shapes = [s for s in base for _ in range(16)]
    sample = [16 * j + (5 * j) % 16 for j in range(len(base))]
    weights = [wl.draw_weight(s, 3600 + i, torch.bfloat16, dev) for i, s in enumerate(shapes)]
    streams = [wl.GradientStream(s, 3700 + i, dev) for i, s in enumerate(shapes)]
    grads = [[st.next() for st in streams] for _ in range(3)]
    hp = wl.HParams(beta_a=0.98, alpha=-25.0)           # the pair reported for the 6B model
    w_cpu = [x.cpu() if i in sample else x for i, x in enumerate(weights)]
    opt, _, hist = H.run_gpu(weights, grads, hp, 0, watch=sample)
    worst = H.check_history(w_cpu, grads, hp, hist, sample, H.TOL_NS_BF16, label="paper shapes")
    say("[worst]", worst)
    assert opt.status() == [0] * len(shapes)
