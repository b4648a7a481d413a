"""The entry point that allocates nothing, mona_step_noalloc, against mona_step on a one-matrix state:
same kernels, same plan, so every output must agree bit for bit.  Two calls in a row, the second on a
smaller matrix (the static workspace keeps the first call's contents)."""
import ctypes as C

import pytest
import torch

from paper_2605_26842_amd import binding as B
from paper_2605_26842_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_pair(shape, seed, steps, w_dtype, state_dtype, hp):
    dev = "cuda:0"
    w0 = wl.draw_weight(shape, seed, w_dtype, dev)
    stream = wl.GradientStream(shape, seed + 1, dev)
    grads = [stream.next() for _ in range(steps)]
    # reference: the existing entry point on a state of this one matrix
    w_ref = w0.clone()
    opt = B.MonaOptimizer([w_ref], state_dtype=state_dtype)
    for g in grads:
        opt.step([g], hp)
    torch.cuda.synchronize()
    # the entry point under test: the caller keeps G_{k-1}, A and M
    w = w0.clone()
    g_prev = torch.zeros(shape, dtype=state_dtype, device=dev)
    acc = torch.zeros(shape, dtype=state_dtype, device=dev)
    mom = torch.zeros(shape, dtype=torch.float32, device=dev)
    opts = B.mona_options(0, B._dtype_code(state_dtype), B.MONA_ACCEL_TWO_BUFFER, 0, 0, 0, (C.c_int32 * 2)())
    hpc = B.make_hparams(hp)
    s = torch.cuda.current_stream().cuda_stream
    for k, g in enumerate(grads):
        mats = B.make_matrices([w], [g])
        B.mona_step_noalloc(mats, opts, g_prev.data_ptr(), acc.data_ptr(), mom.data_ptr(), hpc, k, s)
    torch.cuda.synchronize()
    assert torch.equal(w, w_ref), f"{shape}: parameters differ"
    assert torch.equal(mom, opt.momentum(0)), f"{shape}: M differs"
    assert torch.equal(acc, opt.accel(0)), f"{shape}: A differs"
    assert torch.equal(g_prev, opt.g_prev(0)), f"{shape}: G_prev differs"
    assert not torch.equal(w, w0)
    assert torch.isfinite(w.float()).all()


def test_noalloc_matches_mona_step_twice_in_a_row():
    hp = wl.HParams()
    print("[case] noalloc 512 x 1408 bf16 parameters, 3 steps", flush=True)
    run_pair((512, 1408), 4100, 3, torch.bfloat16, torch.float32, hp)
    print("[case] noalloc 130 x 70 fp32 parameters, bf16 state, 2 steps (smaller, after the larger one)", flush=True)
    run_pair((130, 70), 4200, 2, torch.float32, torch.bfloat16, hp)
    print("[case] noalloc 96 x 200, T = 0", flush=True)
    run_pair((96, 200), 4300, 2, torch.float32, torch.float32, wl.HParams(ns_steps=0))


def test_noalloc_rejects_what_does_not_fit():
    dev = "cuda:0"
    shape = (2048, 8192)
    w = torch.zeros(shape, dtype=torch.bfloat16, device=dev)
    g = torch.zeros(shape, dtype=torch.float32, device=dev)
    st = torch.zeros(shape, dtype=torch.float32, device=dev)
    with pytest.raises(B.MonaError) as ei:
        B.mona_step_noalloc(B.make_matrices([w], [g]), None, st.data_ptr(), st.data_ptr(), st.data_ptr(),
                            B.make_hparams(wl.HParams()), 0, 0)
    assert ei.value.code == B.MONA_ENOMEM and "static scratch" in str(ei.value)
    opts = B.mona_options(0, 0, B.MONA_ACCEL_ONE_BUFFER, 0, 0, 0, (C.c_int32 * 2)())
    small = torch.zeros((64, 64), dtype=torch.float32, device=dev)
    with pytest.raises(B.MonaError) as ei:
        B.mona_step_noalloc(B.make_matrices([small], [small]), opts, small.data_ptr(), small.data_ptr(),
                            small.data_ptr(), B.make_hparams(wl.HParams()), 0, 0)
    assert ei.value.code == B.MONA_EUNSUPPORTED
    with pytest.raises(B.MonaError) as ei:
        B.mona_step_noalloc(B.make_matrices([small], [small]), None, 0, small.data_ptr(), small.data_ptr(),
                            B.make_hparams(wl.HParams()), 0, 0)
    assert ei.value.code == B.MONA_EINVAL
