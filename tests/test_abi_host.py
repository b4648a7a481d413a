"""Host-side checks of the C ABI that need no GPU: the shared library loads, exports every
function include/mona.h declares, sizes arenas and rejects bad arguments before touching HIP."""
import ctypes as C
import os
import re

import pytest
import torch

from paper_2605_26842_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mona.h")

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libmona.so not built")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mona_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = B.load_library()
    names = declared_functions()
    assert "mona_init_state" in names and "mona_step" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mona.h but not exported"
    assert sorted(B.EXPORTED) == names
    assert lib.mona_version().decode().startswith("libmona")


def shapes(*mn, w=B.MONA_BF16, g=B.MONA_F32):
    arr = (B.mona_matrix * len(mn))()
    for i, (m, n) in enumerate(mn):
        arr[i].m, arr[i].n, arr[i].w_dtype, arr[i].g_dtype = m, n, w, g
    return arr


def test_state_size_accounts_for_state_and_workspace():
    one = B.mona_state_size(shapes((256, 512)), 1)
    n = 256 * 512
    # 3 fp32 state arrays + two bf16 working copies + two 256x256 bf16 squares, plus small tables
    assert one >= n * 12 + 2 * n * 2 + 2 * 256 * 256 * 2
    assert one < n * 12 + 2 * n * 2 + 2 * 256 * 256 * 2 + 64 * 1024
    lite = B.mona_state_size(shapes((256, 512)), 1, B.mona_options(0, B.MONA_BF16))
    assert one - lite == 2 * n * 2                      # G_prev and A stored in bf16
    f32 = B.mona_state_size(shapes((256, 512)), 1, B.mona_options(1, B.MONA_F32))
    assert f32 - one == 2 * n * 2 + 2 * 256 * 256 * 2   # fp32 working copies
    # one-buffer form of the acceleration term: no previous-gradient array
    single = B.mona_state_size(shapes((256, 512)), 1, B.mona_options(0, B.MONA_F32, B.MONA_ACCEL_ONE_BUFFER))
    assert one - single == n * 4
    single_lite = B.mona_state_size(shapes((256, 512)), 1, B.mona_options(0, B.MONA_BF16, B.MONA_ACCEL_ONE_BUFFER))
    assert one - single_lite == n * 4 + n * 2           # 6 instead of 12 state bytes per element
    # streaming variant: the caller keeps G_{k-1}, the arena is as small as the one-buffer form's
    kept = B.mona_state_size(shapes((256, 512)), 1, B.mona_options(0, B.MONA_F32, B.MONA_ACCEL_CALLER_SLOT))
    assert kept == single
    # padding: 100 x 300 works on 128 x 384 copies
    rag = B.mona_state_size(shapes((100, 300)), 1)
    assert rag >= 100 * 300 * 12 + 2 * 128 * 384 * 2 + 2 * 128 * 128 * 2
    # the large MoE layer of the benchmark: ~45 GB of state, ~60 GB in all
    layer = shapes(*([(4096, 4096)] * 4 + [(4096, 1536)] * 256 + [(1536, 4096)] * 128))
    elems = 4 * 4096 * 4096 + 384 * 4096 * 1536
    literal = B.mona_state_size(layer, 388, B.mona_options(ns_schedule=B.MONA_NS_SCHEDULE_LITERAL))
    assert elems * 12 < literal < elems * 12 * 1.6
    # the fused Newton-Schulz schedule (the automatic choice for the 384 expert matrices: long side 4096,
    # short side 1536) keeps six p x p working matrices per matrix instead of two
    total = B.mona_state_size(layer, 388)
    assert total - literal == 384 * 4 * 1536 * 1536 * 2
    fused = B.mona_state_size(layer, 388, B.mona_options(ns_schedule=B.MONA_NS_SCHEDULE_FUSED))
    assert fused - total == 4 * 4 * 4096 * 4096 * 2
    # the automatic choice fuses 2048 x 8192 (chunks of three, then two) and 1024 x 2048 (pairs) and leaves
    # 512 x 4096 (short side too small to gain) and squares literal
    for shape, is_fused in (((1024, 2048), True), ((512, 4096), False), ((2048, 8192), True), ((8192, 2048), True),
                            ((1536, 1536), False), ((768, 256), False)):
        auto = B.mona_state_size(shapes(shape), 1)
        lit = B.mona_state_size(shapes(shape), 1, B.mona_options(ns_schedule=B.MONA_NS_SCHEDULE_LITERAL))
        assert (auto > lit) == is_fused, shape
    with pytest.raises(B.MonaError):
        B.mona_state_size(layer, 388, B.mona_options(ns_schedule=4))


def rc_of(fn, *args):
    return fn(*args), B.load_library().mona_last_error().decode()


def test_state_size_properties_on_random_shape_lists():
    """Properties of the arena layout that hold for any list of matrices: it holds at least the state and
    the padded working copies, does not depend on the order of the matrices, and shrinks by exactly the
    previous-gradient arrays when the caller keeps them or the one-buffer form is chosen."""
    import random
    rng = random.Random(20260527)
    pad = lambda v: (v + 127) // 128 * 128
    for _ in range(40):
        k = rng.randint(1, 12)
        base = [(rng.choice([1, 3, 64, 65, 100, 128, 256, 300, 512, 777, 1024]),
                 rng.choice([1, 5, 64, 96, 128, 130, 256, 384, 640, 1000, 2048])) for _ in range(rng.randint(1, 4))]
        mn = [rng.choice(base) for _ in range(k)]
        two = B.mona_state_size(shapes(*mn), k)
        elems = sum(m * n for m, n in mn)
        work = sum(2 * pad(m) * pad(n) * (4 if min(m, n) <= 64 else 2) for m, n in mn)
        assert two >= 12 * elems + work
        assert two <= 12 * elems + 3 * work + 4096 * k + 65536       # X x 2, S, B (S, B <= X), tables, alignment
        shuffled = mn[:]
        rng.shuffle(shuffled)
        assert B.mona_state_size(shapes(*shuffled), k) == two
        one = B.mona_state_size(shapes(*mn), k, B.mona_options(0, B.MONA_F32, B.MONA_ACCEL_ONE_BUFFER))
        kept = B.mona_state_size(shapes(*mn), k, B.mona_options(0, B.MONA_F32, B.MONA_ACCEL_CALLER_SLOT))
        assert one == kept
        aligned = sum((m * n * 4 + 255) // 256 * 256 for m, n in mn)
        assert two - one == aligned
        assert two % 256 == 0 and one % 256 == 0


def test_bad_arguments_are_rejected_on_the_host():
    lib = B.load_library()
    out = C.c_size_t(0)
    rc, msg = rc_of(lib.mona_state_size, None, 1, None, C.byref(out))
    assert rc == B.MONA_EINVAL and "NULL" in msg
    rc, _ = rc_of(lib.mona_state_size, shapes((4, 4)), 0, None, C.byref(out))
    assert rc == B.MONA_EINVAL
    rc, msg = rc_of(lib.mona_state_size, shapes((0, 4)), 1, None, C.byref(out))
    assert rc == B.MONA_EINVAL and ">= 1" in msg
    rc, msg = rc_of(lib.mona_state_size, shapes((65536, 65536)), 1, None, C.byref(out))
    assert rc == B.MONA_EINVAL and "2^31" in msg
    rc, msg = rc_of(lib.mona_state_size, shapes((2 ** 31 - 1, 1)), 1, None, C.byref(out))
    assert rc == B.MONA_EINVAL and "2^30" in msg
    # a long thin matrix below both limits is sized without overflow: 128 x 2^30 padded copies
    assert lib.mona_state_size(shapes((1, 2 ** 30)), 1, None, C.byref(out)) == B.MONA_OK
    assert out.value > 2 * 128 * 2 ** 30 * 2
    rc, _ = rc_of(lib.mona_state_size, shapes((4, 4), w=7), 1, None, C.byref(out))
    assert rc == B.MONA_EINVAL
    rc, _ = rc_of(lib.mona_state_size, shapes((4, 4)), 1, C.byref(B.mona_options(2, 0)), C.byref(out))
    assert rc == B.MONA_EINVAL
    rc, msg = rc_of(lib.mona_state_size, shapes((4, 4)), 1, C.byref(B.mona_options(0, 0, 3)), C.byref(out))
    assert rc == B.MONA_EINVAL and "accel_form" in msg
    rc, msg = rc_of(lib.mona_state_size, shapes((4, 4)), 1,
                    C.byref(B.mona_options(0, 0, 0, 0, 0, 0, (C.c_int32 * 2)(0, 1))), C.byref(out))
    assert rc == B.MONA_EINVAL and "reserved" in msg
    rc, msg = rc_of(lib.mona_state_size, shapes((4, 4)), 1, C.byref(B.mona_options(0, 0, 0, 9)), C.byref(out))
    assert rc == B.MONA_EINVAL and "max_streams" in msg
    rc, _ = rc_of(lib.mona_state_size, shapes((4, 4)), 1, None, None)
    assert rc == B.MONA_EINVAL
    # init: argument errors are reported before any HIP call
    handle = C.c_void_p(0)
    rc, msg = rc_of(lib.mona_init_state, shapes((4, 4)), 1, None, None, 1 << 20, None, C.byref(handle))
    assert rc == B.MONA_EINVAL and "arena" in msg
    rc, msg = rc_of(lib.mona_init_state, shapes((4, 4)), 1, None, 0x1001, 1 << 20, None, C.byref(handle))
    assert rc == B.MONA_EINVAL and "aligned" in msg
    rc, msg = rc_of(lib.mona_init_state, shapes((256, 512)), 1, None, 0x10000, 1024, None, C.byref(handle))
    assert rc == B.MONA_ENOMEM and "too small" in msg
    assert handle.value in (None, 0)
    # step / view / free on a NULL state
    hp = B.mona_hparams()
    assert lib.mona_step(None, shapes((4, 4)), 1, C.byref(hp), None) == B.MONA_EINVAL
    assert lib.mona_step_streaming(None, shapes((4, 4)), None, 1, C.byref(hp), None) == B.MONA_EINVAL
    assert lib.mona_state_view(None, 0, 0, None) == B.MONA_EINVAL
    assert lib.mona_free_state(None) == B.MONA_OK
    with pytest.raises(B.MonaError):
        B.mona_state_size(shapes((0, 0)), 1)


def test_binding_refuses_cpu_tensors_and_bad_layouts():
    w = torch.zeros(4, 6)
    with pytest.raises(RuntimeError, match="GPU"):
        B.MonaOptimizer([w])
    with pytest.raises(ValueError):
        B.make_matrices([torch.zeros(4, 6).t()])
    with pytest.raises(TypeError):
        B.make_matrices([torch.zeros(4, 6, dtype=torch.float16)])
    with pytest.raises(FileNotFoundError):
        B.load_library("/nonexistent/libmona.so")


def vecs(*n, w=B.MONA_BF16, g=B.MONA_F32):
    arr = (B.mona_vector * len(n))()
    for i, k in enumerate(n):
        arr[i].n, arr[i].w_dtype, arr[i].g_dtype = k, w, g
    return arr


def test_adamw_host_side_checks():
    lib = B.load_library()
    # two fp32 moments per element, each array padded to 256 bytes, plus small tables
    one = B.mona_adamw_state_size(vecs(4096), 1)
    assert 2 * 4096 * 4 <= one < 2 * 4096 * 4 + 4096
    two = B.mona_adamw_state_size(vecs(4096, 5), 2)
    assert two - one >= 2 * 256 and two - one < 4096
    out = C.c_size_t(0)
    rc, msg = rc_of(lib.mona_adamw_state_size, None, 1, C.byref(out))
    assert rc == B.MONA_EINVAL and "NULL" in msg
    rc, msg = rc_of(lib.mona_adamw_state_size, vecs(0), 1, C.byref(out))
    assert rc == B.MONA_EINVAL and ">= 1" in msg
    rc, _ = rc_of(lib.mona_adamw_state_size, vecs(8, w=3), 1, C.byref(out))
    assert rc == B.MONA_EINVAL
    handle = C.c_void_p(0)
    rc, msg = rc_of(lib.mona_adamw_init_state, vecs(8), 1, None, 1 << 20, None, C.byref(handle))
    assert rc == B.MONA_EINVAL and "arena" in msg
    rc, msg = rc_of(lib.mona_adamw_init_state, vecs(1 << 20), 1, 0x10000, 1024, None, C.byref(handle))
    assert rc == B.MONA_ENOMEM and "too small" in msg
    hp = B.mona_adamw_hparams(1e-3, 0.9, 0.95, 1e-8, 0.1)
    assert lib.mona_adamw_step(None, vecs(8), 1, C.byref(hp), None) == B.MONA_EINVAL
    assert lib.mona_adamw_free_state(None) == B.MONA_OK
    with pytest.raises(RuntimeError):
        B.AdamWOptimizer([torch.zeros(8)])
