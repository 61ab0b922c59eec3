"""CPU-only checks of the host side of the library: it loads, exports every
symbol the header declares, validates arguments, and its layout / byte
accounting agrees with the paper's tables."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_1905_13727_amd import binding as B
from paper_1905_13727_amd import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    hdr = open(os.path.join(ROOT, "include", "psgd.h")).read()
    names = re.findall(r"PSGD_API\s+[\w\s\*]+?\b(psgd_\w+)\s*\(", hdr)
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert B.status_string(B.PSGD_OK) == "ok"
    assert "invalid" in B.status_string(B.PSGD_EINVAL)
    assert B.status_string(77) == "unknown status"


@pytest.mark.parametrize("kwargs,status", [
    (dict(shapes=[(4, 4)], rank=0), B.PSGD_EINVAL),
    (dict(shapes=[(4, 4)], rank=2, workers=0), B.PSGD_EINVAL),
    (dict(shapes=[(0, 4)], rank=2), B.PSGD_EINVAL),
    (dict(shapes=[(4, -1)], rank=2), B.PSGD_EINVAL),
    (dict(shapes=[], rank=2), B.PSGD_EINVAL),
    (dict(shapes=[(4, 4)], rank=B.PSGD_MAX_RANK + 1), B.PSGD_EUNSUPPORTED),
    (dict(shapes=[(4, 4)], rank=2, grad_dtype=7), B.PSGD_EINVAL),
    # the matrix-core kernels (rank > 8) need row lengths that are multiples of 4, at most 2^20
    (dict(shapes=[(64, 650)], rank=16), B.PSGD_EUNSUPPORTED),
    (dict(shapes=[(8, (1 << 20) + 4)], rank=16), B.PSGD_EUNSUPPORTED),
    # vector-ALU kernels: a strip of 8 rows must stay below 2^31 bytes
    (dict(shapes=[(4, 68_000_000)], rank=2), B.PSGD_EUNSUPPORTED),
])
def test_invalid_plans(kwargs, status):
    with pytest.raises(B.PsgdError) as ei:
        B.Plan(**kwargs)
    assert ei.value.status == status


def test_null_pointers_are_rejected_without_a_gpu():
    lib = B.load_library()
    assert lib.psgd_plan_create(None, 1, 1, 1, 0, 0, None) == B.PSGD_EINVAL
    h = C.c_void_p()
    assert lib.psgd_plan_create(None, 1, 1, 1, 0, 0, C.byref(h)) == B.PSGD_EINVAL
    plan = B.Plan([(8, 8)], 2)
    assert lib.psgd_step(plan._h, None, None, None, None, None, None, None) == B.PSGD_EINVAL
    assert lib.psgd_compress(None, 1, 1, 1, 1, 1, None) == B.PSGD_EINVAL
    assert lib.psgd_decompress(plan._h, 1, 1, None, 1, 1, 1, None) == B.PSGD_EINVAL
    assert lib.psgd_iterate(plan._h, None, 1, 1, 1, None) == B.PSGD_EINVAL
    assert lib.psgd_iterate(None, 1, 1, 1, 1, None) == B.PSGD_EINVAL
    assert lib.psgd_step_update(plan._h, 1, 1, 1, 1, None, 1, 0.1, 0.9, 1, None) == B.PSGD_EINVAL     # no momentum buffer
    assert lib.psgd_step_update(plan._h, 1, 1, 1, 1, 1, 1, float("nan"), 0.9, 1, None) == B.PSGD_EINVAL  # NaN step size
    assert lib.psgd_decompress_update(plan._h, 1, 1, 1, 1, 1, None, 0.1, 0.9, 1, None) == B.PSGD_EINVAL
    # the one-call form of several iterations: a count outside 1 .. 64 is refused
    assert lib.psgd_step_iterations(plan._h, 1, 1, 1, 1, 1, 1, None, 0) == B.PSGD_EINVAL
    assert lib.psgd_step_iterations(plan._h, 1, 1, 1, 1, 1, 1, None, 65) == B.PSGD_EINVAL
    assert lib.psgd_step_iterations(plan._h, 1, 1, 1, 1, None, 1, None, 2) == B.PSGD_EINVAL
    # the step without allocation refuses a plan whose tables are not on a device yet (no GPU call is made for that)
    assert lib.psgd_step_static(plan._h, 1, 1, 1, 1, 1, None) == B.PSGD_EINVAL
    assert b"not on the device" in lib.psgd_plan_last_error(plan._h)
    assert lib.psgd_step_static(plan._h, 1, None, 1, 1, 1, None) == B.PSGD_EINVAL
    assert lib.psgd_plan_kept(plan._h, 3, None, None) == B.PSGD_EINVAL and lib.psgd_plan_kept(plan._h, 0, None, None) == B.PSGD_OK
    assert lib.psgd_plan_sizes(plan._h, None) == B.PSGD_EINVAL
    assert lib.psgd_plan_offsets(plan._h, 5, None, None, None, None) == B.PSGD_EINVAL
    lib.psgd_plan_destroy(None)
    with pytest.raises(B.PsgdError):
        plan.set_tuning("no_such_key", 1)
    with pytest.raises(B.PsgdError):
        plan.set_tuning("k1_nv", 99)
    with pytest.raises(B.PsgdError):
        plan.set_tuning("stream_hints", 2)
    plan.set_tuning("stream_hints", 1)
    with pytest.raises(B.PsgdError):
        plan.set_tuning("gram_fused", 3)
    with pytest.raises(B.PsgdError):
        plan.set_tuning("gram_spin", 0)
    for key, bad in (("resident", 3), ("res_spin", 0), ("res_max_blocks", -1), ("q_reduce_elems", 1), ("k1_mfma", 1),
                     ("ortho_rows", -1), ("ortho_rows", 1025)):
        with pytest.raises(B.PsgdError):     # out of range, or a key that no longer exists
            plan.set_tuning(key, bad)
    plan.set_tuning("res_spin", 1 << 10)
    plan.set_tuning("gram_fused", 0)
    plan.set_tuning("gram_spin", 1024)
    plan.set_tuning("ortho_rows", 1024)
    plan.set_tuning("ortho_rows", 0)
    with pytest.raises(B.PsgdError):
        plan.set_tuning("xcd_order", -2)
    plan.set_tuning("xcd_order", -1)
    plan.set_tuning("xcd_order", 0)
    plan.set_tuning("k1_rows", 16)


def test_layout_resnet18():
    shapes = WL.resnet18_shapes()
    plan = B.Plan(shapes, 2, 1)
    s = plan.sizes
    assert s.n_matrices == 21 and s.n_vec_elems == 9610
    assert s.payload_elems == 11164352 + 9610
    assert s.n_mat_elems == 11164352          # every ResNet18 matrix is a multiple of 64 elements
    # P and Q of each matrix start at multiples of 4 floats
    up4 = lambda x: (x + 3) // 4 * 4
    mats = [sh for sh in shapes if len(sh) > 1]
    assert s.p_elems == sum(up4(2 * sh[0]) for sh in mats) == 2 * 4810
    assert s.q_elems == sum(up4(2 * int(np.prod(sh[1:]))) for sh in mats) == 2 * 31515 + 2
    # traffic model per matrix element: 12 + 4/W compulsory, 24 + 4/W streaming
    assert s.bytes_min == 11164352 * 16 + 9610 * 8
    assert s.bytes_stream == 11164352 * 28 + 9610 * 8
    # offsets: matrices in order, aligned, then vectors in order
    prev_end = 0
    voff = s.n_mat_elems
    for t, sh in enumerate(shapes):
        f, p, q, r = plan.offsets(t)
        if len(sh) == 1:
            assert (f, p, q, r) == (voff, -1, -1, 0)
            voff += sh[0]
        else:
            assert f % 64 == 0 and f >= prev_end and r == 2
            prev_end = f + sh[0] * sh[1]
    assert voff == s.out_elems


def test_effective_rank_and_padding():
    shapes = [(5, 3), (7,), (37, 91), (2, 100)]
    plan = B.Plan(shapes, 4, 3)
    assert [plan.offsets(t)[3] for t in range(4)] == [3, 0, 4, 2]
    assert plan.offsets(0)[0] == 0 and plan.offsets(2)[0] == 64 and plan.offsets(3)[0] == 64 + 3392
    s = plan.sizes
    assert s.n_mat_elems == 64 + 3392 + 256 and s.n_vec_elems == 7
    assert s.grad_stride % 64 == 0 and s.grad_stride >= s.n_mat_elems + 7
    # each factor padded to a multiple of 4 floats
    assert s.p_elems == 16 + 37 * 4 + 2 * 2 and s.q_elems == 12 + 91 * 4 + 100 * 2
    assert [plan.offsets(t)[1] for t in (0, 2, 3)] == [0, 16, 16 + 148]
    assert [plan.offsets(t)[2] for t in (0, 2, 3)] == [0, 12, 12 + 364]
    assert s.workspace_bytes > 0


def test_compression_ratios_match_the_paper():
    """Appendix F / Table 3: 243x, 136x, 72x for ResNet18; 310x, 203x, 120x for the LSTM."""
    from oracle import powersgd_oracle as O
    for shapes, want in ((WL.resnet18_shapes(), {1: 243, 2: 136, 4: 72}),
                         (WL.lstm_shapes(vocab=28869), {1: 310, 2: 203, 4: 120})):
        for r, ratio in want.items():
            s = B.Plan(shapes, r, 1).sizes
            got = s.payload_elems / s.compressed_elems
            assert abs(got - ratio) <= 0.5
            assert s.compressed_elems == O.compressed_floats(shapes, r)


def test_which_kernels_a_plan_runs():
    """psgd_plan_path: the planner's choice among the streaming, resident and matrix-core kernels, from rank, data
    types, shapes and set size (no GPU is needed to ask)."""
    lib = B.load_library()
    small = [(64, 576), (128, 64), (33,)]
    big = [(20000, 4096), (4096, 4096), (4096,)]          # 99 M elements: beyond the memory-side cache
    big_odd = [(20000, 4098), (4096, 4096)]               # a row length that is not a multiple of 4
    assert B.Plan(small, 2, 1).path() == "resident"
    assert B.Plan(small, 2, 2).path() == "streaming"
    assert B.Plan(small, 16, 1).path() == "matrix cores"
    assert B.Plan(big, 4, 1).path() == "streaming"         # fp32 data at rank <= 8
    bf = (B.PSGD_BF16, B.PSGD_BF16)
    assert B.Plan(big, 4, 1, *bf).path() == "matrix cores"  # bf16 data, rank >= 4, a large set
    assert B.Plan(big, 2, 1, *bf).path() == "streaming"
    assert B.Plan(small, 4, 1, *bf).path() == "streaming"
    assert B.Plan(big_odd, 4, 1, *bf).path() == "streaming"
    p = B.Plan(big, 4, 1, *bf)
    p.set_tuning("bf16_valu", 1)
    assert p.path() == "streaming"
    p.set_tuning("bf16_valu", 0)
    assert p.path() == "matrix cores"
    with pytest.raises(B.PsgdError):
        p.set_tuning("bf16_valu", 2)
    q = B.Plan(small, 4, 1, *bf)
    q.set_tuning("bf16_valu", 0)
    assert q.path() == "matrix cores"
    import ctypes as C
    r = C.c_int32()
    assert lib.psgd_plan_path(None, C.byref(r)) == B.PSGD_EINVAL and lib.psgd_plan_path(p._h, None) == B.PSGD_EINVAL
