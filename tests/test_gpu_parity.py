"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element on the same seeded inputs.

Bar (stated by the benchmark spec): relative Frobenius error <= 1e-5 on P_hat, Q and the
new error memory, per matrix, per worker, at every step.

Protocol.  Both sides carry their own state (error memories and warm-start Q)
from step to step: the GPU in its fp32 buffers, updated in place by the
library, the oracle in fp64.  On the noise-dominated synthetic gradients the
step map has almost no spectral gap between the kept and the dropped
directions (sigma_r / sigma_{r+1} of g + e is 1.02 .. 1.3), so any fp32
rounding - already that of storing the state in fp32, kernels aside - grows by
roughly 1.3x per step: a pure numpy fp32 re-run of the oracle's own steps leaves
the fp64 trajectory at the same rate.  Holding 1e-5 over 100 free-running steps
is therefore not a property an fp32 state can have.  The long runs are
free-running in windows of RESYNC steps: at a window boundary the oracle's state
is rounded to fp32 (the paper's storage precision) and the GPU is restarted from
those bits.  RESYNC = 6 comes from measurement on the full ResNet18-shaped set:
the fp64 oracle whose state alone is kept in fp32 is 2.4e-7 away from the exact one
after 6 steps, 6.5e-7 after 8 and 1e-6 after 11 (rank 2); the GPU path, which also
computes in fp32, starts a window at 1.3e-7 and, in the first window of a run (the
fastest growing one), is at 1-2e-6 after 6 steps at every rank, at 6e-6 to 1.3e-5
after 8 depending on rank and seed, and at 5e-5 after 20: six is the longest window
that keeps a factor of five under the bar.  Short runs (the 10-step Tiny configuration) are free-running
throughout.  A separate 100-step run never re-synchronised checks what stays
well defined on a diverging trajectory: orthonormality, conservation of
g + e = Delta' + e', and that the compression quality ||e'|| / ||M|| follows
the oracle's.
"""
import numpy as np
import torch
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu

TOL = 1e-5
RESYNC = 6


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _run(wl, rank, workers, steps, seed=0, tuning=None, split=False, verbose=True, resync=None,
         expect_resident=None, grad_bf16=False, out_bf16=False):
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun, OracleRun, compare
    factors = WL.planted_factors(wl, seed)
    q0 = WL.initial_q(wl, rank, seed)
    gpu = GpuRun(wl.shapes, rank, workers, q0, tuning, grad_bf16=grad_bf16, out_bf16=out_bf16)
    ora = OracleRun(wl.shapes, rank, workers, q0)
    worst_all = {"P_hat": 0.0, "Q": 0.0, "err": 0.0, "out": 0.0}
    for t in range(steps):
        if resync and t > 0 and t % resync == 0:
            ora.round_state_to_fp32()
            gpu.set_err(ora.errs)
            gpu.set_q(ora.Qs)
        grads = [WL.gradients(wl, factors, seed, t, w) for w in range(workers)]
        if grad_bf16:   # the gradient both sides see is the bf16 rounding of the fp32 sample, upcast exactly
            grads = [[WL.bf16_round(g) for g in gw] for gw in grads]
        rg = gpu.step(grads, split=split)
        prev_errs = ora.errs
        ro = ora.step(grads)
        worst = compare(rg, ro, wl.shapes, workers, rank, grads, prev_errs, out_bf16=out_bf16)
        for k in worst:
            worst_all[k] = max(worst_all[k], worst[k])
        assert worst["P_hat"] <= TOL and worst["Q"] <= TOL and worst["err"] <= TOL and worst["out"] <= TOL, \
            (wl.name, rank, workers, t, worst)
        if verbose and steps > 10 and (t + 1) % 10 == 0:   # long runs report as they go
            print("[parity] %s r=%d W=%d step %d of %d ok" % (wl.name, rank, workers, t + 1, steps), flush=True)
    if verbose:
        print("\n[parity] %s r=%d W=%d steps=%d resync=%s resident=%s worst %s"
              % (wl.name, rank, workers, steps, resync, gpu.resident, worst_all), flush=True)
    if expect_resident is not None:
        assert gpu.resident == expect_resident
    return worst_all


def _workload(shapes, planted_rank=4, sigma=0.01, name="custom"):
    from paper_1905_13727_amd import workloads as WL
    return WL.Workload(name, list(shapes), planted_rank, 1.0 / np.arange(1, planted_rank + 1), sigma)


def test_tiny_config_10_steps():
    """The Tiny configuration, free-running for all 10 steps, on the resident kernel (the mode
    psgd_step picks for it) and on the streaming kernels."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run(WL.tiny(), rank=2, workers=1, steps=10, seed=0, expect_resident=True)
    _run(WL.tiny(), rank=2, workers=1, steps=10, seed=0, tuning={"resident": 0}, expect_resident=False)


RAGGED_1W = [(37, 91), (7,), (50, 650), (130, 1028), (5, 3), (300, 2), (1, 40), (1031,), (3, 4700), (257, 260),
             (512, 36), (64, 27)]


@pytest.mark.parametrize("rank", [1, 2, 3, 4])
def test_resident_ragged_shapes(rank):
    """Resident kernel on shapes with scalar, 2-wide and 4-wide row access in one model, strips with
    a ragged last strip, column chunks with a ragged tail, clipped ranks, vectors; default strip
    height, the thinnest and the tallest strips."""
    _need_gpu()
    wl = _workload(RAGGED_1W)
    _run(wl, rank=rank, workers=1, steps=4, seed=10 + rank, expect_resident=True)
    _run(wl, rank=rank, workers=1, steps=3, seed=20 + rank, tuning={"res_rows": 32 if rank <= 2 else 24},
         expect_resident=True)
    _run(wl, rank=rank, workers=1, steps=3, seed=30 + rank, tuning={"res_rows": 5}, expect_resident=True)


def test_resident_falls_back_when_the_model_does_not_fit():
    _need_gpu()
    # a 600-row matrix is taller than the resident Gram-Schmidt handles; W = 2 is not resident either
    _run(_workload([(600, 64), (64, 64)]), rank=2, workers=1, steps=2, seed=3, expect_resident=False)
    _run(_workload([(64, 64)]), rank=2, workers=2, steps=2, seed=4, expect_resident=False)
    _run(_workload([(64, 64)]), rank=5, workers=1, steps=2, seed=5, expect_resident=False)


@pytest.mark.parametrize("rank", [1, 2, 3, 4, 8])
def test_ragged_shapes_three_workers(rank):
    """Row lengths that are not multiples of 4 or 2 (scalar / 2-wide row access), rows that
    do not divide the tile heights, several column chunks with a ragged tail, ranks clipped
    by a tiny matrix, vectors between matrices."""
    _need_gpu()
    shapes = [(37, 91), (7,), (50, 650), (130, 1028), (5, 3), (300, 2), (1, 40), (1031,), (3, 4700), (257, 260)]
    _run(_workload(shapes), rank=rank, workers=3, steps=4, seed=rank)
    # the same with the short panels orthogonalised by one workgroup (Gram-Schmidt in LDS)
    _run(_workload(shapes), rank=rank, workers=3, steps=3, seed=40 + rank, tuning={"ortho_rows": 1024})


@pytest.mark.parametrize("rank,workers", [(1, 1), (3, 2), (4, 1), (8, 2)])
def test_tall_panels(rank, workers):
    """Panels too tall for one workgroup's LDS take the multi-workgroup Cholesky-QR route (same
    orthonormal factor as Gram-Schmidt): ragged last row block, several Gram blocks, W = 1 and 2,
    and an all-zero gradient on the same plan shape."""
    _need_gpu()
    from gpu_harness import GpuRun
    shapes = [(7000, 36), (33,), (13001, 6), (2600, 650), (64, 64)]
    wl = _workload(shapes)
    _run(wl, rank=rank, workers=workers, steps=3, seed=40 + rank, expect_resident=False)
    from paper_1905_13727_amd import workloads as WL
    g = GpuRun(shapes, rank, workers, WL.initial_q(wl, rank, 1))
    r = g.step([[np.zeros(s, dtype=np.float32) for s in shapes] for _ in range(workers)])
    for t, s in enumerate(shapes):
        if len(s) == 2:
            assert np.abs(r["P_hat"][t]).max() == 0 and np.abs(r["Q"][t]).max() == 0
            assert np.abs(r["err"][0][t]).max() == 0 and np.abs(r["out"][t]).max() == 0


@pytest.mark.parametrize("rank,workers", [(2, 1), (4, 2), (7, 1)])
def test_tall_panels_in_one_launch_and_in_two(rank, workers):
    """The tall-panel factorisation runs as one launch whose row blocks exchange their Gram matrices through
    tagged slots (the planner's choice when the device holds a matrix's row blocks at once), or as two launches
    (gram_fused = 0).  Both add the same numbers in the same order: parity holds for the two-launch form as well,
    and the two agree bit for bit over several steps on one plan (the slots are reused, told apart by their
    epoch), including a panel of 130 row blocks."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun
    shapes = [(7000, 36), (33,), (33278, 65), (2600, 650), (64, 64), (257, 9)]
    wl = _workload(shapes)
    two = {"resident": 0, "gram_fused": 0}
    _run(wl, rank=rank, workers=workers, steps=2, seed=90 + rank, tuning=two, expect_resident=False)
    factors = WL.planted_factors(wl, 6)
    q0 = WL.initial_q(wl, rank, 6)
    a = GpuRun(wl.shapes, rank, workers, q0, {"resident": 0, "gram_fused": 1})
    b = GpuRun(wl.shapes, rank, workers, q0, two)
    for t in range(4):
        grads = [WL.gradients(wl, factors, 6, t, w) for w in range(workers)]
        ra, rb = a.step(grads), b.step(grads)
        for key in ("P_hat", "Q", "out"):
            for x, y in zip(ra[key], rb[key]):
                assert x is None or np.array_equal(x, y)
        for w in range(workers):
            for x, y in zip(ra["err"][w], rb["err"][w]):
                assert x is None or np.array_equal(x, y)


def test_one_launch_factorisation_reports_a_wait_that_gives_up():
    """A panel of 4297 row blocks is more than the device holds at once, so its workgroups cannot all wait for each
    other: the planner takes the two launches for it (parity below).  Forced into one launch (gram_fused = 2) with
    a small poll limit, the waits give up, every workgroup still runs to its end, psgd_plan_check reports the
    failure and clears the slots, and the next call on the plan behaves the same way instead of hanging."""
    _need_gpu()
    from paper_1905_13727_amd import binding as B
    shapes = [(1100000, 8), (300, 40)]
    _run(_workload(shapes), rank=2, workers=1, steps=1, seed=95, expect_resident=False)
    dev = torch.device("cuda:0")
    plan = B.Plan(shapes, 2, 1)
    for key, value in (("resident", 0), ("gram_fused", 2), ("gram_spin", 256)):
        plan.set_tuning(key, value)
    sz = plan.sizes
    gen = torch.Generator(device="cpu")
    gen.manual_seed(3)
    grad = (torch.randn(sz.grad_stride, generator=gen) * 0.01).to(dev)
    err = torch.zeros(sz.err_stride, device=dev)
    q = torch.randn(sz.q_elems, generator=gen).to(dev)
    p = torch.zeros(sz.p_elems, device=dev)
    out = torch.zeros(sz.out_elems, device=dev)
    ws = torch.zeros(sz.workspace_bytes // 4 + 64, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    for attempt in range(2):
        print("[timeout] forced one-launch step %d" % attempt, flush=True)
        plan.step(grad, err, q, p, out, ws, stream)
        with pytest.raises(B.PsgdError):
            plan.check(stream)
        assert "timed out" in plan.last_error()
    plan.destroy()


def test_resident_wait_that_gives_up_is_reported_and_the_plan_streams_on():
    """The resident kernel's workgroups wait for each other, so all of them must be on the chip at once; the planner
    sizes the grid for that.  Here the check is switched off (resident = 2) and the ResNet18-shaped set is cut into
    8-row strips: four times more workgroups than the device holds.  With a poll limit of two rounds (far less than
    the time until a workgroup that is not yet on the chip has delivered) waits give up,
    every workgroup still runs to its end, psgd_plan_check reports the failure and moves the plan to the streaming
    kernels, and the next step on the same plan (state restored) is at parity."""
    _need_gpu()
    from paper_1905_13727_amd import binding as B, workloads as WL
    from gpu_harness import GpuRun, OracleRun, compare
    wl = WL.resnet18()
    rank, seed = 2, 7
    factors = WL.planted_factors(wl, seed)
    q0 = WL.initial_q(wl, rank, seed)
    gpu = GpuRun(wl.shapes, rank, 1, q0, {"resident": 2, "res_max_blocks": 4096, "res_rows": 8, "res_spin": 2})
    ora = OracleRun(wl.shapes, rank, 1, q0)
    grads = [WL.gradients(wl, factors, seed, 0, 0)]
    print("[resident give-up] oversubscribed launch", flush=True)
    with pytest.raises(B.PsgdError):
        gpu.step(grads)
    assert "timed out" in gpu.plan.last_error()
    stream = torch.cuda.current_stream().cuda_stream
    assert gpu.plan.check(stream) is False          # no longer resident, nothing further to report
    zero = [[np.zeros(s, dtype=np.float32) for s in wl.shapes]]
    for t in range(2):
        if t == 0:      # the abandoned step left err and q half-updated
            gpu.set_err(zero)
            gpu.set_q(q0)
        grads = [WL.gradients(wl, factors, seed, t, 0)]
        rg = gpu.step(grads)
        assert gpu.resident is False
        prev = ora.errs
        ro = ora.step(grads)
        worst = compare(rg, ro, wl.shapes, 1, rank, grads, prev)
        assert max(worst.values()) <= TOL, (t, worst)


@pytest.mark.parametrize("rank,workers,bf16", [(3, 2, False), (4, 1, True)])
def test_tall_and_wide_matrices(rank, workers, bf16):
    """Matrices of at least 2048 x 2048 get 1024-row blocks in the second sweep and 16-row tiles in the first and
    third (the planner's choice for them): one exactly at the limit, one ragged in both directions, next to a
    small one; fp32 with two workers, and bf16 data."""
    _need_gpu()
    shapes = [(2048, 2048), (2100, 2052), (64, 576), (300,)]
    _run(_workload(shapes), rank=rank, workers=workers, steps=2, seed=50 + rank, expect_resident=False,
         grad_bf16=bf16, out_bf16=bf16)


def _steps(env_name, default):
    """Step count of the long parity runs.  The defaults keep the suite to a few minutes (the fp64 oracle is the
    slow side: 16 workers cost 2.5 s per step); PSGD_PARITY_STEPS_W16 / PSGD_PARITY_STEPS_LSTM change them."""
    import os
    return int(os.environ.get(env_name, default))


def test_lstm_r4_100_steps():
    """LSTM-shaped set (tied embedding with 5 % of the rows non-zero per step), rank 4."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run(WL.lstm(), rank=4, workers=1, steps=_steps("PSGD_PARITY_STEPS_LSTM", 100), seed=0, resync=RESYNC,
         expect_resident=False)


@pytest.mark.parametrize("rank", [1, 2, 4])
def test_resnet18_16_workers(rank):
    """ResNet18-shaped set with 16 simulated workers, ranks 1, 2, 4: 20 steps each by default (the oracle needs 16
    times the single-worker time, 2.5 s a step), so that window boundaries are crossed and the error memories
    carry more than a window's history; PSGD_PARITY_STEPS_W16 changes the count (100 is the stated run)."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run(WL.resnet18(), rank=rank, workers=16, steps=_steps("PSGD_PARITY_STEPS_W16", 20), seed=rank, resync=RESYNC,
         expect_resident=False)


@pytest.mark.parametrize("rank", [1, 3, 4])
def test_resnet18_resident_other_ranks(rank):
    """The full-size ResNet18-shaped set on the resident kernel at the other ranks of the sweep: ranks 3 and 4 cut the
    21 matrices into strips of 24 rows instead of 32, a different tiling from rank 2's."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run(WL.resnet18(), rank=rank, workers=1, steps=10, seed=rank, resync=RESYNC, expect_resident=True)


@pytest.mark.parametrize("rank", [1, 2])
def test_lstm_low_ranks(rank):
    """LSTM-shaped set at ranks 1 and 2 (the target names ranks 1-4), full size."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run(WL.lstm(), rank=rank, workers=1, steps=10, seed=rank, resync=RESYNC, expect_resident=False)


TRANSFORMER_SMALL = [(1000, 256), (256,), (256, 256), (256, 256), (1024, 256), (1024,), (256, 1024), (20, 12), (3000, 64),
                     (130, 2308)]


@pytest.mark.parametrize("rank,workers,gbf,obf", [(16, 1, False, False), (32, 2, False, False), (9, 1, False, False),
                                                  (64, 1, False, False), (16, 1, True, True), (32, 1, True, False),
                                                  (4, 2, True, True), (2, 1, False, True)])
def test_matrix_core_path(rank, workers, gbf, obf):
    """Ranks above 8 run on the matrix-core kernels, with fp32 or bf16 gradients / output; so do bf16 data at
    rank <= 8 when asked to (`bf16_valu` = 0): a small transformer-shaped set (ragged row blocks and column
    chunks, a matrix smaller than the rank, vectors), planted rank 64 with a 1/k spectrum."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    wl = WL.Workload("tr-small", list(TRANSFORMER_SMALL), 64, 1.0 / np.arange(1, 65), 0.001)
    _run(wl, rank=rank, workers=workers, steps=3, seed=60 + rank, expect_resident=False, grad_bf16=gbf, out_bf16=obf,
         tuning={"bf16_valu": 0})


@pytest.mark.parametrize("rank,workers,gbf,obf", [(4, 2, True, True), (2, 1, False, True), (8, 1, True, False),
                                                  (3, 3, True, True)])
def test_streaming_path_bf16(rank, workers, gbf, obf):
    """bf16 gradients and / or output at rank <= 8 on the streaming kernels (the default for them): the gradient is
    widened as it is read, Delta' is rounded to nearest even as it is stored, the state stays fp32.  Also with the
    large-set cache policy forced."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    wl = WL.Workload("tr-small", list(TRANSFORMER_SMALL), 64, 1.0 / np.arange(1, 65), 0.001)
    _run(wl, rank=rank, workers=workers, steps=3, seed=80 + rank, expect_resident=False, grad_bf16=gbf, out_bf16=obf)
    _run(wl, rank=rank, workers=workers, steps=2, seed=90 + rank, expect_resident=False, grad_bf16=gbf, out_bf16=obf,
         tuning={"stream_hints": 1})


@pytest.mark.parametrize("rank,workers,gbf,obf", [(4, 2, True, True), (1, 1, True, False), (8, 1, False, True),
                                                  (3, 3, True, True)])
def test_streaming_path_bf16_any_row_length(rank, workers, gbf, obf):
    """bf16 gradients / output on matrices whose row length is odd or even but not a multiple of 4 (the LSTM's rows
    of 650 among them): 2- and 4-byte accesses to the bf16 buffers instead of 8-byte ones."""
    _need_gpu()
    shapes = [(37, 91), (7,), (50, 650), (130, 1028), (5, 3), (300, 2), (1, 40), (1031,), (3, 4700), (257, 262),
              (2600, 650)]
    _run(_workload(shapes), rank=rank, workers=workers, steps=3, seed=110 + rank, expect_resident=False, grad_bf16=gbf,
         out_bf16=obf)
    if rank == 4:
        _run_update(_workload(shapes), rank=rank, workers=workers, steps=2, seed=115, grad_bf16=True,
                    expect_resident=False)


@pytest.mark.parametrize("rows,cols", [(64, 64), (256, 192), (128, 4096)])
def test_matrix_core_tilings(rows, cols):
    """P = M Q on the matrix cores with rows split into many column ranges (partials summed in
    index order; ranges of 192 columns end inside a 128-column chunk), one range only, and the tallest workgroup
    tile; at one and two rank tiles; the decompression with workgroups of 48 rows (wavefront strips of 12: every
    16-row step is ragged)."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    wl = WL.Workload("tr-small", list(TRANSFORMER_SMALL), 64, 1.0 / np.arange(1, 65), 0.001)
    tuning = {"hr_k1_rows": rows, "hr_k1_cols": cols}
    _run(wl, rank=16, workers=2, steps=2, seed=77, expect_resident=False, tuning=tuning)
    _run(wl, rank=32, workers=1, steps=2, seed=79, expect_resident=False, tuning=dict(tuning, hr_k4_rows=48),
         grad_bf16=True, out_bf16=True)
    _run(wl, rank=4, workers=1, steps=2, seed=78, expect_resident=False, tuning=tuning, grad_bf16=True)


def test_small_tiles_many_partials():
    """Forces many column chunks and row blocks per matrix so that the fixed-order partial
    sums are exercised."""
    _need_gpu()
    shapes = [(200, 1500), (64, 576), (33,)]
    tuning = {"k1_rows": 8, "k1_nv": 1, "k3_rows": 16, "k4_rows": 8, "ortho_rows": 64}
    _run(_workload(shapes), rank=3, workers=2, steps=3, seed=5, tuning=tuning)
    tuning = {"k1_rows": 64, "k1_nv": 2, "k3_rows": 300, "k3_nv": 2, "k4_rows": 300, "k4_nv": 2}
    _run(_workload(shapes), rank=4, workers=2, steps=3, seed=6, tuning=tuning)


def test_split_calls_equal_step_bitwise():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun
    wl = WL.tiny()
    factors = WL.planted_factors(wl, 0)
    q0 = WL.initial_q(wl, 2, 0)
    a = GpuRun(wl.shapes, 2, 2, q0)
    b = GpuRun(wl.shapes, 2, 2, q0)
    for t in range(3):
        grads = [WL.gradients(wl, factors, 0, t, w) for w in range(2)]
        ra = a.step(grads, split=False)
        rb = b.step(grads, split=True)
        for key in ("P_hat", "Q", "out"):
            for x, y in zip(ra[key], rb[key]):
                assert x is None or np.array_equal(x, y)
        for w in range(2):
            for x, y in zip(ra["err"][w], rb["err"][w]):
                assert x is None or np.array_equal(x, y)


@pytest.mark.parametrize("rank,workers", [(2, 3), (4, 1)])
def test_streaming_hints(rank, workers):
    """Sets larger than the memory-side cache read M and write the new error memory with non-temporal accesses in
    the second and third sweep.  The planner picks this by size (the 16-worker ResNet18 set runs that way); here
    it is forced on a small ragged set: parity holds, and since the arithmetic is the same the results are
    bit-identical to those of the ordinary accesses."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun
    wl = _workload(RAGGED_1W + [(2600, 650)])
    hints = {"resident": 0, "stream_hints": 1}
    _run(wl, rank=rank, workers=workers, steps=3, seed=70 + rank, tuning=hints, expect_resident=False)
    factors = WL.planted_factors(wl, 5)
    q0 = WL.initial_q(wl, rank, 5)
    a = GpuRun(wl.shapes, rank, workers, q0, hints)
    b = GpuRun(wl.shapes, rank, workers, q0, {"resident": 0, "stream_hints": 0})
    for t in range(3):
        grads = [WL.gradients(wl, factors, 5, t, w) for w in range(workers)]
        ra, rb = a.step(grads), b.step(grads)
        for key in ("P_hat", "Q", "out"):
            for x, y in zip(ra[key], rb[key]):
                assert x is None or np.array_equal(x, y)
        for w in range(workers):
            for x, y in zip(ra["err"][w], rb["err"][w]):
                assert x is None or np.array_equal(x, y)
    # matrix-core path: the second sweep reads M that way
    _run(_workload(TRANSFORMER_SMALL), rank=16, workers=1, steps=2, seed=75, tuning={"stream_hints": 1})


@pytest.mark.parametrize("mode", ["resident", "streaming", "streaming_w3_bf16", "matrix_cores"])
def test_step_replayed_from_a_hip_graph(mode):
    """psgd_step makes no allocation, no memset and no host synchronisation once the plan's tables are on the device,
    so it can be captured into a HIP graph.  The graph is replayed several times (new gradients copied into the
    captured buffer, other GPU work and synchronisations in between); every replay must leave exactly the bits the
    same steps leave when launched directly."""
    _need_gpu()
    from paper_1905_13727_amd import binding as B
    dev = torch.device("cuda:0")
    shapes = [(37, 91), (7,), (64, 576), (130, 1028), (5, 3), (300, 4), (512, 36)]
    rank, workers, gdt, tune = 2, 1, torch.float32, {}
    if mode == "streaming":
        tune = {"resident": 0}
    elif mode == "streaming_w3_bf16":
        shapes = [(40, 92), (7,), (64, 576), (130, 1028), (300, 4), (2600, 64)]
        rank, workers, gdt = 4, 3, torch.bfloat16
    elif mode == "matrix_cores":
        shapes = [(40, 92), (7,), (64, 576), (130, 1028), (300, 4)]
        rank = 16
    dt = B.PSGD_BF16 if gdt == torch.bfloat16 else B.PSGD_F32
    plan = B.Plan(shapes, rank, workers, dt, dt)
    for k, v in tune.items():
        plan.set_tuning(k, v)
    s = plan.sizes
    gen = torch.Generator(device="cpu")
    gen.manual_seed(11)
    grads = [(torch.randn(workers * s.grad_stride, generator=gen) * 0.01).to(gdt).to(dev) for _ in range(4)]
    q0 = torch.randn(s.q_elems, generator=gen).to(dev)

    def fresh_state():
        return dict(err=torch.zeros(workers * s.err_stride, device=dev), q=q0.clone(),
                    p=torch.zeros(s.p_elems, device=dev), out=torch.zeros(s.out_elems, device=dev, dtype=gdt),
                    ws=torch.zeros(s.workspace_bytes // 4 + 64, device=dev))

    def snapshot(st):
        torch.cuda.synchronize()
        return [st[k].clone() for k in ("err", "q", "p", "out")]

    g_in = torch.zeros_like(grads[0])
    # launched directly (the first call also uploads the plan's tables, which a capture could not)
    st = fresh_state()
    want = []
    for t in range(4):
        g_in.copy_(grads[t])
        plan.step(g_in, st["err"], st["q"], st["p"], st["out"], st["ws"], torch.cuda.current_stream().cuda_stream)
        want.append(snapshot(st))
    assert plan.check(torch.cuda.current_stream().cuda_stream) == (mode == "resident")
    # captured once, replayed four times
    st = fresh_state()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.step(g_in, st["err"], st["q"], st["p"], st["out"], st["ws"], torch.cuda.current_stream().cuda_stream)
    for k in ("err", "p", "out", "ws"):
        st[k].zero_()
    st["q"].copy_(q0)
    for t in range(4):
        g_in.copy_(grads[t])
        graph.replay()
        noise = (torch.randn(1 << 20, device=dev) * 2).sum()   # unrelated work between the replays
        got = snapshot(st)
        assert torch.isfinite(noise)
        for name, a, b in zip(("err", "q", "p", "out"), got, want[t]):
            assert torch.equal(a, b), (mode, t, name)
    plan.check(torch.cuda.current_stream().cuda_stream)
    plan.destroy()


def test_between_compress_and_decompress_err_holds_m():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun
    wl = WL.tiny()
    factors = WL.planted_factors(wl, 0)
    q0 = WL.initial_q(wl, 2, 0)
    g = GpuRun(wl.shapes, 2, 1, q0)
    grads = [WL.gradients(wl, factors, 0, 0, 0)]
    e0 = [np.full(s, 0.25, dtype=np.float32) for s in wl.shapes]
    g.set_err([e0])
    g.upload(grads)
    stream = torch.cuda.current_stream().cuda_stream
    g.plan.compress(g.grad, g.err, g.q, g.p, g.ws, stream)
    torch.cuda.synchronize()
    m = g.download()["err"][0]
    for t in range(len(wl.shapes)):
        assert np.array_equal(m[t], grads[0][t] + e0[t])


def test_zero_gradient_and_reproducibility():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun
    wl = WL.tiny()
    q0 = WL.initial_q(wl, 2, 0)
    for tuning in ({}, {"resident": 0}):
        g = GpuRun(wl.shapes, 2, 1, q0, tuning)
        zero = [[np.zeros(s, dtype=np.float32) for s in wl.shapes]]
        r = g.step(zero)
        for t in range(len(wl.shapes)):
            assert not np.isnan(r["P_hat"][t]).any()
            assert np.abs(r["P_hat"][t]).max() == 0 and np.abs(r["Q"][t]).max() == 0
            assert np.abs(r["out"][t]).max() == 0 and np.abs(r["err"][0][t]).max() == 0
    # same inputs twice on fresh state: bit-identical (streaming W = 2, resident W = 1)
    factors = WL.planted_factors(wl, 3)
    for workers in (2, 1):
        runs = []
        for _ in range(2):
            h = GpuRun(wl.shapes, 2, workers, q0)
            for t in range(3):
                res = h.step([WL.gradients(wl, factors, 3, t, w) for w in range(workers)])
            assert h.resident == (workers == 1)
            runs.append(res)
        for key in ("P_hat", "Q", "out"):
            for x, y in zip(runs[0][key], runs[1][key]):
                assert np.array_equal(x, y)
        for x, y in zip(runs[0]["err"][0], runs[1]["err"][0]):
            assert np.array_equal(x, y)


def test_orthonormality_and_conservation_invariants():
    """Properties that hold at any size: P_hat^T P_hat = I and Delta' + e_new = g + e_old."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun
    wl = WL.resnet18()
    factors = WL.planted_factors(wl, 1)
    q0 = WL.initial_q(wl, 4, 1)
    g = GpuRun(wl.shapes, 4, 1, q0)
    prev_err = [np.zeros(s, dtype=np.float32) if len(s) == 2 else None for s in wl.shapes]
    for t in range(2):
        grads = [WL.gradients(wl, factors, 1, t, 0)]
        r = g.step(grads)
        for i, s in enumerate(wl.shapes):
            if len(s) == 1:
                assert np.array_equal(r["out"][i], grads[0][i])
                continue
            P = r["P_hat"][i].astype(np.float64)
            assert np.abs(P.T @ P - np.eye(P.shape[1])).max() < 1e-6
            lhs = r["out"][i].astype(np.float64) + r["err"][0][i]
            rhs = grads[0][i].astype(np.float64) + prev_err[i]
            assert np.abs(lhs - rhs).max() <= 4 * np.finfo(np.float32).eps * (np.abs(rhs).max() + np.abs(r["out"][i]).max())
            prev_err[i] = r["err"][0][i]


def test_resnet18_r2_100_steps():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run(WL.resnet18(), rank=2, workers=1, steps=100, seed=0, resync=RESYNC, expect_resident=True)


def test_resnet18_r2_streaming_kernels_20_steps():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run(WL.resnet18(), rank=2, workers=1, steps=20, seed=0, resync=RESYNC, tuning={"resident": 0},
         expect_resident=False)


def test_resnet18_r2_100_steps_never_resynchronised():
    """100 free-running steps: invariants of every step, and the compression quality
    ||e'||_F / ||g + e||_F over the whole model stays within 1 % of the free-running oracle's."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun, OracleRun
    wl = WL.resnet18()
    rank, seed = 2, 0
    factors = WL.planted_factors(wl, seed)
    q0 = WL.initial_q(wl, rank, seed)
    gpu = GpuRun(wl.shapes, rank, 1, q0)
    ora = OracleRun(wl.shapes, rank, 1, q0)
    mats = [i for i, s in enumerate(wl.shapes) if len(s) == 2]
    prev = {i: np.zeros(wl.shapes[i], dtype=np.float32) for i in mats}
    for t in range(100):
        grads = [WL.gradients(wl, factors, seed, t, 0)]
        rg = gpu.step(grads)
        prev_o = ora.errs
        ro = ora.step(grads)
        num_g = den_g = num_o = den_o = 0.0
        for i in mats:
            P = rg["P_hat"][i].astype(np.float64)
            assert np.abs(P.T @ P - np.eye(rank)).max() < 1e-6, (t, i)
            m_gpu = grads[0][i].astype(np.float64) + prev[i]
            lhs = rg["out"][i].astype(np.float64) + rg["err"][0][i]
            assert np.abs(lhs - m_gpu).max() <= 4 * np.finfo(np.float32).eps * (np.abs(m_gpu).max() + np.abs(rg["out"][i]).max())
            m_ora = grads[0][i].astype(np.float64) + prev_o[0][i]
            num_g += np.linalg.norm(rg["err"][0][i]) ** 2
            den_g += np.linalg.norm(m_gpu) ** 2
            num_o += np.linalg.norm(ro["err"][0][i]) ** 2
            den_o += np.linalg.norm(m_ora) ** 2
            prev[i] = rg["err"][0][i]
        q_gpu, q_ora = np.sqrt(num_g / den_g), np.sqrt(num_o / den_o)
        assert abs(q_gpu - q_ora) <= 0.01 * q_ora, (t, q_gpu, q_ora)


# ---- fused momentum / parameter update (Algorithm 2, last two lines) ------------------------------------

def _run_update(wl, rank, workers, steps, seed, lr=0.05, lam=0.9, tuning=None, grad_bf16=False, split=False,
                expect_resident=None):
    """psgd_step_update against the oracle's step followed by its momentum_update: the momentum buffer
    must match to the parity bar (it accumulates Delta'), the parameters to the bar relative to the size of
    the update they received plus one fp32 rounding of their own magnitude; P_hat, Q, E' as for psgd_step."""
    from oracle import powersgd_oracle as O
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun, OracleRun, compare, rel_fro
    factors = WL.planted_factors(wl, seed)
    q0 = WL.initial_q(wl, rank, seed)
    gpu = GpuRun(wl.shapes, rank, workers, q0, tuning, grad_bf16=grad_bf16)
    ora = OracleRun(wl.shapes, rank, workers, q0)
    lay, sizes = gpu.lay, gpu.plan.sizes
    rng = np.random.default_rng(seed + 1000)
    x0 = [rng.standard_normal(sh).astype(np.float32) for sh in wl.shapes]
    m0 = [(0.1 * rng.standard_normal(sh)).astype(np.float32) for sh in wl.shapes]
    dev = gpu.dev
    mom = torch.from_numpy(lay.pack_flat(m0)).to(dev)
    par = torch.from_numpy(lay.pack_flat(x0)).to(dev)
    assert mom.numel() == sizes.out_elems
    xo = [a.astype(np.float64) for a in x0]
    mo = [a.astype(np.float64) for a in m0]
    stream = torch.cuda.current_stream(dev).cuda_stream
    for t in range(steps):
        grads = [WL.gradients(wl, factors, seed, t, w) for w in range(workers)]
        if grad_bf16:
            grads = [[WL.bf16_round(g) for g in gw] for gw in grads]
        gpu.upload(grads)
        if split:
            gpu.plan.compress(gpu.grad, gpu.err, gpu.q, gpu.p, gpu.ws, stream)
            gpu.plan.decompress_update(gpu.p, gpu.q, gpu.err, gpu.grad, mom, par, lr, lam, gpu.ws, stream)
        else:
            gpu.plan.step_update(gpu.grad, gpu.err, gpu.q, gpu.p, mom, par, lr, lam, gpu.ws, stream)
        resident = gpu.plan.check(stream)
        torch.cuda.synchronize(dev)
        prev_errs = ora.errs
        ro = ora.step(grads)
        got = gpu.download()
        got["out"] = [np.asarray(ro["out"][i], dtype=np.float32).reshape(np.asarray(got["out"][i]).shape)
                      for i in range(len(wl.shapes))]    # Delta' is not stored by the fused call
        worst = compare(got, ro, wl.shapes, workers, rank, grads, prev_errs)
        assert worst["P_hat"] <= TOL and worst["Q"] <= TOL and worst["err"] <= TOL, (wl.name, t, worst)
        gm = lay.unpack_flat(mom.cpu().numpy())
        gx = lay.unpack_flat(par.cpu().numpy())
        for i, sh in enumerate(wl.shapes):
            delta = np.asarray(ro["out"][i], dtype=np.float64).reshape(sh)
            x_new, m_new = O.momentum_update(xo[i], mo[i], delta, lr, lam)
            assert rel_fro(gm[i].reshape(sh), m_new) <= TOL, (wl.name, t, i, "momentum")
            upd_norm = np.linalg.norm(lr * (delta + m_new))
            assert np.linalg.norm(gx[i].reshape(sh).astype(np.float64) - x_new) <= \
                TOL * upd_norm + 2.0 ** -23 * np.linalg.norm(x_new), (wl.name, t, i, "parameters")
            xo[i], mo[i] = x_new, m_new
    if expect_resident is not None:
        assert resident == expect_resident
    gpu.plan.destroy()


def test_fused_update_resident():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run_update(WL.tiny(), rank=2, workers=1, steps=4, seed=3, expect_resident=True)
    _run_update(_workload(RAGGED_1W), rank=3, workers=1, steps=3, seed=4, expect_resident=True)


def test_fused_update_streaming():
    _need_gpu()
    _run_update(_workload(RAGGED_1W[:10]), rank=4, workers=3, steps=3, seed=5, expect_resident=False)
    _run_update(_workload(RAGGED_1W[:10]), rank=2, workers=2, steps=2, seed=6, split=True, expect_resident=False)
    _run_update(_workload(RAGGED_1W), rank=1, workers=1, steps=2, seed=7, tuning={"resident": 0, "k4_nv": 2},
                expect_resident=False)


def test_fused_update_streaming_tiles_of_its_own():
    """A single-worker set of 16 M elements or more that fits the memory-side cache gets taller tiles for the fused
    pass than for the plain decompression (ragged last row blocks, a tall panel, vectors): parity of the fused
    step, and psgd_step on the same plan still at parity (it keeps the plain pass's tiles)."""
    _need_gpu()
    shapes = [(2600, 650), (33, ), (3333, 2700), (1031, 7), (9001, 650), (70, 4100), (129, )]
    assert sum(int(np.prod(s)) for s in shapes if len(s) == 2) >= (1 << 24)
    wl = _workload(shapes)
    _run_update(wl, rank=4, workers=1, steps=2, seed=11, expect_resident=False)
    _run_update(wl, rank=2, workers=1, steps=2, seed=12, split=True, expect_resident=False)
    _run(wl, rank=4, workers=1, steps=2, seed=13, expect_resident=False)


def test_fused_update_matrix_cores():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    wl = WL.Workload("tr-small", list(TRANSFORMER_SMALL), 64, 1.0 / np.arange(1, 65), 0.001)
    _run_update(wl, rank=16, workers=2, steps=2, seed=8, expect_resident=False)
    _run_update(wl, rank=4, workers=1, steps=2, seed=9, grad_bf16=True, expect_resident=False, tuning={"bf16_valu": 0})
    _run_update(wl, rank=4, workers=1, steps=2, seed=9, grad_bf16=True, expect_resident=False)   # streaming kernels


# ---- the 24-layer transformer-shaped set at full size, sampled tensors ---------------------------------

@pytest.mark.parametrize("rank,path", [(32, "matrix cores"), (16, "matrix cores"), (4, "matrix cores"), (4, "streaming")])
def test_transformer_full_size_sampled(rank, path):
    """The whole 145-matrix set (1.31 G elements, bf16 gradients and output, fp32 state) runs on the GPU in
    the launch configuration bench.py times.  The method treats every matrix on its own, so the oracle run
    on a sample of the tensors alone (the embedding, one matrix of each other shape from the first and the
    last layer, two vectors) gives exactly what the full-set step must produce for them.  The sampled
    tensors carry the planted-spectrum recipe from the host generator; the rest is noise drawn on the GPU.
    Five free-running steps at each of the three ranks of the configuration; rank 4 on the kernels the planner
    takes for it (matrix cores) and on the streaming kernels."""
    _need_gpu()
    from oracle import powersgd_oracle as O
    from paper_1905_13727_amd import binding as B, workloads as WL
    from paper_1905_13727_amd.flat import FlatLayout
    from gpu_harness import rel_fro
    wl = WL.transformer(24)
    shapes = wl.shapes
    mat_idx = [i for i, sh in enumerate(shapes) if len(sh) == 2]
    vec_idx = [i for i, sh in enumerate(shapes) if len(sh) == 1]
    first = {}
    for i in mat_idx:
        first.setdefault(shapes[i], i)
    last = {}
    for i in mat_idx:
        last[shapes[i]] = i
    sample = sorted(set(first.values()) | set(last.values()) | {vec_idx[0], vec_idx[-1]})
    assert (50304, 2048) in first and (2048, 8192) in first and len(sample) >= 8
    dev = torch.device("cuda:0")
    plan = B.Plan(shapes, rank, 1, B.PSGD_BF16, B.PSGD_BF16)
    if path == "streaming":
        plan.set_tuning("bf16_valu", 1)
    assert plan.path() == path
    lay = FlatLayout(plan, shapes)
    s = plan.sizes
    seed = 90 + rank
    factors = WL.planted_factors(wl, seed, only=sample)
    q0 = WL.initial_q(wl, rank, seed, only=sample)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    q = torch.randn(s.q_elems, generator=gen, device=dev)
    for i in sample:
        if q0[i] is not None:
            _, _, qo, r = plan.offsets(i)
            q[qo: qo + q0[i].size] = torch.from_numpy(q0[i].reshape(-1)).to(dev)
    err = torch.zeros(s.err_stride, device=dev)
    p = torch.zeros(s.p_elems, device=dev)
    out = torch.zeros(s.out_elems, dtype=torch.bfloat16, device=dev)
    ws = torch.empty(s.workspace_bytes // 4 + 64, device=dev)
    grad = torch.empty(s.grad_stride, dtype=torch.bfloat16, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    Qs = [None if q0[i] is None else q0[i].astype(np.float64) for i in sample]
    Es = [[None if len(shapes[i]) == 1 else np.zeros(shapes[i]) for i in sample]]
    sub_shapes = [shapes[i] for i in sample]
    for t in range(_steps("PSGD_PARITY_STEPS_TRANSFORMER", 5)):
        grad.normal_(0.0, wl.sigma, generator=gen)
        g_host = WL.gradients(wl, factors, seed, t, 0, only=sample)
        sub = []
        for i in sample:
            g = WL.bf16_round(g_host[i])
            sub.append(g)
            fo = plan.offsets(i)[0]
            grad[fo: fo + g.size] = torch.from_numpy(g.reshape(-1)).to(dev).to(torch.bfloat16)
        plan.step(grad, err, q, p, out, ws, stream)
        assert plan.check(stream) is False
        torch.cuda.synchronize(dev)
        ro = O.powersgd_step([sub], Es, Qs, rank)
        Qs, Es = ro["Q"], ro["err"]
        for k, i in enumerate(sample):
            fo, po, qo, r = plan.offsets(i)
            sh = shapes[i]
            n_el = int(np.prod(sh))
            got_out = out[fo: fo + n_el].float().cpu().numpy().reshape(sh).astype(np.float64)
            want_out = np.asarray(ro["out"][k]).reshape(sh)
            assert rel_fro(got_out, want_out) <= 2.0 ** -8, (rank, t, i, "out")
            if len(sh) == 1:
                continue
            n, m = sh
            got_p = p[po: po + n * r].cpu().numpy().reshape(n, r)
            got_q = q[qo: qo + m * r].cpu().numpy().reshape(m, r)
            got_e = err[fo: fo + n_el].cpu().numpy().reshape(sh)
            worst = (rel_fro(got_p, ro["P_hat"][k]), rel_fro(got_q, ro["Q"][k]), rel_fro(got_e, ro["err"][0][k]))
            print("[transformer full size] r=%d step %d tensor %d %s: P %.2e Q %.2e E %.2e"
                  % (rank, t, i, sh, *worst), flush=True)
            assert max(worst) <= TOL, (rank, t, i, sh, worst)
    plan.destroy()


def test_transformer_one_layer_50_steps():
    """The 50 steps of the transformer configuration on a sub-set the oracle can follow: one whole layer (four
    2048 x 2048 projections, 8192 x 2048, 2048 x 8192: 50 M elements) with its vectors, bf16 gradients and output,
    rank 16 on the matrix-core kernels, free-running in windows like the other long runs.  (The embedding and the
    24-layer launch configuration are covered by test_transformer_full_size_sampled.)"""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    shapes = WL.transformer_shapes(layers=1)[1:]          # without the embedding
    assert shapes[0] == (2048, 2048) and sum(len(s) == 2 for s in shapes) == 6
    wl = WL.Workload("transformer-1-layer", shapes, 64, 1.0 / np.arange(1, 65), 0.001)
    _run(wl, rank=16, workers=1, steps=_steps("PSGD_PARITY_STEPS_TRANSFORMER_LAYER", 50), seed=16, resync=RESYNC,
         expect_resident=False, grad_bf16=True, out_bf16=True)


# ---- several subspace iterations per step (Appendix G.7) --------------------------------------------------

def _run_iterations(wl, rank, workers, iterations, seed, tuning=None, grad_bf16=False, one_call=False,
                    expect_resident=None):
    """psgd_compress, iterations - 1 calls of psgd_iterate, psgd_decompress, from a fresh Q every step,
    against the oracle's best_approx_compress on the same M = g + e followed by its decompression."""
    from oracle import powersgd_oracle as O
    from paper_1905_13727_amd import workloads as WL
    from gpu_harness import GpuRun, rel_fro
    factors = WL.planted_factors(wl, seed)
    gpu = GpuRun(wl.shapes, rank, workers, WL.initial_q(wl, rank, seed), tuning, grad_bf16=grad_bf16)
    stream = torch.cuda.current_stream(gpu.dev).cuda_stream
    mats = [i for i, sh in enumerate(wl.shapes) if len(sh) > 1]
    errs = [[None if len(sh) == 1 else np.zeros(O.matrix_view(sh)) for sh in wl.shapes] for _ in range(workers)]
    for t in range(2):
        q0 = WL.initial_q(wl, rank, seed + 100 + t)    # no warm start: a fresh Q every step
        gpu.set_q(q0)
        grads = [WL.gradients(wl, factors, seed, t, w) for w in range(workers)]
        if grad_bf16:
            grads = [[WL.bf16_round(g) for g in gw] for gw in grads]
        gpu.upload(grads)
        if one_call:
            gpu.plan.step_iterations(gpu.grad, gpu.err, gpu.q, gpu.p, gpu.out, gpu.ws, iterations, stream)
        else:
            gpu.plan.compress(gpu.grad, gpu.err, gpu.q, gpu.p, gpu.ws, stream)
            for _ in range(iterations - 1):
                gpu.plan.iterate(gpu.err, gpu.q, gpu.p, gpu.ws, stream)
            gpu.plan.decompress(gpu.p, gpu.q, gpu.err, gpu.grad, gpu.out, gpu.ws, stream)
        resident = gpu.plan.check(stream)
        if expect_resident is not None:
            assert resident == expect_resident
        torch.cuda.synchronize(gpu.dev)
        got = gpu.download()
        new_errs = [[None] * len(wl.shapes) for _ in range(workers)]
        for i in mats:
            sh = O.matrix_view(wl.shapes[i])
            Ms = [np.asarray(grads[w][i], dtype=np.float64).reshape(sh) + errs[w][i] for w in range(workers)]
            P_hat, Q = O.best_approx_compress(Ms, q0[i].astype(np.float64), iterations)
            delta = O.decompress(P_hat, Q)
            assert rel_fro(got["P_hat"][i], P_hat) <= TOL, (wl.name, t, i, "P_hat", rel_fro(got["P_hat"][i], P_hat))
            assert rel_fro(got["Q"][i], Q) <= TOL, (wl.name, t, i, "Q")
            assert rel_fro(np.asarray(got["out"][i]).reshape(sh), delta) <= TOL, (wl.name, t, i, "out")
            for w in range(workers):
                new_errs[w][i] = Ms[w] - delta
                # full-rank case: the new error memory is a rounding residue, measured against ||M_w|| (as in compare())
                scale = np.linalg.norm(Ms[w]) if min(rank, *sh) == min(sh) else np.linalg.norm(new_errs[w][i])
                assert np.linalg.norm(np.asarray(got["err"][w][i]).reshape(sh) - new_errs[w][i]) <= TOL * scale, \
                    (wl.name, t, i, w, "err")
        # the oracle carries its own error memory on (rounded to fp32 as the GPU holds it)
        errs = [[None if e is None else e.astype(np.float32).astype(np.float64) for e in ew] for ew in new_errs]
        gpu.set_err([[np.zeros(wl.shapes[i], dtype=np.float32) if e is None else e.reshape(wl.shapes[i])
                      for i, e in enumerate(ew)] for ew in errs])
    gpu.plan.destroy()


@pytest.mark.parametrize("iterations", [2, 4])
def test_iterations_streaming(iterations):
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run_iterations(WL.tiny(), rank=2, workers=1, iterations=iterations, seed=11)
    _run_iterations(_workload(RAGGED_1W[:10]), rank=3, workers=2, iterations=iterations, seed=12)


@pytest.mark.parametrize("iterations", [2, 4])
def test_iterations_on_chip(iterations):
    """psgd_step_iterations on a plan in resident mode: all the rounds of P = M Q, orthogonalise, Q = M^T P_hat run on
    the tile of M held in registers, one kernel per step.  Tiny and the full-size ResNet18-shaped set at rank 2, a
    ragged set at ranks 3 and 4 (24-row strips); and the same call on plans that stream (the split calls in one)."""
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    _run_iterations(WL.tiny(), rank=2, workers=1, iterations=iterations, seed=21, one_call=True, expect_resident=True)
    _run_iterations(WL.resnet18(), rank=2, workers=1, iterations=iterations, seed=22, one_call=True,
                    expect_resident=True)
    _run_iterations(_workload(RAGGED_1W), rank=3, workers=1, iterations=iterations, seed=23, one_call=True,
                    expect_resident=True)
    _run_iterations(_workload(RAGGED_1W), rank=4, workers=1, iterations=iterations + 1, seed=24, one_call=True,
                    expect_resident=True)
    _run_iterations(_workload(RAGGED_1W), rank=1, workers=1, iterations=iterations, seed=25, one_call=True,
                    expect_resident=True)
    _run_iterations(_workload(RAGGED_1W[:10]), rank=3, workers=2, iterations=iterations, seed=26, one_call=True,
                    expect_resident=False)


def test_iterations_matrix_cores():
    _need_gpu()
    from paper_1905_13727_amd import workloads as WL
    wl = WL.Workload("tr-small", list(TRANSFORMER_SMALL), 64, 1.0 / np.arange(1, 65), 0.001)
    _run_iterations(wl, rank=16, workers=1, iterations=3, seed=13)
    _run_iterations(wl, rank=4, workers=2, iterations=2, seed=14, grad_bf16=True, tuning={"bf16_valu": 0})
    _run_iterations(wl, rank=4, workers=2, iterations=2, seed=14, grad_bf16=True)   # streaming kernels
