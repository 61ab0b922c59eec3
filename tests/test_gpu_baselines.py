"""GPU parity of the Random Block and Random K baselines (Appendix G inside Algorithm 2) against the CPU oracle.

Positions are index work: Delta' must be non-zero exactly where the oracle's is, and outside the kept set the new
error memory is the single fp32 addition g + e, which has one correct result: compared bit for bit when both sides
start the step from the same fp32 state.  Values are floating point: relative Frobenius error <= 1e-5 per tensor
(and worker) at every step of a free-running run, as for the PowerSGD path."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

gpu = pytest.mark.gpu

TOL = 1e-5


class BaselineRun:
    def __init__(self, shapes, rank, workers, device="cuda:0"):
        from paper_1905_13727_amd import binding as B
        from paper_1905_13727_amd.flat import FlatLayout
        self.dev = torch.device(device)
        self.plan = B.Plan(shapes, rank, workers)
        self.lay = FlatLayout(self.plan, shapes)
        self.shapes = [tuple(s) for s in shapes]
        s = self.plan.sizes
        self.W = workers
        self.grad = torch.zeros(workers * s.grad_stride, device=self.dev)
        self.err = torch.zeros(workers * max(1, s.err_stride), device=self.dev)
        self.out = torch.full((max(1, s.out_elems),), float("nan"), device=self.dev)
        self.vals = torch.full((max(1, s.kept_elems),), float("nan"), device=self.dev)
        self.kept = [self.plan.kept(t) for t in range(len(shapes))]

    def upload(self, grads):
        s = self.plan.sizes
        host = np.zeros((self.W, s.grad_stride), dtype=np.float32)
        for w in range(self.W):
            host[w, : s.n_mat_elems + s.n_vec_elems] = self.lay.pack_flat(grads[w])
        self.grad.copy_(torch.from_numpy(host.reshape(-1)))

    def set_err(self, errs):
        s = self.plan.sizes
        host = np.zeros((self.W, s.err_stride), dtype=np.float32)
        for w in range(self.W):
            host[w] = self.lay.pack_flat(errs[w], matrices_only=True)
        self.err.copy_(torch.from_numpy(host.reshape(-1)))

    def step(self, grads, starts=None, indices=None):
        self.upload(grads)
        stream = torch.cuda.current_stream(self.dev).cuda_stream
        if starts is not None:
            st = torch.tensor([0 if v is None else int(v) for v in starts], dtype=torch.int64, device=self.dev)
            self.plan.random_block_step(self.grad, self.err, st, self.vals, self.out, stream)
        else:
            packed = np.zeros(max(1, self.plan.sizes.kept_elems), dtype=np.int64)
            for t, idx in enumerate(indices):
                if idx is not None:
                    off, n = self.kept[t]
                    assert len(idx) == n
                    packed[off: off + n] = idx
            ix = torch.from_numpy(packed).to(self.dev)
            self.plan.random_k_step(self.grad, self.err, ix, self.vals, self.out, stream)
        self.plan.check(stream)
        torch.cuda.synchronize(self.dev)
        s = self.plan.sizes
        err = self.err.cpu().numpy()[: self.W * s.err_stride].reshape(self.W, max(1, s.err_stride))
        vals = self.vals.cpu().numpy()
        return {"out": self.lay.unpack_flat(self.out.cpu().numpy()),
                "err": [self.lay.unpack_flat(err[w], matrices_only=True) for w in range(self.W)],
                "values": [None if n == 0 else vals[off: off + n] for off, n in self.kept]}


def _rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    if nb == 0.0:
        return 0.0 if np.linalg.norm(a) == 0.0 else np.inf
    return float(np.linalg.norm(a - b) / nb)


def _compare(got, want, shapes, workers, where):
    for t, s in enumerate(shapes):
        w_out = np.asarray(want["out"][t]).reshape(got["out"][t].shape)
        assert _rel(got["out"][t], w_out) <= TOL, (where, t, "out")
        if len(s) == 1:
            continue
        # index work: Delta' is non-zero at exactly the kept positions
        assert np.array_equal(got["out"][t] != 0, w_out != 0), (where, t, "positions")
        assert _rel(got["values"][t], want["values"][t]) <= TOL, (where, t, "values")
        assert np.array_equal(got["values"][t] != 0, want["values"][t] != 0), (where, t, "value slots")
        for w in range(workers):
            assert _rel(got["err"][w][t], want["err"][w][t]) <= TOL, (where, t, w, "err")
            if workers == 1:   # what is sent leaves the memory entirely
                assert not got["err"][0][t][w_out != 0].any(), (where, t, "kept entries of e")


def _workload(shapes, sigma=0.01):
    from paper_1905_13727_amd import workloads as WL
    return WL.Workload("custom", list(shapes), 4, 1.0 / np.arange(1, 5), sigma)


def _run(wl, rank, workers, steps, seed, force_late_start=False):
    """Both compressors, free-running for `steps` steps (each side carries its own error memory), then one step
    from a common fp32 state in which the untouched part of the error memory must agree bit for bit."""
    from oracle import powersgd_oracle as O
    from paper_1905_13727_amd import workloads as WL
    factors = WL.planted_factors(wl, seed)
    for kind in ("block", "k"):
        gpu = BaselineRun(wl.shapes, rank, workers)
        errs = [[None if len(s) == 1 else np.zeros(O.matrix_view(s)) for s in wl.shapes] for _ in range(workers)]
        for t in range(steps + 1):
            common = t == steps
            if common:      # last step: the oracle restarts from the GPU-representable state
                errs = [[None if e is None else e.astype(np.float32).astype(np.float64) for e in ew] for ew in errs]
                gpu.set_err([[np.zeros(wl.shapes[i], dtype=np.float32) if e is None else e.reshape(wl.shapes[i])
                              for i, e in enumerate(ew)] for ew in errs])
            grads = [WL.gradients(wl, factors, seed, t, w) for w in range(workers)]
            if kind == "block":
                starts = WL.block_starts(wl, rank, seed, t)
                if force_late_start:     # blocks cut short by the end of the vector
                    starts = [None if s is None else int(np.prod(wl.shapes[i])) - 1 - (i % 3)
                              for i, s in enumerate(starts)]
                got = gpu.step(grads, starts=starts)
                want = O.random_block_step(grads, errs, starts, rank)
            else:
                idx = WL.random_indices(wl, rank, seed, t)
                got = gpu.step(grads, indices=idx)
                want = O.random_k_step(grads, errs, idx, rank)
            _compare(got, want, wl.shapes, workers, (wl.name, kind, rank, workers, t))
            if common:
                for i, s in enumerate(wl.shapes):
                    if len(s) == 1:
                        continue
                    untouched = np.asarray(want["out"][i]) == 0
                    for w in range(workers):
                        exact = (np.asarray(grads[w][i], dtype=np.float32) + errs[w][i].astype(np.float32).reshape(s))
                        assert np.array_equal(got["err"][w][i][untouched], exact[untouched]), (kind, i, w)
            errs = want["err"]
        gpu.plan.destroy()


RAGGED = [(37, 91), (7,), (50, 650), (130, 1028), (5, 3), (300, 2), (1, 40), (1031,), (3, 4700), (257, 260), (64, 27)]


@gpu
@pytest.mark.parametrize("rank,workers", [(1, 1), (2, 3), (4, 2)])
def test_baselines_ragged_shapes(rank, workers):
    """Row lengths and element counts that are not multiples of 4 (scalar tails), a matrix smaller than its budget
    (every entry kept), vectors between matrices, one and several workers."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    _run(_workload(RAGGED), rank, workers, steps=3, seed=300 + rank)


@gpu
def test_random_block_cut_short_at_the_end():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    _run(_workload(RAGGED), 2, 2, steps=1, seed=310, force_late_start=True)


@gpu
def test_baselines_tiny_config_10_steps():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_13727_amd import workloads as WL
    _run(WL.tiny(), 2, 1, steps=10, seed=0)


@gpu
@pytest.mark.parametrize("workers,rank,steps", [(1, 2, 5), (16, 4, 1)])
def test_baselines_resnet18_full_size(workers, rank, steps):
    """The ResNet18-shaped set at full size, in the launch configuration bench.py times."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_13727_amd import workloads as WL
    _run(WL.resnet18(), rank, workers, steps=steps, seed=320 + workers)


@gpu
def test_baselines_lstm_full_size():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_13727_amd import workloads as WL
    _run(WL.lstm(), 4, 1, steps=1, seed=330)


def test_baselines_refuse_bf16_plans_and_null_pointers():
    from paper_1905_13727_amd import binding as B
    lib = B.load_library()
    plan = B.Plan([(8, 8)], 2, 1, B.PSGD_BF16, B.PSGD_BF16)
    assert lib.psgd_random_block_step(plan._h, 1, 1, 1, 1, 1, None) == B.PSGD_EUNSUPPORTED
    assert lib.psgd_random_k_step(plan._h, 1, 1, 1, 1, 1, None) == B.PSGD_EUNSUPPORTED
    plan = B.Plan([(8, 8), (5,)], 2, 1)
    assert lib.psgd_random_block_step(plan._h, 1, 1, None, 1, 1, None) == B.PSGD_EINVAL
    assert lib.psgd_random_k_step(None, 1, 1, 1, 1, 1, None) == B.PSGD_EINVAL
    assert plan.kept(0) == (0, 32) and plan.kept(1) == (-1, 0) and plan.sizes.kept_elems == 32
