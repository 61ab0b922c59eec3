"""psgd_step_static: the step for callers that cannot allocate.  Its workspace is an array the library holds on the
GPU; everything else is psgd_step.  Checked against psgd_step (caller's workspace) bit for bit, on two calls in a
row that share the array, the second on a smaller model, and on its refusals."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu


def _state(plan, dev, seed):
    s = plan.sizes
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    W = plan.workers
    return dict(grad=(torch.randn(W * s.grad_stride, generator=gen) * 0.01).to(dev),
                err=(torch.randn(W * s.err_stride, generator=gen) * 0.003).to(dev),
                q=torch.randn(s.q_elems, generator=gen).to(dev),
                p=torch.zeros(s.p_elems, device=dev), out=torch.zeros(s.out_elems, device=dev))


def test_static_workspace_step_equals_psgd_step():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1905_13727_amd import binding as B, workloads as WL
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream(dev).cuda_stream
    big = B.Plan(WL.resnet18().shapes, 2, 3)                 # streams (three workers): partial P, Q and Gram in the workspace
    small = B.Plan([(37, 91), (7,), (130, 1028), (5, 3), (2600, 12)], 4, 2)
    assert small.sizes.workspace_bytes < big.sizes.workspace_bytes <= 32 << 20
    # a plan whose tables are not on the device is refused (the upload would allocate) ...
    st = _state(big, dev, 1)
    with pytest.raises(B.PsgdError) as ei:
        big.step_static(st["grad"], st["err"], st["q"], st["p"], st["out"], stream)
    assert ei.value.status == B.PSGD_EINVAL and "not on the device" in big.last_error()
    # ... psgd_plan_check puts them there
    assert big.check(stream) is False and small.check(stream) is False
    for plan, seed in ((big, 1), (small, 2), (big, 3)):     # back to back: the array keeps the previous call's contents
        for step in range(2):
            a, b = _state(plan, dev, seed + 10 * step), _state(plan, dev, seed + 10 * step)
            ws = torch.full((plan.sizes.workspace_bytes // 4 + 64,), float("nan"), device=dev)
            plan.step(a["grad"], a["err"], a["q"], a["p"], a["out"], ws, stream)
            plan.step_static(b["grad"], b["err"], b["q"], b["p"], b["out"], stream)
            plan.check(stream)
            torch.cuda.synchronize(dev)
            for key in ("err", "q", "p", "out"):
                assert torch.equal(a[key], b[key]), (seed, step, key)
            assert torch.isfinite(b["out"]).all() and b["out"].abs().max() > 0
    # a plan whose workspace does not fit the array is refused
    huge = B.Plan(WL.transformer(24).shapes, 4, 1, B.PSGD_BF16, B.PSGD_BF16)
    huge.set_tuning("bf16_valu", 1)   # on the streaming kernels, whose partial sums for this set need more than the array holds
    assert huge.sizes.workspace_bytes > 32 << 20
    huge.check(stream)
    with pytest.raises(B.PsgdError) as ei:
        huge.step_static(1, 1, 1, 1, 1, stream)
    assert ei.value.status == B.PSGD_EUNSUPPORTED and "workspace" in huge.last_error()
    lib = B.load_library()
    assert lib.psgd_step_static(None, 1, 1, 1, 1, 1, None) == B.PSGD_EINVAL
    assert lib.psgd_step_static(big._h, None, 1, 1, 1, 1, None) == B.PSGD_EINVAL
    for plan in (big, small, huge):
        plan.destroy()
