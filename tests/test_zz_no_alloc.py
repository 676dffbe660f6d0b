"""orthdion_step_static (the step on the library's own device scratch, for callers that cannot
allocate) against orthdion_step on a caller workspace: same kernels in the same order, so
the results must agree bit for bit - which is inside every tolerance of the parity tests.
Two calls in a row, the second with a smaller input: the scratch keeps the first call's
contents and the second must not be disturbed by them."""
import numpy as np
import pytest

from gpu_harness import GpuRun
from paper_2605_16341_amd import binding, synth

pytestmark = pytest.mark.gpu


def _pair(shape, r, variant, steps=2):
    import torch
    w = synth.Workload(f"static{shape[0]}x{shape[1]}r{r}", (shape,), r=r, x_dtype="bf16", steps=steps)
    stream, st = synth.make_stream(w, 0), synth.make_state(w, 0)
    ref = GpuRun(w.shapes, r, "bf16", [st], variant=variant, mu=w.mu, lr=w.lr)
    twin = GpuRun(w.shapes, r, "bf16", [st], variant=variant, mu=w.mu, lr=w.lr)
    assert binding.orthdion_workspace_bytes(twin.opt.handle) <= binding.orthdion_static_scratch_bytes()
    sh = torch.cuda.current_stream().cuda_stream
    for t in range(steps):
        g = stream.gradient(t)
        assert ref.step([g]) == [0]
        from paper_2605_16341_amd.device_inputs import to_device
        gd = to_device(g, torch)
        binding.orthdion_step_static(twin.opt.handle, [twin.X[0].data_ptr()], [gd.data_ptr()], [twin.M[0].data_ptr()],
                                     [twin.Q[0].data_ptr()], sh)
        torch.cuda.synchronize()
        assert twin.opt.info() == [0]
        a, b = ref.fetch(0, with_factors=False), twin.fetch(0, with_factors=False)
        for key in ("X", "M", "Q"):
            assert a[key].tobytes() == b[key].tobytes(), (shape, r, variant, t, key)
    return True


def test_static_scratch_step_matches_workspace_step_twice_second_smaller():
    assert _pair((640, 512), 128, "qr")
    assert _pair((256, 192), 32, "qr")            # smaller input right after, on the same scratch
    assert _pair((384, 640), 136, "colnorm")


def test_static_scratch_step_rejects_what_does_not_fit():
    w = synth.WORKLOADS["C5-r1024"]
    h = binding.orthdion_create(w.shapes, w.r, binding.ORTHDION_BF16, binding.ORTHDION_BF16)
    assert binding.orthdion_workspace_bytes(h) > binding.orthdion_static_scratch_bytes()
    with pytest.raises(binding.OrthDionError) as exc:
        binding.orthdion_step_static(h, [256], [256], [256], [256], 0)
    assert exc.value.status == binding.ORTHDION_E_WORKSPACE_TOO_SMALL
    binding.orthdion_destroy(h)
