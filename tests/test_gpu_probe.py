"""The stream probe (a measurement aid): its read sweep sees every float once, its update sweep
leaves the buffer as it was (it adds 0.0f)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_probe_stream_reads_everything_and_changes_nothing():
    import torch
    from paper_1003_0358_amd import binding
    lib = binding.load()
    rng = np.random.default_rng(0)
    for nf, wgs in ((4, 1), (4 * 1000 + 4, 3), (1 << 20, 256), (4 * 123457, 1000)):
        v = rng.integers(-8, 9, nf).astype(np.float32)          # small integers: every sum is exact
        buf = torch.from_numpy(v).cuda()
        sink = torch.zeros(4 * wgs, dtype=torch.float32, device="cuda")
        lib.check(lib.probe_stream(buf, nf, wgs, 3, sink))
        torch.cuda.synchronize()
        assert np.array_equal(buf.cpu().numpy(), v)
        assert float(sink.cpu().numpy().astype(np.float64).sum()) == float(v.astype(np.float64).sum())
    assert lib.probe_stream(buf, 6, 1, 1, sink) == binding.E_ARG          # not a multiple of 4
    assert lib.probe_stream(None, 4, 1, 1, sink) == binding.E_ARG
    assert lib.probe_stream(buf, 4, 0, 1, sink) == binding.E_ARG
    assert lib.probe_stream(buf, 4, 1, 0, sink) == binding.OK             # no sweeps: nothing to do
