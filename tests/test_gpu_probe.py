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


def test_probe_handover_ends_and_nobody_gives_up():
    """The bare hand-over across the chip and inside a die: every poll finds its words (on a device
    whose workgroup g runs on die g % 8 the workgroup-scope stores reach the same die's pollers)."""
    import torch
    from paper_1003_0358_amd import binding
    lib = binding.load()
    buf = torch.ones(2 * 256 * 64, dtype=torch.int64, device="cuda")     # dirty on purpose: the call clears it
    gave = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    for within in (0, 1):
        lib.check(lib.probe_handover(within, 300, buf, gave))
        torch.cuda.synchronize()
        assert int(gave.item()) == 0
        words = buf.cpu().numpy().view(np.uint64).reshape(2, 256, 64)
        assert (words[0] >> np.uint64(32) == 300).all() and (words[1] >> np.uint64(32) == 299).all()   # last two rounds
        assert ((words & np.uint64(0xFFFFFFFF)) == np.arange(64, dtype=np.uint64)).all()
    assert lib.probe_handover(2, 10, buf, gave) == binding.E_ARG
    assert lib.probe_handover(0, -1, buf, gave) == binding.E_ARG
    assert lib.probe_handover(0, 10, None, gave) == binding.E_ARG
