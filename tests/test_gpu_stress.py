"""Ten thousand on-line steps in a row: the persistent kernel (whose workgroups hand partial sums to
each other with no barrier) against the launch-per-phase mode (kernel boundaries order everything)
and against the oracle, and against itself."""
import numpy as np
import pytest

from inputs_util import pixels_to_inputs
from paper_1003_0358_amd import datagen

pytestmark = pytest.mark.gpu


def test_ten_thousand_steps(oracle):
    """A missed or stale hand-over anywhere in 10^4 steps x 5 hand-overs x 256 workgroups would leave
    a weight far off (a stale partial sum is wrong by its whole size, about 1e-2 in a delta, so about
    1e-5 in every weight of a row at once, and it would differ from run to run): two persistent runs
    must agree bit for bit; persistent, launch-per-phase and oracle differ only by summation order and
    the activation's 4e-7: measured 2.6e-7 between the modes, 2.3e-7 against the oracle, 1.4e-6 on a
    loss; asserted at a tenth of the 100-step bar."""
    import torch
    from paper_1003_0358_amd import binding
    sizes = [784, 800, 400, 10]
    n = 10000
    img, lab = datagen.stroke_images(n, seed=77)
    X = pixels_to_inputs(img)
    xs, ys = torch.from_numpy(X).cuda(), torch.from_numpy(lab).cuda()
    eta = np.float32(1e-3)
    res = []
    for mode in (binding.MODE_PERSISTENT, binding.MODE_PERSISTENT, binding.MODE_LAUNCHES):
        m = binding.Mlp(sizes, seed=8, mode=mode)
        p0 = m.get_params()
        loss = torch.zeros(n, dtype=torch.float32, device="cuda")
        # several calls of uneven length, as an epoch driver would make them
        for a, b in ((0, 1), (1, 1000), (1000, 1003), (1003, 7000), (7000, n)):
            m.bp_steps(xs[a:b], ys[a:b], eta, loss[a:b])
        m.status()
        res.append((m.get_params(), loss.cpu().numpy()))
        m.close()
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])
    oracle.set_threads(min(oracle.max_threads(), 16))
    ref, lref = oracle.bp_steps(sizes, p0, X, lab, eta, "f32")
    oracle.set_threads(1)
    d_modes = float(np.abs(res[0][0] - res[2][0]).max())
    d_oracle = float(np.abs(res[0][0] - ref).max())
    d_loss = float(np.abs(res[0][1] - lref).max())
    print("10^4 steps: persistent vs launches %.3g, vs oracle %.3g, loss %.3g" % (d_modes, d_oracle, d_loss))
    assert d_modes <= 1e-5, d_modes
    assert d_oracle <= 1e-5, d_oracle
    assert d_loss <= 1e-4, d_loss
    assert np.abs(res[0][0] - p0).max() > 1e-2          # the weights did move


def test_five_thousand_steps_on_the_full_size_net_in_both_cuts():
    """The 12 M-weight net, whose banded tiles use every register slot: 5,000 steps in five launches,
    twice with the banded cut (bit-identical: a hand-over inside a die that came late or stale would
    show) and once with the plain cut (same step, partial sums grouped differently)."""
    import torch
    from paper_1003_0358_amd import binding
    sizes = [784, 2500, 2000, 1500, 1000, 500, 10]
    n = 5000
    img, lab = datagen.stroke_images(n, seed=78)
    xs, ys = torch.from_numpy(pixels_to_inputs(img)).cuda(), torch.from_numpy(lab).cuda()
    res = []
    for banded in (True, True, False):
        m = binding.Mlp(sizes, seed=9)
        m.set_variant(banded=banded)
        assert (m.get_variant()[2] > 0) == banded
        p0 = m.get_params()
        loss = torch.zeros(n, dtype=torch.float32, device="cuda")
        for a in range(0, n, 1000):
            m.bp_steps(xs[a:a + 1000], ys[a:a + 1000], 1e-3, loss[a:a + 1000])
        m.status()
        res.append((m.get_params(), loss.cpu().numpy()))
        m.close()
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])
    d = float(np.abs(res[0][0] - res[2][0]).max())
    print("5000 steps on the full-size net: banded vs plain cut %.3g" % d)
    assert d <= 1e-5, d
    assert np.abs(res[0][1] - res[2][1]).max() <= 1e-4
    assert np.abs(res[0][0] - p0).max() > 1e-3
