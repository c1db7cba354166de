"""dbsn_classify_static, the entry point that allocates nothing: its labels against dbsn_classify's
on two calls in a row through the C ABI, the second with a smaller input (the static staging
array keeps the first call's contents), and the size limit."""
import numpy as np
import pytest

from inputs_util import pixels_to_inputs
from paper_1003_0358_amd import datagen

pytestmark = pytest.mark.gpu


def test_classify_static_matches_classify_on_two_calls_in_a_row():
    import torch
    from paper_1003_0358_amd import binding
    sizes = [784, 1000, 500, 10]
    m = binding.Mlp(sizes, seed=6)
    lib = m.lib
    img, lab = datagen.stroke_images(3000, seed=51)
    xs = torch.from_numpy(pixels_to_inputs(img)).cuda()
    # train a little so that the outputs are not all alike
    m.bp_steps(xs[:200], torch.from_numpy(lab[:200]).cuda(), 1e-2)
    m.status()
    want_big = m.classify(xs).cpu().numpy()
    small_in = xs[517:1530].contiguous()                  # 1013 samples: a ragged tile of other images
    want_small = m.classify(small_in).cpu().numpy()
    assert len(np.unique(want_big)) >= 3

    out_big = torch.full((3000,), -1, dtype=torch.int32, device="cuda")
    out_small = torch.full((1013,), -1, dtype=torch.int32, device="cuda")
    lib.check(lib.classify_static(m.h, xs, 3000, out_big))
    lib.check(lib.classify_static(m.h, small_in, 1013, out_small))
    m.status()
    assert np.array_equal(out_big.cpu().numpy(), want_big)
    assert np.array_equal(out_small.cpu().numpy(), want_small)

    # a second network of another width shares the array: its call must not see the first one's values
    other = binding.Mlp([784, 301, 77, 10], seed=2)
    want_other = other.classify(xs[:700]).cpu().numpy()
    out_other = torch.full((700,), -1, dtype=torch.int32, device="cuda")
    lib.check(lib.classify_static(other.h, xs[:700], 700, out_other))
    other.status()
    assert np.array_equal(out_other.cpu().numpy(), want_other)
    other.close()

    # limits and arguments: 2 * n * 4 * 1000 bytes must fit 64 MiB -> at most 8388 samples
    assert lib.classify_static(m.h, xs, 8389, out_big) == binding.E_SHAPE
    assert "at most 8388 samples" in lib.last_error()
    assert lib.classify_static(m.h, xs, 0, out_big) == binding.OK
    assert lib.classify_static(m.h, None, 5, out_big) == binding.E_ARG
    assert lib.classify_static(m.h, xs, -1, out_big) == binding.E_ARG
    assert lib.classify_static(None, xs, 5, out_big) == binding.E_ARG
    m.close()
