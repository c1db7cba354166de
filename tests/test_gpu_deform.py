"""GPU-vs-oracle parity of the deformation kernel, through the C ABI (run with -m gpu).

Tolerance (the benchmark spec): every deformed pixel within 1e-5 absolute of the oracle.
"""
import numpy as np
import pytest

from inputs_util import pixels_to_inputs
from paper_1003_0358_amd import datagen

pytestmark = pytest.mark.gpu


def _run(imgs, seed, first, **kw):
    import torch
    from paper_1003_0358_amd import binding
    p = binding.default_deform_params()
    for k, v in kw.items():
        setattr(p, k, v)
    src = torch.from_numpy(np.ascontiguousarray(imgs)).cuda()
    out = binding.deform_batch(src, seed, first, p)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_parity_default_parameters(oracle):
    imgs = datagen.stroke_images(600, seed=3)[0]
    got = _run(imgs, seed=17, first=1000)
    oracle.set_threads(8)
    ref32 = oracle.deform_batch(imgs, 17, 1000, mode="f32")
    ref64 = oracle.deform_batch(imgs, 17, 1000, mode="f64")
    oracle.set_threads(1)
    assert np.abs(got - ref32).max() <= 1e-5
    assert np.abs(got - ref64).max() <= 1e-5
    assert np.abs(got - pixels_to_inputs(imgs)).max() > 0.5     # it did deform


@pytest.mark.parametrize("kw", [
    dict(sigma=5.0, alpha=38.0, beta_deg=15.0, gamma_pct=20.0, ktaps=21),   # other end of the paper's ranges
    dict(sigma=2.0, alpha=8.0, beta_deg=0.0, gamma_pct=0.0, ktaps=5),
    dict(sigma=0.0, alpha=1.5, beta_deg=30.0, gamma_pct=50.0, ktaps=1),     # unsmoothed field
    dict(sigma=9.0, alpha=60.0, beta_deg=90.0, gamma_pct=0.0, ktaps=63),    # widest supported kernel
])
def test_parity_other_parameters(oracle, kw):
    imgs = datagen.stroke_images(64, seed=4)[0]
    got = _run(imgs, seed=1, first=0, **kw)
    ref = oracle.deform_batch(imgs, 1, 0, mode="f64", **kw)
    assert np.abs(got - ref).max() <= 1e-5


def test_zero_displacement_is_exact_identity(oracle):
    imgs = datagen.stroke_images(50, seed=5)[0]
    got = _run(imgs, seed=9, first=0, alpha=0.0, beta_deg=0.0, gamma_pct=0.0)
    ref = oracle.deform_batch(imgs, 9, 0, alpha=0.0, beta_deg=0.0, gamma_pct=0.0, mode="f32")
    assert np.array_equal(got, ref)                    # bit for bit the oracle's intensity map
    assert got.min() == -1.0 and got.max() <= 1.0


def test_chunking_empty_and_single(oracle):
    import torch
    from paper_1003_0358_amd import binding
    imgs = datagen.stroke_images(10, seed=6)[0]
    whole = _run(imgs, seed=2, first=40)
    parts = np.concatenate([_run(imgs[:3], 2, 40), _run(imgs[3:4], 2, 43), _run(imgs[4:], 2, 44)])
    assert np.array_equal(whole, parts)
    lib = binding.load()
    dst = torch.full((1, 784), 7.0, device="cuda")
    assert lib.deform_batch(binding.default_deform_params(), dst, 0, 0, 0, dst) == binding.OK
    torch.cuda.synchronize()
    assert float(dst.min()) == 7.0                                # n = 0 writes nothing


def test_more_images_than_workgroups(oracle):
    """70,000 images in one call (the grid is capped below that): check sampled images one by one."""
    imgs = datagen.stroke_images(1000, seed=7)[0]
    big = np.tile(imgs, (70, 1))
    got = _run(big, seed=5, first=123)
    pick = [0, 1, 65535, 65536, 65537, 69999, 31337]
    for k in pick:
        ref = oracle.deform_batch(big[k:k + 1], 5, 123 + k, mode="f32")
        assert np.abs(got[k] - ref[0]).max() <= 1e-5, k
    assert got.min() >= -1.0 and got.max() <= 1.0
    # same source image, different index: different deformation
    assert np.abs(got[0] - got[1000]).max() > 0.1


def test_shear_and_per_image_angle_bounds(oracle):
    """Horizontal shear instead of rotation, and the bound of the angle following the label (section
    "Deforming images ...": 7.5 degrees for the digits 1 and 7, 15 for the others): the library
    takes the labels (dbsn_deform_batch_labels) or one bound per image (dbsn_deform_batch_beta); the
    oracle is given the bounds this test works out from the paper's rule."""
    import torch
    from paper_1003_0358_amd import binding
    imgs, lab = datagen.stroke_images(300, seed=8)
    src = torch.from_numpy(imgs).cuda()
    labels = torch.from_numpy(lab).cuda()
    bh = np.where((lab == 1) | (lab == 7), 7.5, 15.0).astype(np.float32)
    assert 20 < (bh == 7.5).sum() < 120
    beta = torch.from_numpy(bh).cuda()
    oracle.set_threads(8)
    for shear in (1, 0):
        p = binding.default_deform_params()
        p.shear = shear
        p.beta_deg = 15.0                    # the bound of the classes that are not look-alikes
        by_label = binding.deform_batch(src, 21, 500, p, labels=labels, beta_similar_deg=7.5).cpu().numpy()
        p.beta_deg = 99.0                    # (ignored when every image brings its own bound)
        got = binding.deform_batch(src, 21, 500, p, beta_deg=beta).cpu().numpy()
        assert np.array_equal(by_label, got)
        ref32 = oracle.deform_batch(imgs, 21, 500, mode="f32", shear=bool(shear), beta_each=bh)
        ref64 = oracle.deform_batch(imgs, 21, 500, mode="f64", shear=bool(shear), beta_each=bh)
        assert np.abs(got - ref32).max() <= 1e-5
        assert np.abs(got - ref64).max() <= 1e-5
        # another set of look-alike classes, and labels outside 0..63, which count as "other"
        odd = lab.copy(); odd[::7] = -3; odd[3::11] = 64; odd[5::13] = 1000
        mask = (1 << 0) | (1 << 9)
        bo = np.where((odd == 0) | (odd == 9), 3.0, 15.0).astype(np.float32)
        p.beta_deg = 15.0
        lib = binding.load()
        out = torch.empty((300, 784), dtype=torch.float32, device="cuda")
        lib.check(lib.deform_batch_labels(p, src, torch.from_numpy(odd).cuda(), mask, 3.0, 300, 21, 500, out))
        ref = oracle.deform_batch(imgs, 21, 500, mode="f32", shear=bool(shear), beta_each=bo)
        assert np.abs(out.cpu().numpy() - ref).max() <= 1e-5
        # the scalar bound, sheared
        p.beta_deg = 15.0
        got = binding.deform_batch(src[:64], 21, 500, p).cpu().numpy()
        ref = oracle.deform_batch(imgs[:64], 21, 500, mode="f64", shear=bool(shear), beta_deg=15.0)
        assert np.abs(got - ref).max() <= 1e-5
    oracle.set_threads(1)
    # shear with a zero angle bound and nothing else is the identity, exactly
    p = binding.default_deform_params()
    p.shear, p.alpha, p.beta_deg, p.gamma_pct = 1, 0.0, 0.0, 0.0
    got = binding.deform_batch(src[:20], 3, 0, p).cpu().numpy()
    ref = oracle.deform_batch(imgs[:20], 3, 0, alpha=0.0, beta_deg=0.0, gamma_pct=0.0, shear=True, mode="f32")
    assert np.array_equal(got, ref)
    # a shear flag outside {0, 1} is an argument error
    p.shear = 2
    lib = binding.load()
    out = torch.empty((1, 784), dtype=torch.float32, device="cuda")
    assert lib.deform_batch(p, src, 1, 0, 0, out) == binding.E_ARG
    p.shear = 0
    assert lib.deform_batch_labels(p, src, None, 2, 7.5, 1, 0, 0, out) == binding.E_ARG     # labels missing
    assert lib.deform_batch_labels(p, src, labels, 2, float("nan"), 1, 0, 0, out) == binding.E_ARG
    assert lib.deform_batch_beta(p, src, None, 1, 0, 0, out) == binding.E_ARG
    p.kernel = 5
    assert lib.deform_batch(p, src, 1, 0, 0, out) == binding.E_ARG


def test_the_21_tap_kernel_and_the_general_kernel_agree_bit_for_bit():
    """21 taps run in a kernel of their own (padded lines, windows in registers); the general kernel
    computes the same sums in the same order, so the two must give identical floats, rotation and
    shear alike."""
    import torch
    from paper_1003_0358_amd import binding, datagen
    img, lab = datagen.stroke_images(300, seed=31)
    src = torch.from_numpy(img.reshape(300, 784)).cuda()
    for shear in (0, 1):
        p = binding.default_deform_params()
        p.shear = shear
        fast = binding.deform_batch(src, 7, 1234, p).cpu().numpy()
        p.kernel = binding.DEFORM_KERNEL_GENERAL
        general = binding.deform_batch(src, 7, 1234, p).cpu().numpy()
        assert np.array_equal(fast, general)
        assert np.abs(fast - (img.reshape(300, 784) / 127.5 - 1.0)).max() > 0.1   # it did deform
