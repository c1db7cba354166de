"""The epoch driver (deform the whole set anew every epoch, one on-line pass, validate on the
un-deformed set, keep the best weights, shrink the learning rate by a constant factor): host logic
around the library calls, checked for what it must do rather than against the oracle's arithmetic,
which the parity tests of the calls themselves cover."""
import numpy as np
import pytest

from paper_1003_0358_amd import datagen

pytestmark = pytest.mark.gpu


def test_eta_schedule_is_geometric_between_the_paper_s_ends():
    from paper_1003_0358_amd import epochs
    eta = epochs.eta_schedule(13)
    assert eta.dtype == np.float32 and len(eta) == 13
    assert eta[0] == np.float32(1e-3) and eta[-1] == pytest.approx(1e-6, rel=1e-5)
    r = eta[1:].astype(np.float64) / eta[:-1].astype(np.float64)
    assert np.allclose(r, r[0], rtol=1e-5) and 0 < r[0] < 1
    assert list(epochs.eta_schedule(1)) == [np.float32(1e-3)]


def _teacher_labels(imgs, seed=0):
    """Labels a net can learn: the largest of ten fixed random projections of the image."""
    rng = np.random.default_rng(seed)
    T = rng.normal(size=(10, 784))
    return np.argmax(datagen.to_inputs(imgs).astype(np.float64) @ T.T, axis=1).astype(np.int32)


def test_one_epoch_is_the_sequence_of_calls_and_training_learns():
    import torch
    from paper_1003_0358_amd import binding, epochs
    imgs, _ = datagen.stroke_images(3000, seed=31)
    lab = _teacher_labels(imgs)
    src, labels = torch.from_numpy(imgs).cuda(), torch.from_numpy(lab).cuda()
    sizes = [784, 300, 10]

    # (1) one epoch of the driver == deform + bp_steps by hand, bit for bit
    a = binding.Mlp(sizes, seed=5)
    hist = epochs.run_epochs(a, src, labels, epochs=1, eta_start=1e-3, seed=7, chunk=700, keep_best=False)
    b = binding.Mlp(sizes, seed=5)
    beta = binding.beta_for_labels(labels)
    for at in range(0, 3000, 700):
        m = min(700, 3000 - at)
        x = binding.deform_batch(src[at:at + m], 7, at, beta_deg=beta[at:at + m])
        b.bp_steps(x, labels[at:at + m], float(np.float32(1e-3)))
    b.status()
    assert np.array_equal(a.get_params(), b.get_params())
    val = binding.deform_batch(src, 0, 0, epochs.identity_params())
    assert np.array_equal(val.cpu().numpy(), datagen.to_inputs(imgs))     # validation inputs are un-deformed
    assert hist[0]["val_errors"] == int((b.classify(val) != labels).sum().item())
    assert hist[0]["val_n"] == 3000 and hist[0]["eta"] == float(np.float32(1e-3))
    a.close(); b.close()

    # (2) a few epochs on a learnable task: the validation error falls well below chance and the
    # network ends with the weights of its best epoch
    c = binding.Mlp(sizes, seed=1)
    mild = binding.DeformParams(6.0, 8.0, 3.0, 5.0, 21, 0)
    hist = epochs.run_epochs(c, src, labels, epochs=6, eta_start=3e-3, eta_end=3e-4, params=mild, seed=2)
    errs = [h["val_errors"] for h in hist]
    assert hist[0]["train_loss"] > hist[-1]["train_loss"]
    assert min(errs) < 0.35 * 3000                      # chance would be about 0.9 * 3000
    final = int((c.classify(val) != labels).sum().item())
    assert final == min(errs)
    etas = [h["eta"] for h in hist]
    assert etas[0] == pytest.approx(3e-3, rel=1e-6) and etas[-1] == pytest.approx(3e-4, rel=1e-5)
    c.close()
