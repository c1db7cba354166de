"""The epoch driver (deform the whole set anew every epoch, one on-line pass, validate on the
un-deformed set, keep the best weights, shrink the learning rate by a constant factor): host logic
around the library calls, checked for what it must do rather than against the oracle's arithmetic,
which the parity tests of the calls themselves cover."""
import numpy as np
import pytest

from inputs_util import pixels_to_inputs
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
    return np.argmax(pixels_to_inputs(imgs).astype(np.float64) @ T.T, axis=1).astype(np.int32)


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
    wide = binding.default_deform_params()
    wide.beta_deg = 15.0
    for at in range(0, 3000, 700):
        m = min(700, 3000 - at)
        x = binding.deform_batch(src[at:at + m], 7, at, wide, labels=labels[at:at + m], beta_similar_deg=7.5)
        b.bp_steps(x, labels[at:at + m], float(np.float32(1e-3)))
    b.status()
    assert np.array_equal(a.get_params(), b.get_params())
    val = binding.deform_batch(src, 0, 0, epochs.identity_params())
    assert np.array_equal(val.cpu().numpy(), pixels_to_inputs(imgs))     # validation inputs are un-deformed
    assert hist[0]["val_errors"] == int((b.classify(val) != labels).sum().item())
    assert hist[0]["val_n"] == 3000 and hist[0]["eta"] == float(np.float32(1e-3))
    a.close(); b.close()

    # (2) a few epochs on a learnable task: the validation error falls well below chance and the
    # network ends with the weights of its best epoch
    c = binding.Mlp(sizes, seed=1)
    mild = binding.DeformParams(6.0, 8.0, 3.0, 5.0, 21, 0, 0)
    hist = epochs.run_epochs(c, src, labels, epochs=6, eta_start=3e-3, eta_end=3e-4, params=mild, seed=2)
    errs = [h["val_errors"] for h in hist]
    assert hist[0]["train_loss"] > hist[-1]["train_loss"]
    assert min(errs) < 0.35 * 3000                      # chance would be about 0.9 * 3000
    final = int((c.classify(val) != labels).sum().item())
    assert final == min(errs)
    etas = [h["eta"] for h in hist]
    assert etas[0] == pytest.approx(3e-3, rel=1e-6) and etas[-1] == pytest.approx(3e-4, rel=1e-5)
    c.close()


def test_epochs_against_the_oracle(oracle):
    """The epoch driver against the same epochs taken by the oracle (sections "Data",
    "Architectures", "Deforming images ...", "Results"): every epoch deforms the whole set anew
    (image k of epoch e draws from index e * n + k; digits 1 and 7 get the smaller angle bound),
    takes one on-line pass over it at that epoch's learning rate, and validates on the un-deformed
    set; the weights of the epoch with the fewest validation errors are the ones kept.  Chunks of
    700 over 2,000 images, so the chunking must not show either."""
    import torch
    from paper_1003_0358_amd import binding, epochs
    n, E, seed = 2000, 3, 11
    sizes = [784, 300, 10]
    imgs, _ = datagen.stroke_images(n, seed=41)
    lab = _teacher_labels(imgs, seed=3)
    src, labels = torch.from_numpy(imgs).cuda(), torch.from_numpy(lab).cuda()
    m = binding.Mlp(sizes, seed=9)
    p0 = m.get_params()
    hist = epochs.run_epochs(m, src, labels, epochs=E, eta_start=1e-3, eta_end=1e-5, seed=seed, chunk=700,
                             keep_best=True, autotune=False)
    got = m.get_params()
    m.close()

    # the learning rates: a constant factor per epoch from the first value to the last, as float32
    etas = np.array([h["eta"] for h in hist], dtype=np.float32)
    want = np.array([1e-3, 1e-4, 1e-5])
    assert np.abs(etas.astype(np.float64) / want - 1).max() < 2e-7
    assert [float(e) for e in etas] == [h["eta"] for h in hist]        # they are float32 values already

    oracle.set_threads(min(oracle.max_threads(), 16))
    beta = np.where((lab == 1) | (lab == 7), 7.5, 15.0).astype(np.float32)      # the paper's rule
    val = oracle.deform_batch(imgs, 0, 0, alpha=0.0, beta_deg=0.0, gamma_pct=0.0, mode="f32")   # un-deformed
    p, after = p0, []
    for e in range(E):
        x = oracle.deform_batch(imgs, seed, e * n, mode="f32", beta_each=beta)
        p, loss = oracle.bp_steps(sizes, p, x, lab, etas[e], "f32")
        after.append(p)
        logits = oracle.logits_batch(sizes, p, val, "f64")
        ref = np.argmax(logits, axis=1)
        top2 = np.sort(logits, axis=1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > 1e-4
        sure = int((ref[clear] != lab[clear]).sum())
        # validation errors: those of the clear decisions, plus at most the decisions within rounding
        assert sure <= hist[e]["val_errors"] <= sure + int((~clear).sum()), (e, sure, hist[e])
        assert clear.sum() >= n - 20
        assert abs(hist[e]["train_loss"] - float(loss.astype(np.float64).mean())) <= 1e-5
        assert hist[e]["val_n"] == n
    oracle.set_threads(1)
    # the network ends with the weights of its best epoch (the first of the lowest error count)
    errs = [h["val_errors"] for h in hist]
    best = int(np.argmin(errs))
    assert np.abs(got - after[best]).max() <= 1e-4
    if best != E - 1:
        assert np.abs(got - after[E - 1]).max() > 1e-4 or errs[best] == errs[E - 1]
    assert errs[0] > min(errs) or errs[0] < 0.5 * n                    # training did something


def test_count_errors_and_mean_loss():
    import torch
    from paper_1003_0358_amd import binding
    rng = np.random.default_rng(0)
    for n in (1, 63, 1024, 60000):
        a = rng.integers(0, 10, n).astype(np.int32)
        b = a.copy()
        flip = rng.random(n) < 0.3
        b[flip] = (b[flip] + 1 + rng.integers(0, 9, int(flip.sum()))) % 10
        assert binding.count_errors(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()) == int((a != b).sum())
        v = rng.uniform(0, 5, n).astype(np.float32)
        got = binding.mean_loss(torch.from_numpy(v).cuda())
        assert got == pytest.approx(float(v.astype(np.float64).mean()), rel=1.5e-7)
    empty = torch.zeros(0, dtype=torch.int32, device="cuda")
    assert binding.count_errors(empty, empty) == 0
