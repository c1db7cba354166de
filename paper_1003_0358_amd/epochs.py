"""Epoch driver around the library calls, as the paper runs its training (sections "Data",
"Architectures", "Deforming images ...", "Results"):

* at the beginning of every epoch the whole training set is deformed anew (dbsn_deform_batch with
  first_index = epoch * n, so every epoch sees different deformations of every image); chunk by
  chunk, on a side stream, while the network trains on the chunk before;
* one on-line back-propagation pass over it (dbsn_bp_steps), with a learning rate that shrinks by
  a constant factor after each epoch, from eta_start down to eta_end;
* validation on the UN-deformed training set (or a set the caller gives), forward only
  (dbsn_classify); the weights with the lowest validation error are the ones kept.

Host logic only: every array operation on the data runs in the library's kernels (the un-deformed
inputs are produced by the deformation kernel with all amplitudes at zero, which is the exact
intensity map; the angle bound per class, the error count and the mean loss are library calls).
"""
import numpy as np

from . import binding


def eta_schedule(epochs, eta_start=1e-3, eta_end=1e-6):
    """Learning rates of the epochs as float32: eta_start * f**e with the constant f that reaches
    eta_end in the last epoch."""
    if epochs < 1:
        return np.zeros(0, np.float32)
    if epochs == 1:
        return np.array([eta_start], np.float32)
    f = (eta_end / eta_start) ** (1.0 / (epochs - 1))
    return np.array([eta_start * f ** e for e in range(epochs)], dtype=np.float32)


def identity_params():
    """Deformation parameters that leave the image alone: the kernel then only maps intensities to
    p / 127.5 - 1."""
    return binding.DeformParams(0.0, 0.0, 0.0, 0.0, 1, 0, 0)


def run_epochs(mlp, train_u8, train_labels, epochs, eta_start=1e-3, eta_end=1e-6, params=None,
               beta_by_label=True, seed=0, chunk=1000, val_u8=None, val_labels=None, keep_best=True,
               log=None, autotune=True):
    """Train `mlp` (binding.Mlp) for `epochs` epochs.

    train_u8: uint8 device tensor [n, 784]; train_labels: int32 device tensor [n];
    params: binding.DeformParams (default: the paper's values); beta_by_label: the bound of the
    rotation / shear angle follows the label (dbsn_deform_batch_labels): the look-alike digits 1
    and 7 get params.beta_deg, all others twice that (7.5 and 15 degrees with the default),
    instead of params.beta_deg for all;
    val_u8 / val_labels: validation set (default: the un-deformed training set).
    autotune: tune the training kernel's pauses once before the first epoch (dbsn_mlp_autotune on the
    first deformed chunk; steps with eta = 0, so the weights and every result stay as they are).
    Returns the history: one dict per epoch with eta, mean training loss, validation errors.
    With keep_best the network ends with the weights of the epoch of lowest validation error.
    """
    import torch
    n = train_u8.shape[0]
    assert train_u8.dtype == torch.uint8 and train_u8.shape[1] == 784
    assert train_labels.dtype == torch.int32 and train_labels.numel() == n
    params = params or binding.default_deform_params()
    if val_u8 is None:
        val_u8, val_labels = train_u8, train_labels
    if beta_by_label:
        # the struct carries the bound of the other classes, the call the one of the look-alikes
        wide = binding.DeformParams(params.sigma, params.alpha, 2.0 * params.beta_deg, params.gamma_pct, params.ktaps,
                                    params.shear, params.kernel)
        similar = params.beta_deg

    def deform(a, m, first_index, out, stream=None):
        if beta_by_label:
            binding.deform_batch(train_u8[a:a + m], seed, first_index, wide, out=out[:m], stream=stream,
                                 labels=train_labels[a:a + m], beta_similar_deg=similar)
        else:
            binding.deform_batch(train_u8[a:a + m], seed, first_index, params, out=out[:m], stream=stream)

    dev = train_u8.device
    main = torch.cuda.current_stream(dev)
    assert main.cuda_stream == mlp.stream, "run_epochs must run on the stream the network was created on"
    val_x = binding.deform_batch(val_u8, 0, 0, identity_params())
    # two input buffers: while the network trains on one chunk, the next one is deformed on a side
    # stream (default priority); `ready` says a buffer holds its chunk, `spent` that training is done with it
    xbuf = [torch.empty((chunk, 784), dtype=torch.float32, device=dev) for _ in range(2)]
    side = torch.cuda.Stream(dev)
    ready = [torch.cuda.Event() for _ in range(2)]
    spent = [torch.cuda.Event() for _ in range(2)]
    loss = torch.zeros(n, dtype=torch.float32, device=dev)
    history, best, best_params = [], None, None
    if autotune and min(chunk, n) >= 64:
        m0 = min(chunk, n)
        deform(0, m0, 0, xbuf[0])
        mlp.autotune(xbuf[0][:m0], train_labels[:m0])
    etas = eta_schedule(epochs, eta_start, eta_end)
    work = [(e, a, min(chunk, n - a)) for e in range(len(etas)) for a in range(0, n, chunk)]

    def start_deform(k):
        e, a, m = work[k]
        side.wait_event(spent[k % 2])       # (an event never recorded yet holds nobody up)
        deform(a, m, e * n + a, xbuf[k % 2], stream=side.cuda_stream)
        ready[k % 2].record(side)

    side.wait_stream(main)                  # the buffers exist and the tuning run is over
    if work:
        start_deform(0)
    for k, (e, a, m) in enumerate(work):
        if k + 1 < len(work):
            start_deform(k + 1)
        main.wait_event(ready[k % 2])
        mlp.bp_steps(xbuf[k % 2][:m], train_labels[a:a + m], float(etas[e]), loss[a:a + m])
        spent[k % 2].record(main)
        if a + m < n:
            continue
        # the epoch is complete: validate on the un-deformed set
        mlp.status()
        pred = mlp.classify(val_x)
        errors = binding.count_errors(pred, val_labels)
        rec = {"epoch": e, "eta": float(etas[e]), "train_loss": binding.mean_loss(loss), "val_errors": errors,
               "val_n": int(val_labels.numel())}
        history.append(rec)
        if log:
            log(rec)
        if keep_best and (best is None or errors < best):
            best, best_params = errors, mlp.get_params()
    main.wait_stream(side)
    if keep_best and best_params is not None and history[-1]["val_errors"] != best:
        mlp.set_params(best_params)
    return history
