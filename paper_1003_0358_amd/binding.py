"""ctypes binding of libdbsn (include/dbsn.h): argument marshalling only.

Every function of the C ABI appears here under its own name, as a method of `Lib`; device buffers
are torch tensors (PyTorch serves as the device allocator and stream provider, nothing else).
`Mlp` is a small convenience owner for the arena tensor and the handle.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdbsn.so")

OK, E_ARG, E_SHAPE, E_HIP, E_TIMEOUT = 0, -1, -2, -3, -4
MODE_LAUNCHES, MODE_PERSISTENT = 0, 1
LAUNCH_COOPERATIVE, LAUNCH_PLAIN = 0, 1

SYMBOLS = [
    "dbsn_mlp_arena_bytes", "dbsn_mlp_init", "dbsn_mlp_free", "dbsn_mlp_set_weights", "dbsn_mlp_get_weights",
    "dbsn_mlp_get_activations", "dbsn_mlp_get_deltas", "dbsn_mlp_set_mode", "dbsn_mlp_set_launch", "dbsn_mlp_set_spin_limit",
    "dbsn_mlp_set_pauses", "dbsn_mlp_get_pauses", "dbsn_mlp_set_variant", "dbsn_mlp_get_variant",
    "dbsn_mlp_status", "dbsn_mlp_autotune", "dbsn_deform_batch", "dbsn_deform_batch_beta", "dbsn_deform_batch_labels",
    "dbsn_bp_steps", "dbsn_bp_step", "dbsn_forward", "dbsn_classify", "dbsn_classify_static", "dbsn_count_errors", "dbsn_mean_loss", "dbsn_probe_stream", "dbsn_probe_handover",
    "dbsn_last_error",
]
DEFORM_KERNEL_AUTO, DEFORM_KERNEL_GENERAL = 0, 1


class DeformParams(C.Structure):
    _fields_ = [("sigma", C.c_float), ("alpha", C.c_float), ("beta_deg", C.c_float), ("gamma_pct", C.c_float),
                ("ktaps", C.c_int32), ("shear", C.c_int32), ("kernel", C.c_int32)]


class DbsnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libdbsn error %d: %s" % (code, msg))
        self.code = code


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / None."""
    if t is None:
        return C.c_void_p(0)
    if isinstance(t, np.ndarray):
        return C.c_void_p(t.ctypes.data)
    return C.c_void_p(t.data_ptr())


class Lib:
    def __init__(self, path=LIB_PATH):
        if not os.path.exists(path):
            raise RuntimeError("libdbsn.so is not built (%s): run `python -m paper_1003_0358_amd.build` or "
                               "__graft_entry__.build()" % path)
        # PyTorch ships its own HIP runtime; it has to be in the process before libdbsn.so is
        # loaded so that both resolve to that one runtime (two runtimes cannot share a device).
        import torch  # noqa: F401
        self.c = C.CDLL(path)
        c = self.c
        vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
        c.dbsn_mlp_arena_bytes.restype = C.c_size_t
        c.dbsn_mlp_arena_bytes.argtypes = [vp, i32]
        c.dbsn_mlp_init.argtypes = [C.POINTER(vp), vp, i32, u64, vp, C.c_size_t, vp]
        c.dbsn_mlp_free.argtypes = [vp]
        c.dbsn_mlp_set_weights.argtypes = [vp, i32, vp, vp]
        c.dbsn_mlp_get_weights.argtypes = [vp, i32, vp, vp]
        c.dbsn_mlp_get_activations.argtypes = [vp, i32, vp]
        c.dbsn_mlp_get_deltas.argtypes = [vp, i32, vp]
        c.dbsn_mlp_set_mode.argtypes = [vp, i32]
        c.dbsn_mlp_set_launch.argtypes = [vp, i32]
        c.dbsn_mlp_set_spin_limit.argtypes = [vp, C.c_uint32]
        c.dbsn_mlp_set_pauses.argtypes = [vp, vp, vp]
        c.dbsn_mlp_get_pauses.argtypes = [vp, vp, vp]
        c.dbsn_mlp_set_variant.argtypes = [vp, i32, i32, i32]
        c.dbsn_mlp_get_variant.argtypes = [vp, vp, vp, vp]
        c.dbsn_mlp_status.argtypes = [vp]
        c.dbsn_mlp_autotune.argtypes = [vp, vp, vp, i64]
        c.dbsn_deform_batch.argtypes = [C.POINTER(DeformParams), vp, i64, u64, u64, vp, vp]
        c.dbsn_deform_batch_beta.argtypes = [C.POINTER(DeformParams), vp, vp, i64, u64, u64, vp, vp]
        c.dbsn_deform_batch_labels.argtypes = [C.POINTER(DeformParams), vp, vp, u64, f32, i64, u64, u64, vp, vp]
        c.dbsn_count_errors.argtypes = [vp, vp, i64, vp, vp]
        c.dbsn_mean_loss.argtypes = [vp, i64, vp, vp]
        c.dbsn_probe_stream.argtypes = [vp, i64, i32, i32, vp, vp]
        c.dbsn_probe_handover.argtypes = [i32, i32, vp, vp, vp]
        c.dbsn_bp_steps.argtypes = [vp, vp, vp, i64, f32, vp]
        c.dbsn_bp_step.argtypes = [vp, vp, i32, f32]
        c.dbsn_forward.argtypes = [vp, vp, vp]
        c.dbsn_classify.argtypes = [vp, vp, i64, vp]
        c.dbsn_classify_static.argtypes = [vp, vp, i64, vp]
        c.dbsn_last_error.restype = C.c_char_p
        for name in SYMBOLS:
            if name not in ("dbsn_mlp_arena_bytes", "dbsn_last_error"):
                getattr(c, name).restype = i32

    # -- raw calls: return the C return code ------------------------------------------------
    def last_error(self):
        return self.c.dbsn_last_error().decode()

    def check(self, rc):
        if rc != OK:
            raise DbsnError(rc, self.last_error())

    def mlp_arena_bytes(self, sizes):
        s = np.ascontiguousarray(sizes, dtype=np.int32)
        return int(self.c.dbsn_mlp_arena_bytes(s.ctypes.data, len(s)))

    def mlp_init(self, sizes, seed, arena, stream=0):
        """-> (rc, handle)"""
        s = np.ascontiguousarray(sizes, dtype=np.int32)
        h = C.c_void_p(0)
        nbytes = 0 if arena is None else arena.numel() * arena.element_size()
        rc = self.c.dbsn_mlp_init(C.byref(h), s.ctypes.data, len(s), seed, _ptr(arena), nbytes, C.c_void_p(stream))
        return rc, h

    def mlp_free(self, h):
        return self.c.dbsn_mlp_free(h)

    def mlp_set_weights(self, h, layer, W_host, b_host):
        return self.c.dbsn_mlp_set_weights(h, layer, _ptr(W_host), _ptr(b_host))

    def mlp_get_weights(self, h, layer, W_host, b_host):
        return self.c.dbsn_mlp_get_weights(h, layer, _ptr(W_host), _ptr(b_host))

    def mlp_get_activations(self, h, layer, x_host):
        return self.c.dbsn_mlp_get_activations(h, layer, _ptr(x_host))

    def mlp_get_deltas(self, h, layer, d_host):
        return self.c.dbsn_mlp_get_deltas(h, layer, _ptr(d_host))

    def mlp_set_mode(self, h, mode):
        return self.c.dbsn_mlp_set_mode(h, mode)

    def mlp_set_launch(self, h, kind):
        return self.c.dbsn_mlp_set_launch(h, kind)

    def mlp_set_spin_limit(self, h, polls):
        return self.c.dbsn_mlp_set_spin_limit(h, polls)

    def mlp_status(self, h):
        return self.c.dbsn_mlp_status(h)

    def mlp_set_pauses(self, h, fwd_host, bwd_host):
        return self.c.dbsn_mlp_set_pauses(h, _ptr(fwd_host), _ptr(bwd_host))

    def mlp_get_pauses(self, h, fwd_host, bwd_host):
        return self.c.dbsn_mlp_get_pauses(h, _ptr(fwd_host), _ptr(bwd_host))

    def mlp_set_variant(self, h, stationary, fixed_layout, banded):
        return self.c.dbsn_mlp_set_variant(h, stationary, fixed_layout, banded)

    def mlp_get_variant(self, h, stationary, layout, banded_pairs):
        return self.c.dbsn_mlp_get_variant(h, _ptr(stationary), _ptr(layout), _ptr(banded_pairs))

    def mlp_autotune(self, h, samples, labels, n):
        return self.c.dbsn_mlp_autotune(h, _ptr(samples), _ptr(labels), n)

    def deform_batch(self, params, src, n, seed, first_index, dst, stream=0):
        return self.c.dbsn_deform_batch(C.byref(params) if params is not None else None, _ptr(src), n, seed,
                                        first_index, _ptr(dst), C.c_void_p(stream))

    def deform_batch_beta(self, params, src, beta_deg, n, seed, first_index, dst, stream=0):
        return self.c.dbsn_deform_batch_beta(C.byref(params) if params is not None else None, _ptr(src),
                                             _ptr(beta_deg), n, seed, first_index, _ptr(dst), C.c_void_p(stream))

    def deform_batch_labels(self, params, src, labels, similar_mask, beta_similar_deg, n, seed, first_index, dst,
                            stream=0):
        return self.c.dbsn_deform_batch_labels(C.byref(params) if params is not None else None, _ptr(src),
                                               _ptr(labels), similar_mask, beta_similar_deg, n, seed, first_index,
                                               _ptr(dst), C.c_void_p(stream))

    def count_errors(self, predicted, labels, n, count, stream=0):
        return self.c.dbsn_count_errors(_ptr(predicted), _ptr(labels), n, _ptr(count), C.c_void_p(stream))

    def mean_loss(self, loss, n, mean, stream=0):
        return self.c.dbsn_mean_loss(_ptr(loss), n, _ptr(mean), C.c_void_p(stream))

    def probe_stream(self, buf, n_floats, workgroups, sweeps, sink, stream=0):
        return self.c.dbsn_probe_stream(_ptr(buf), n_floats, workgroups, sweeps, _ptr(sink), C.c_void_p(stream))

    def probe_handover(self, within_die, rounds, buf, gave_up, stream=0):
        return self.c.dbsn_probe_handover(int(within_die), rounds, _ptr(buf), _ptr(gave_up), C.c_void_p(stream))

    def bp_steps(self, h, samples, labels, n, eta, loss=None):
        return self.c.dbsn_bp_steps(h, _ptr(samples), _ptr(labels), n, eta, _ptr(loss))

    def bp_step(self, h, sample, label, eta):
        return self.c.dbsn_bp_step(h, _ptr(sample), label, eta)

    def forward(self, h, sample, probs):
        return self.c.dbsn_forward(h, _ptr(sample), _ptr(probs))

    def classify(self, h, samples, n, labels_out):
        return self.c.dbsn_classify(h, _ptr(samples), n, _ptr(labels_out))

    def classify_static(self, h, samples, n, labels_out):
        return self.c.dbsn_classify_static(h, _ptr(samples), n, _ptr(labels_out))


_lib = None


def load():
    """The process-wide Lib; raises if libdbsn.so has not been built."""
    global _lib
    if _lib is None:
        _lib = Lib()
    return _lib


def default_deform_params():
    """sigma 6, alpha 36, rotation +-7.5 degrees, scaling +-15 %, 21 taps (values the paper reports using)."""
    return DeformParams(6.0, 36.0, 7.5, 15.0, 21, 0, 0)


PAPER_SIMILAR_MASK = (1 << 1) | (1 << 7)   # the look-alike digits 1 and 7 (section "Deforming images ...")


class Mlp:
    """Owns the arena tensor and the handle of one network; methods raise DbsnError on failure."""

    def __init__(self, sizes, seed=0, device="cuda:0", mode=MODE_PERSISTENT):
        import torch
        self.lib = load()
        self.sizes = [int(s) for s in sizes]
        nbytes = self.lib.mlp_arena_bytes(self.sizes)
        if nbytes == 0:
            raise DbsnError(E_SHAPE, "unsupported layer sizes %r" % (self.sizes,))
        self.torch = torch
        self.device = torch.device(device)
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device).cuda_stream
        rc, self.h = self.lib.mlp_init(self.sizes, seed, self.arena, self.stream)
        self.lib.check(rc)
        self.lib.check(self.lib.mlp_set_mode(self.h, mode))

    def close(self):
        if getattr(self, "h", None) is not None and self.h:
            self.lib.mlp_free(self.h)
            self.h = None

    __del__ = close

    @property
    def L(self):
        return len(self.sizes) - 1

    def set_mode(self, mode):
        self.lib.check(self.lib.mlp_set_mode(self.h, mode))

    def set_launch(self, kind):
        self.lib.check(self.lib.mlp_set_launch(self.h, kind))

    def status(self):
        self.lib.check(self.lib.mlp_status(self.h))

    def set_variant(self, stationary=True, fixed_layout=True, banded=True):
        self.lib.check(self.lib.mlp_set_variant(self.h, int(stationary), int(fixed_layout), int(banded)))

    def get_variant(self):
        """-> (stationary, layout, banded_pairs) in force"""
        v = [np.zeros(1, np.int32) for _ in range(3)]
        self.lib.check(self.lib.mlp_get_variant(self.h, v[0], v[1], v[2]))
        return int(v[0][0]), int(v[1][0]), int(v[2][0])

    def get_pauses(self):
        f = np.zeros(self.L, np.int32)
        b = np.zeros(self.L, np.int32)
        self.lib.check(self.lib.mlp_get_pauses(self.h, f, b))
        return f, b

    def set_pauses(self, fwd=None, bwd=None):
        f = None if fwd is None else np.ascontiguousarray(fwd, dtype=np.int32)
        b = None if bwd is None else np.ascontiguousarray(bwd, dtype=np.int32)
        assert (f is None or f.size == self.L) and (b is None or b.size == self.L)
        self.lib.check(self.lib.mlp_set_pauses(self.h, f, b))

    def autotune(self, samples, labels):
        """Tunes the persistent kernel's pauses on these samples (steps with eta = 0: weights unchanged)."""
        self.lib.check(self.lib.mlp_autotune(self.h, samples, labels, samples.shape[0]))

    def get_weights(self, layer):
        W = np.empty((self.sizes[layer], self.sizes[layer - 1]), dtype=np.float32)
        b = np.empty(self.sizes[layer], dtype=np.float32)
        self.lib.check(self.lib.mlp_get_weights(self.h, layer, W, b))
        return W, b

    def set_weights(self, layer, W, b):
        W = None if W is None else np.ascontiguousarray(W, dtype=np.float32)
        b = None if b is None else np.ascontiguousarray(b, dtype=np.float32)
        self.lib.check(self.lib.mlp_set_weights(self.h, layer, W, b))

    def get_params(self):
        """All layers, packed [W_1, b_1, W_2, b_2, ...] dense row-major."""
        parts = []
        for l in range(1, self.L + 1):
            W, b = self.get_weights(l)
            parts += [W.ravel(), b]
        return np.concatenate(parts)

    def set_params(self, params):
        o = 0
        for l in range(1, self.L + 1):
            nin, nout = self.sizes[l - 1], self.sizes[l]
            W = params[o:o + nin * nout].reshape(nout, nin); o += nin * nout
            b = params[o:o + nout]; o += nout
            self.set_weights(l, W, b)

    def get_activations(self, layer):
        x = np.empty(self.sizes[layer], dtype=np.float32)
        self.lib.check(self.lib.mlp_get_activations(self.h, layer, x))
        return x

    def get_deltas(self, layer):
        d = np.empty(self.sizes[layer], dtype=np.float32)
        self.lib.check(self.lib.mlp_get_deltas(self.h, layer, d))
        return d

    def bp_steps(self, samples, labels, eta, loss=None):
        n = samples.shape[0]
        self.lib.check(self.lib.bp_steps(self.h, samples, labels, n, float(eta), loss))

    def bp_step(self, sample, label, eta):
        self.lib.check(self.lib.bp_step(self.h, sample, int(label), float(eta)))

    def forward(self, sample):
        probs = self.torch.empty(self.sizes[-1], dtype=self.torch.float32, device=self.device)
        self.lib.check(self.lib.forward(self.h, sample, probs))
        return probs

    def classify(self, samples):
        n = samples.shape[0]
        out = self.torch.empty(n, dtype=self.torch.int32, device=self.device)
        self.lib.check(self.lib.classify(self.h, samples, n, out))
        return out


def deform_batch(src_u8, seed, first_index, params=None, out=None, stream=None, beta_deg=None, labels=None,
                 similar_mask=PAPER_SIMILAR_MASK, beta_similar_deg=None):
    """src_u8: uint8 device tensor [n, 784] -> float32 device tensor [n, 784].  beta_deg: optional
    float32 device tensor [n], one bound of the angle per image instead of params.beta_deg.
    labels: optional int32 device tensor [n]: images of the classes in similar_mask take
    beta_similar_deg (default: half of params.beta_deg), all others params.beta_deg."""
    import torch
    lib = load()
    n = src_u8.shape[0]
    if out is None:
        out = torch.empty((n, 784), dtype=torch.float32, device=src_u8.device)
    if stream is None:
        stream = torch.cuda.current_stream(src_u8.device).cuda_stream
    params = params or default_deform_params()
    if beta_deg is not None:
        assert beta_deg.dtype == torch.float32 and beta_deg.numel() == n and beta_deg.is_contiguous()
        lib.check(lib.deform_batch_beta(params, src_u8, beta_deg, n, seed, first_index, out, stream))
    elif labels is not None:
        assert labels.dtype == torch.int32 and labels.numel() == n and labels.is_contiguous()
        bs = 0.5 * params.beta_deg if beta_similar_deg is None else beta_similar_deg
        lib.check(lib.deform_batch_labels(params, src_u8, labels, similar_mask, bs, n, seed, first_index, out, stream))
    else:
        lib.check(lib.deform_batch(params, src_u8, n, seed, first_index, out, stream))
    return out


def count_errors(predicted, labels):
    """Number of positions where two int32 device tensors differ (one small kernel + one read-back)."""
    import torch
    lib = load()
    n = predicted.numel()
    assert labels.numel() == n and predicted.dtype == torch.int32 and labels.dtype == torch.int32
    out = torch.empty(1, dtype=torch.int64, device=predicted.device)
    lib.check(lib.count_errors(predicted, labels, n, out, torch.cuda.current_stream(predicted.device).cuda_stream))
    return int(out.item())


def mean_loss(loss):
    """Mean of a float32 device tensor of per-step losses (one small kernel + one read-back)."""
    import torch
    lib = load()
    out = torch.empty(1, dtype=torch.float32, device=loss.device)
    lib.check(lib.mean_loss(loss, loss.numel(), out, torch.cuda.current_stream(loss.device).cuda_stream))
    return float(out.item())
