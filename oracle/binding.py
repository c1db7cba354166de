"""ctypes wrapper around the CPU oracle (test infrastructure, see dbsn_oracle.cpp)."""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dbsn_oracle.cpp")
_LIB = os.path.join(_HERE, "libdbsn_oracle.so")


def build(force=True):
    """Compile the oracle with g++ (-O2, no fast-math, no FMA contraction)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["g++", "-O2", "-std=c++14", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", _SRC, "-o", _LIB]
    subprocess.run(cmd, check=True)
    return _LIB


def load():
    if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        build()
    return C.CDLL(_LIB)


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def pack_params(Ws, bs, dtype):
    """[W_1 (n_1 x n_0) row-major, b_1, W_2, b_2, ...] -> one flat vector."""
    parts = []
    for W, b in zip(Ws, bs):
        parts.append(np.asarray(W, dtype=dtype).ravel())
        parts.append(np.asarray(b, dtype=dtype).ravel())
    return np.ascontiguousarray(np.concatenate(parts))


def unpack_params(sizes, params):
    Ws, bs, o = [], [], 0
    for l in range(1, len(sizes)):
        nin, nout = sizes[l - 1], sizes[l]
        Ws.append(params[o:o + nin * nout].reshape(nout, nin)); o += nin * nout
        bs.append(params[o:o + nout]); o += nout
    return Ws, bs


class Oracle:
    """Thin numpy front-end; `mode` is 'f32' or 'f64' for every real-valued routine."""

    def __init__(self):
        self.lib = load()
        L = self.lib
        L.dbsn_oracle_param_count.restype = C.c_int64
        L.dbsn_oracle_bp_step_f32.restype = C.c_float
        L.dbsn_oracle_bp_step_f64.restype = C.c_double
        L.dbsn_oracle_act_f32.restype = C.c_float
        L.dbsn_oracle_act_f64.restype = C.c_double
        L.dbsn_oracle_dact_from_y_f32.restype = C.c_float
        L.dbsn_oracle_dact_from_y_f64.restype = C.c_double
        L.dbsn_oracle_act_f32.argtypes = [C.c_float]
        L.dbsn_oracle_act_f64.argtypes = [C.c_double]
        L.dbsn_oracle_dact_from_y_f32.argtypes = [C.c_float]
        L.dbsn_oracle_dact_from_y_f64.argtypes = [C.c_double]
        L.dbsn_oracle_get_threads.restype = C.c_int32
        L.dbsn_oracle_max_threads.restype = C.c_int32

    # ---- helpers -------------------------------------------------------
    @staticmethod
    def _t(mode):
        return (np.float32, C.c_float) if mode == "f32" else (np.float64, C.c_double)

    @staticmethod
    def _sizes(sizes):
        s = np.ascontiguousarray(np.asarray(sizes, dtype=np.int32))
        return s, _p(s, C.c_int32), C.c_int32(len(s))

    def set_threads(self, n):
        self.lib.dbsn_oracle_set_threads(C.c_int32(int(n)))
        return int(self.lib.dbsn_oracle_get_threads())

    def max_threads(self):
        return int(self.lib.dbsn_oracle_max_threads())

    def param_count(self, sizes):
        s, sp, ns = self._sizes(sizes)
        return int(self.lib.dbsn_oracle_param_count(sp, ns))

    # ---- random numbers ------------------------------------------------
    def rng_raw(self, seed, stream, first_counter, n):
        out = np.empty(n, dtype=np.uint64)
        self.lib.dbsn_oracle_rng_raw(C.c_uint64(seed), C.c_uint64(stream), C.c_uint64(first_counter),
                                     C.c_int64(n), _p(out, C.c_uint64))
        return out

    def rng_sym(self, seed, stream, first_counter, n):
        out = np.empty(n, dtype=np.float32)
        self.lib.dbsn_oracle_rng_sym(C.c_uint64(seed), C.c_uint64(stream), C.c_uint64(first_counter),
                                     C.c_int64(n), _p(out, C.c_float))
        return out

    # ---- MLP -----------------------------------------------------------
    def init_params(self, sizes, seed):
        s, sp, ns = self._sizes(sizes)
        out = np.empty(self.param_count(sizes), dtype=np.float32)
        self.lib.dbsn_oracle_init_params_f32(sp, ns, C.c_uint64(seed), _p(out, C.c_float))
        return out

    def forward(self, sizes, params, x0, mode="f64"):
        """-> (acts: x_1..x_{L-1} then logits, probs)"""
        dt, ct = self._t(mode)
        s, sp, ns = self._sizes(sizes)
        params = np.ascontiguousarray(params, dtype=dt)
        x0 = np.ascontiguousarray(x0, dtype=dt)
        assert params.size == self.param_count(sizes) and x0.size == sizes[0]
        acts = np.empty(int(sum(sizes[1:])), dtype=dt)
        probs = np.empty(sizes[-1], dtype=dt)
        getattr(self.lib, "dbsn_oracle_forward_" + mode)(sp, ns, _p(params, ct), _p(x0, ct), _p(acts, ct),
                                                         _p(probs, ct))
        return acts, probs

    def loss(self, sizes, params, x0, label, mode="f64"):
        _, probs = self.forward(sizes, params, x0, mode)
        return -np.log(probs[label])

    def bp_step(self, sizes, params, x0, label, eta, mode="f64", want_deltas=False):
        """In-place on a copy: -> (new_params, loss[, deltas])"""
        dt, ct = self._t(mode)
        s, sp, ns = self._sizes(sizes)
        p = np.array(params, dtype=dt, copy=True, order="C")
        x0 = np.ascontiguousarray(x0, dtype=dt)
        assert p.size == self.param_count(sizes) and x0.size == sizes[0]
        assert 0 <= int(label) < sizes[-1]
        deltas = np.empty(int(sum(sizes[1:])), dtype=dt) if want_deltas else None
        dptr = _p(deltas, ct) if want_deltas else None
        loss = getattr(self.lib, "dbsn_oracle_bp_step_" + mode)(sp, ns, _p(p, ct), _p(x0, ct),
                                                                C.c_int32(int(label)), ct(eta), dptr)
        return (p, loss, deltas) if want_deltas else (p, loss)

    def bp_steps(self, sizes, params, samples, labels, eta, mode="f64"):
        dt, ct = self._t(mode)
        s, sp, ns = self._sizes(sizes)
        p = np.array(params, dtype=dt, copy=True, order="C")
        samples = np.ascontiguousarray(samples, dtype=dt).reshape(-1, sizes[0])
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        n = samples.shape[0]
        assert labels.size == n and p.size == self.param_count(sizes)
        assert n == 0 or (labels.min() >= 0 and labels.max() < sizes[-1])
        loss = np.empty(n, dtype=dt)
        getattr(self.lib, "dbsn_oracle_bp_steps_" + mode)(sp, ns, _p(p, ct), _p(samples, ct),
                                                          _p(labels, C.c_int32), C.c_int64(n), ct(eta),
                                                          _p(loss, ct))
        return p, loss

    def classify(self, sizes, params, samples, mode="f64"):
        dt, ct = self._t(mode)
        s, sp, ns = self._sizes(sizes)
        params = np.ascontiguousarray(params, dtype=dt)
        samples = np.ascontiguousarray(samples, dtype=dt).reshape(-1, sizes[0])
        out = np.empty(samples.shape[0], dtype=np.int32)
        getattr(self.lib, "dbsn_oracle_classify_" + mode)(sp, ns, _p(params, ct), _p(samples, ct),
                                                          C.c_int64(samples.shape[0]), _p(out, C.c_int32))
        return out

    def logits_batch(self, sizes, params, samples, mode="f64"):
        """Output-layer pre-activations of every sample: [n, classes]."""
        dt, ct = self._t(mode)
        s, sp, ns = self._sizes(sizes)
        params = np.ascontiguousarray(params, dtype=dt)
        samples = np.ascontiguousarray(samples, dtype=dt).reshape(-1, sizes[0])
        assert params.size == self.param_count(sizes)
        out = np.empty((samples.shape[0], sizes[-1]), dtype=dt)
        getattr(self.lib, "dbsn_oracle_logits_batch_" + mode)(sp, ns, _p(params, ct), _p(samples, ct),
                                                              C.c_int64(samples.shape[0]), _p(out, ct))
        return out

    def act(self, a, mode="f64"):
        return getattr(self.lib, "dbsn_oracle_act_" + mode)(a)

    def dact_from_y(self, y, mode="f64"):
        return getattr(self.lib, "dbsn_oracle_dact_from_y_" + mode)(y)

    # ---- deformation ---------------------------------------------------
    def gauss_taps(self, sigma, ktaps, mode="f64"):
        dt, ct = self._t(mode)
        out = np.empty(ktaps, dtype=dt)
        getattr(self.lib, "dbsn_oracle_gauss_taps_" + mode)(ct(sigma), C.c_int32(ktaps), _p(out, ct))
        return out

    def smooth_field(self, field, sigma, ktaps, alpha, mode="f64"):
        dt, ct = self._t(mode)
        f = np.ascontiguousarray(field, dtype=dt)
        H, W = f.shape
        out = np.empty((H, W), dtype=dt)
        getattr(self.lib, "dbsn_oracle_smooth_field_" + mode)(_p(f, ct), C.c_int32(H), C.c_int32(W), ct(sigma),
                                                              C.c_int32(ktaps), ct(alpha), _p(out, ct))
        return out

    def draw_image_randoms(self, seed, index, HW=784):
        s3 = np.empty(3, dtype=np.float32)
        Dx = np.empty(HW, dtype=np.float32)
        Dy = np.empty(HW, dtype=np.float32)
        self.lib.dbsn_oracle_draw_image_randoms(C.c_uint64(seed), C.c_uint64(index), C.c_int32(HW),
                                                _p(s3, C.c_float), _p(Dx, C.c_float), _p(Dy, C.c_float))
        return s3, Dx, Dy

    def affine_scalars(self, beta_deg, gamma_pct, s3, mode="f64"):
        """-> (cos, sin, sx, sy)"""
        dt, ct = self._t(mode)
        s3 = np.ascontiguousarray(s3, dtype=np.float32)
        out = np.empty(4, dtype=dt)
        getattr(self.lib, "dbsn_oracle_affine_scalars_" + mode)(C.c_float(beta_deg), C.c_float(gamma_pct),
                                                                _p(s3, C.c_float), _p(out, ct))
        return out

    def resample(self, img, cs, sn, sx, sy, dx, dy, mode="f64"):
        dt, ct = self._t(mode)
        img = np.ascontiguousarray(img, dtype=np.uint8)
        H, W = img.shape
        dx = np.ascontiguousarray(dx, dtype=dt).reshape(H, W)
        dy = np.ascontiguousarray(dy, dtype=dt).reshape(H, W)
        out = np.empty((H, W), dtype=dt)
        getattr(self.lib, "dbsn_oracle_resample_" + mode)(_p(img, C.c_uint8), C.c_int32(H), C.c_int32(W), ct(cs),
                                                          ct(sn), ct(sx), ct(sy), _p(dx, ct), _p(dy, ct),
                                                          _p(out, ct))
        return out

    def linear_part(self, shear, beta_deg, s3, mode="f64"):
        """-> (p, q, r, t): X' = p u + q v, Y' = r u + t v (rotation, or horizontal shear when `shear`)."""
        dt, ct = self._t(mode)
        s3 = np.ascontiguousarray(s3, dtype=np.float32)
        out = np.empty(4, dtype=dt)
        getattr(self.lib, "dbsn_oracle_linear_part_" + mode)(C.c_int32(int(shear)), C.c_float(beta_deg),
                                                             _p(s3, C.c_float), _p(out, ct))
        return out

    def resample_lin(self, img, pqrt, sx, sy, dx, dy, mode="f64"):
        dt, ct = self._t(mode)
        img = np.ascontiguousarray(img, dtype=np.uint8)
        H, W = img.shape
        pqrt = np.ascontiguousarray(pqrt, dtype=dt)
        dx = np.ascontiguousarray(dx, dtype=dt).reshape(H, W)
        dy = np.ascontiguousarray(dy, dtype=dt).reshape(H, W)
        out = np.empty((H, W), dtype=dt)
        getattr(self.lib, "dbsn_oracle_resample_lin_" + mode)(_p(img, C.c_uint8), C.c_int32(H), C.c_int32(W),
                                                              _p(pqrt, ct), ct(sx), ct(sy), _p(dx, ct), _p(dy, ct),
                                                              _p(out, ct))
        return out

    def deform_batch(self, src, seed, first_index, sigma=6.0, alpha=36.0, beta_deg=7.5, gamma_pct=15.0, ktaps=21,
                     mode="f64", shear=False, beta_each=None):
        """beta_each: one angle bound (degrees) per image instead of beta_deg; shear: horizontal
        shearing instead of rotation."""
        dt, ct = self._t(mode)
        src = np.ascontiguousarray(src, dtype=np.uint8).reshape(-1, 784)
        n = src.shape[0]
        out = np.empty((n, 784), dtype=dt)
        be = None
        if beta_each is not None:
            be = np.ascontiguousarray(beta_each, dtype=np.float32)
            assert be.shape == (n,)
        getattr(self.lib, "dbsn_oracle_deform_batch_" + mode)(
            C.c_float(sigma), C.c_float(alpha), C.c_float(beta_deg), C.c_float(gamma_pct), C.c_int32(ktaps),
            C.c_int32(int(bool(shear))), _p(be, C.c_float) if be is not None else None,
            _p(src, C.c_uint8), C.c_int64(n), C.c_uint64(seed), C.c_uint64(first_index), _p(out, ct))
        return out
