"""Host-side checks of libdbsn that need no GPU: the library loads, exports every function the
header declares, sizes arenas sensibly and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    with open(os.path.join(ROOT, "include", "dbsn.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dbsn_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(dbsn):
    from paper_1003_0358_amd import binding
    names = _declared()
    assert len(names) >= 16
    for n in names:
        assert hasattr(dbsn.c, n), n
    assert sorted(binding.SYMBOLS) == names


def test_arena_bytes(dbsn):
    net4 = [784, 2500, 2000, 1500, 1000, 500, 10]
    nb = dbsn.mlp_arena_bytes(net4)
    nw = sum((net4[i] + 1) * net4[i + 1] for i in range(6))
    assert nw == 11972510
    # weights, a few MB of vectors and partial sums, and two activation buffers of 16384 samples x 2500
    # for the batched classification pass
    assert 4 * nw + 2 * 16384 * 2500 * 4 < nb < 4 * nw + 2 * 16384 * 2500 * 4 + 20 * 2 ** 20
    assert nb % 256 == 0
    assert dbsn.mlp_arena_bytes([784, 10]) > 4 * 7850
    # unsupported shapes
    assert dbsn.mlp_arena_bytes([784]) == 0
    assert dbsn.mlp_arena_bytes([784, 0, 10]) == 0
    assert dbsn.mlp_arena_bytes([784, 5000, 10]) == 0
    assert dbsn.mlp_arena_bytes([784, 100, 65]) == 0
    assert dbsn.mlp_arena_bytes([10] * 18) == 0
    assert dbsn.mlp_arena_bytes([10] * 17) > 0


def test_argument_errors_without_device(dbsn):
    from paper_1003_0358_amd import binding
    rc, h = dbsn.mlp_init([784, 10], 0, None)
    assert rc == binding.E_ARG and "arena" in dbsn.last_error()
    assert not h
    assert dbsn.bp_step(None, None, 0, 0.1) == binding.E_ARG
    assert dbsn.bp_steps(None, None, None, 1, 0.1) == binding.E_ARG
    assert dbsn.classify(None, None, 1, None) == binding.E_ARG
    assert dbsn.forward(None, None, None) == binding.E_ARG
    assert dbsn.mlp_status(None) == binding.E_ARG
    assert dbsn.mlp_get_weights(None, 1, None, None) == binding.E_ARG
    assert dbsn.mlp_free(None) == binding.OK
    p = binding.default_deform_params()
    assert dbsn.deform_batch(None, None, 1, 0, 0, None) == binding.E_ARG
    assert dbsn.deform_batch(p, None, -1, 0, 0, None) == binding.E_ARG
    assert dbsn.deform_batch(p, None, 0, 0, 0, None) == binding.OK          # empty batch: nothing to do
    assert dbsn.deform_batch(p, None, 1, 0, 0, None) == binding.E_ARG       # null buffers
    for bad in (0, 20, 65, -3):
        q = binding.DeformParams(6.0, 36.0, 7.5, 15.0, bad)
        assert dbsn.deform_batch(q, None, 1, 0, 0, None) == binding.E_ARG
    q = binding.DeformParams(float("nan"), 36.0, 7.5, 15.0, 21)
    assert dbsn.deform_batch(q, None, 1, 0, 0, None) == binding.E_ARG
    assert dbsn.last_error() != ""
    assert dbsn.deform_batch_labels(None, None, None, 0, 7.5, 1, 0, 0, None) == binding.E_ARG
    assert dbsn.deform_batch_labels(p, None, None, 0, 7.5, 0, 0, 0, None) == binding.OK      # empty
    assert dbsn.count_errors(None, None, -1, None) == binding.E_ARG
    assert dbsn.count_errors(None, None, 0, None) == binding.E_ARG          # nowhere to write the count
    assert dbsn.mean_loss(None, 0, None) == binding.E_ARG
    assert dbsn.mlp_set_pauses(None, None, None) == binding.E_ARG
    assert dbsn.mlp_get_pauses(None, None, None) == binding.E_ARG
    assert dbsn.mlp_set_variant(None, 1, 1, 1) == binding.E_ARG
    assert dbsn.mlp_get_variant(None, None, None, None) == binding.E_ARG


def test_missing_library_fails_loudly(tmp_path):
    from paper_1003_0358_amd import binding
    with pytest.raises(RuntimeError, match="not built"):
        binding.Lib(str(tmp_path / "libdbsn.so"))


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1003_0358_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                with open(os.path.join(dirpath, f)) as fh:
                    text = fh.read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
    with open(os.path.join(ROOT, "oracle", "dbsn_oracle.cpp")) as fh:
        assert "paper_1003_0358_amd" not in fh.read()
