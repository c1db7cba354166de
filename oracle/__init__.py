"""CPU oracle for the on-line back-propagation / deformation path.

TEST INFRASTRUCTURE ONLY: imported by the test-suite, by the smoke check and by
the CPU-baseline leg of the benchmark.  The GPU package never imports it, and
it never imports the GPU package.

`build()` compiles `dbsn_oracle.cpp` with g++ into `libdbsn_oracle.so` next to
the source; `Oracle` wraps the exported C functions with numpy arrays.
"""
from .binding import Oracle, build, load, pack_params, unpack_params  # noqa: F401
