"""MI355X-native arbitrary-precision (p-bit x q-bit) bit-plane GEMM / convolution.

The package holds two things only:
  * ``workloads``  seeded synthetic input generators and workload shapes
                   (pure numpy, none of the method's arithmetic);
  * ``binding``    the thin ctypes binding over the C-ABI library ``libapnn.so``
                   built from ``csrc/`` (argument marshalling only).

Nothing is imported eagerly so that ``workloads`` stays usable without the
compiled library (it feeds the CPU oracle tests as well).
"""

__all__ = ["workloads", "binding"]
