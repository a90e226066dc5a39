"""MI355X-native GPU data path of the Fault Tolerant All Reduce (FTAR).

`binding` is the thin ctypes layer over the C-ABI library built from `csrc/`
(argument marshalling only); `workloads` holds the seeded synthetic input
generators that tests and the benchmark share.  Importing the package does not
load the HIP library; the first call into `binding` does, and fails loudly if
the library has not been built.
"""

__all__ = ["binding", "workloads"]
