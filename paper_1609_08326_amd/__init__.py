"""MI355X-native DC-ASGD parameter-server update (gfx950 HIP kernels behind a C ABI).

``workloads`` describes the seeded synthetic inputs; ``binding`` is the thin
ctypes layer over ``libdcasgd.so`` (argument marshalling only).  Importing the
package loads nothing heavy; the library is opened on first use.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads"]
