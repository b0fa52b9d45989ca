"""MI355X (gfx950) row-wise sparse x sparse products behind a C ABI.

`workloads` (numpy-only generators) imports without the built library; everything in
`binding` needs libspgemm_gfx950.so and raises if it is missing.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    if name in ("binding", "Handle", "DeviceCSR", "to_device", "spgemm", "spgemm_symbolic", "spgemm_numeric", "SpgemmError"):
        import importlib
        b = importlib.import_module(".binding", __name__)
        return b if name == "binding" else getattr(b, name)
    raise AttributeError(name)
