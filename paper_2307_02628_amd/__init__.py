"""SkipDecode decode path for AMD MI355X: HIP kernels behind a C ABI (include/skd.h)
plus this thin ctypes binding.  `from paper_2307_02628_amd import skd`."""
from . import skd  # noqa: F401
