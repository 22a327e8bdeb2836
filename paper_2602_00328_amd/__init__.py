"""MI355X-native tiered cache fetch (Harvest, arxiv 2602.00328): HIP kernels behind a C ABI, plus a thin binding.

``paper_2602_00328_amd.binding`` loads ``libharvest.so`` (built in-tree by ``_build.build_library`` / the repository's
``__graft_entry__.build``) and exposes the entry points of ``include/harvest.h`` under the same names.
"""
from . import _build  # noqa: F401

__all__ = ["_build"]
