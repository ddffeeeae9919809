"""MI355X-native (gfx950) implementation of the DistGrid training hot path (arXiv 2405.04416).

`binding` exposes the C entry points of libdistgrid.so one to one; `step` sequences them into a
forward + backward pass.  Importing the package does not load the library; the first call does,
and raises if it has not been built.
"""
from . import binding  # noqa: F401
