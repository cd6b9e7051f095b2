"""DeepSqueeze compress-and-gossip step (arXiv:1907.07346, Algorithm 1) on MI355X.

`binding` is the ctypes front end of libdsq.so (HIP kernels behind a C ABI);
`workloads` makes the seeded synthetic inputs; `build` compiles the library.
"""
from . import workloads  # noqa: F401
