"""MI355X-native brute-force Euclidean-distance epsilon self-join (hot path of arXiv 2508.21230).

The work is done by hand-written HIP kernels behind the C ABI declared in include/ejoin.h;
`binding.EJoin` marshals torch device tensors to it.
"""
from .binding import EJoin, EJoinError, EJoinSet, load_library, tiles_evaluated, tiles_evaluated2  # noqa: F401
