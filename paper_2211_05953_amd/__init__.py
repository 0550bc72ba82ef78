"""MI355X-native hot path of Breadth-First Pipeline Parallelism (arXiv 2211.05953): one
pipeline rank's training step in breadth-first or depth-first order, in hand-written HIP
behind the C ABI of include/bf.h.  This package is the thin Python binding."""
from .binding import *  # noqa: F401,F403
from .binding import load, Stack, make_config, BfError  # noqa: F401
