"""MI355X-native hot path of Cephalo's training method (arXiv 2411.01075): one GPU's share of a
sharded data-parallel transformer step.  The work is done by libcephalo.so (hand-written HIP
for gfx950, C ABI in include/cephalo.h); this package only marshals arguments to it."""
from .binding import *  # noqa: F401,F403
