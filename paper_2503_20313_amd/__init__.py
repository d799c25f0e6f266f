"""MI355X-native tile-centric overlapped tensor-parallel operators (AllGather+GEMM,
GEMM+ReduceScatter, ...).  The compute path is the HIP library in csrc/; this package only
marshals arguments to its C ABI (see include/tilelink_mi355.h)."""
from .binding import *  # noqa: F401,F403
