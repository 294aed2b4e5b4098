"""MI355X-native hot path of sample-based GNN training with hot-embedding reuse (NeutronOrch).

The product is the HIP library `libneutronorch.so` (C ABI in include/neutronorch.h);
`binding` marshals arguments for it and nothing else.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
