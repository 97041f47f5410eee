"""MI355X-native hot path of one Talon speculative-decoding step (arXiv 2601.07353):
budget-driven adaptive draft-tree expansion and tree-attention verification, as
hand-written HIP kernels behind the C ABI of include/talon.h.  This package holds the
kernels (csrc/), their build script and the ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import (Candidates, TalonError, TreeState, load_library, make_expand_workspace,
                      make_literal_workspace, make_verify_workspace)  # noqa: F401
