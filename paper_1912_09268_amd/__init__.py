"""MI355X-native merged-gradient hot path of MG-WFBP: thin ctypes binding over libmgwfbp.so.

Every step (plan, layout, pack, reduce, unpack + update) runs inside the C-ABI library; this package
only marshals arguments.  Importing it does not load the library; the first call does, and fails
loudly if the library has not been built (run `python -m paper_1912_09268_amd.build`)."""
from .binding import (  # noqa: F401
    AR_BINARY_TREE, AR_DOUBLE_BINARY_TREES, AR_HALVING_DOUBLING, AR_RECURSIVE_DOUBLING, AR_RING, allreduce_ab,
    fit_ab, group_ready_times, simulate,
    BF16, F16, F32, Context, MgwfbpError, eval_plan, lib, library_path, plan, plan_opt,
)
