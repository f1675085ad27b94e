"""MI355X-native CD-GraB pair-balancing path (arXiv 2302.00845).

The work is done by ``libcdgrab.so`` (hand-written HIP for gfx950 behind the C ABI
declared in ``include/cdgrab.h``).  This package is a thin ctypes binding with the
same entry-point names; PyTorch is used only for device memory and streams.
"""
from .cdgrab import (  # noqa: F401
    CdgrabError,
    Handle,
    cdgrab_balance_epoch,
    cdgrab_balance_epoch_independent,
    cdgrab_balance_epoch_randomized,
    cdgrab_balance_epoch_stale_mean,
    cdgrab_balance_epoch_static,
    cdgrab_herding_bound,
    cdgrab_pergrad,
    cdgrab_plan_epoch,
    cdgrab_reorder,
    cdgrab_train_epoch_softmax,
    cdgrab_train_softmax,
    library_path,
    load_library,
)
