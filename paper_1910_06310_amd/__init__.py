"""MI355X-native marginalized graph kernel solver (HIP, gfx950).

The work happens in ``libmgk.so`` (see ``include/mgk.h``); this package is the
thin Python binding plus the in-tree build step.
"""
from .binding import (  # noqa: F401
    Batch, MgkError, Solver, load_library, EXPORTS,
    REORDER_NONE, REORDER_PBR, REORDER_RCM, TILE_AUTO, TILE_SPARSE, TILE_DENSE, TILE_SPARSE_GATHER,
)
