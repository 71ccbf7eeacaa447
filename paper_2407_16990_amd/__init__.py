"""Region-aware enhancer for MI355X: thin Python binding over librh.so (see include/rh.h)."""
from .binding import (RH, Config, NetDesc, Segment, BOX_DTYPE, PLACE_DTYPE, RhError, lib_path,  # noqa: F401
                      load_library, needed_radii, select_regions_noalloc)
