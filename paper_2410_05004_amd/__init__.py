"""MI355X-native HCache KV restoration: thin ctypes binding over libhcache.so.

Every step of the restoration path runs inside the HIP library; this package only
marshals arguments (pointers, sizes, stream handles).  There is no CPU fallback: if
the library has not been built, importing `paper_2410_05004_amd.binding` raises.
"""
from .binding import (  # noqa: F401
    HCacheError,
    ModelDesc,
    Context,
    Store,
    Saver,
    lib,
    lib_path,
    version,
    validate_desc,
    static_stage_bytes,
    diag_mfma_duty,
    diag_tile_map,
    diag_split_plan,
    partition_layers,
    HC_OK, HC_EINVAL, HC_ERANGE, HC_EALIGN, HC_ENOMEM, HC_EHIP, HC_ESTATE,
    HC_DEV_BAD_POSITION, HC_DEV_BAD_PAGE, HC_NORM_RMS, HC_NORM_LAYER,
)
