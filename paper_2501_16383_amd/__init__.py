"""RotateKV 2-bit KV-cache hot path for MI355X: thin Python binding over librkv.so."""
from .binding import (  # noqa: F401
    RkvConfig, RkvCache, RkvError, calibrate_perm, fold_rotation, layout_locate, library_path, load_library, query_sizes, select_sinks,
)
