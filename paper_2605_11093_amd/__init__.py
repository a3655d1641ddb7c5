"""MI355X-native capture-and-stage path for model-internal observability.

The product is libdmi.so (HIP kernels + C ABI, see include/dmi.h); this package
only marshals arguments for it.
"""
from .binding import (DmiError, PreparedBatch, PreparedObserve, Ring, Step, Stats, RecordView, lib, library_path,  # noqa: F401
                      record_bytes, version)
from . import binding  # noqa: F401
