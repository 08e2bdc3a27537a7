"""Batch-1 Pipelined Backpropagation tick engine for MI355X: thin Python
binding over the C ABI of libpb_hip.so (see include/pb.h)."""
from .binding import (PBEngine, PBError, lib_path, load_library, scale_hyperparameters,  # noqa: F401
                      update_standalone)
