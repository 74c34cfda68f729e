"""MI355X-native incremental GNN inference on streaming graphs (thin binding over libink.so)."""
from .binding import (Ink, InkError, load_library, lib_path, EDGE_UPDATE_DTYPE, STATUS_NAMES,
                      MODEL_KINDS, AGGS)

__all__ = ["Ink", "InkError", "load_library", "lib_path", "EDGE_UPDATE_DTYPE", "STATUS_NAMES",
           "MODEL_KINDS", "AGGS"]
