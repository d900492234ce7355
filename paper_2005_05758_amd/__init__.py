"""MI355X-native CSB-RNN inference: thin ctypes binding over libcsbrnn.so.

The binding only marshals arguments; every step of the path runs in the library's
gfx950 kernels (device calls) or its host packer/planner.  There is no CPU fallback: if
the library is missing, importing the binding's functions raises.
"""
from .binding import (CsbMatrix, CsbRnn, CsbError, CELL_LSTM, CELL_GRU, CELL_LSTMP, CELL_LIGRU, CELL_GRU_RB, VAL_F32, VAL_F16, VAL_BF16, lib, lib_path,
                      load_library, stream_read, project)

__all__ = ["CsbMatrix", "CsbRnn", "CsbError", "CELL_LSTM", "CELL_GRU", "CELL_LSTMP", "CELL_LIGRU", "CELL_GRU_RB", "VAL_F32", "VAL_F16", "VAL_BF16", "lib", "lib_path",
           "load_library", "stream_read", "project"]
