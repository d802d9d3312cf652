"""Integer-only LSTM cell step (arXiv 2101.05453) for AMD MI355X.

The product is the C-ABI library liblstm_int.so (include/lstm_int.h), built
from csrc/ by paper_2101_05453_amd.build; binding.py exposes the same entry
points to Python (argument marshalling only).
"""
from . import binding  # noqa: F401
from .binding import (CIFG, LAYER_NORM, PEEPHOLE, PROJECTION, LstmIntError, Model, prepare,  # noqa: F401
                      strerror)
