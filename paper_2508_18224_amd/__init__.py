"""MI355X-native selected-block attention (the `sel` branch of Native Sparse Attention, FSA paper Sec. 3).

Thin ctypes binding over libnsa_sel.so (include/nsa_sel.h).  PyTorch is used for device memory and streams
only; every step of the path runs in the library's HIP kernels.  There is no CPU fallback: without the built
library, or without a GPU, the calls raise.
"""
from .binding import (NsaSelError, Shape, build_index, index_view, lib, nsa_sel_bwd, nsa_sel_fwd, nsa_sel_fwd_static,  # noqa: F401
                      workspace_bytes, workspace_bytes_min, SelAttention, select_blocks, window_blocks, profile_enable, profile_select, profile_collect, calibration_copy, mfma_probe, SYMBOLS)
from .autograd import selected_attention  # noqa: F401,E402
