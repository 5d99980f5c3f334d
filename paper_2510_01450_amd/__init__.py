"""MI355X-native Local Linear Attention (arxiv 2510.01450): thin Python binding of the C ABI.

``llla_forward`` / ``llla_decode`` marshal torch device tensors into the ``extern "C"`` entry points
of ``libllla.so`` (declared in ``include/llla.h``); every step of the method runs in the library's
HIP kernels.  There is no CPU or PyTorch fallback: a missing library is an error.
"""
from .binding import (LlaError, PATHS, decode_workspace_bytes, forward_cg_workspace_bytes, forward_workspace_bytes, lib,
                      llla_forward_cg, llla_backward, backward_workspace_bytes,  # noqa: F401
                      lib_path, llla_decode, llla_decode_static, llla_forward, measure_lib, measure_lib_path, probe_copy, probe_mfma_f16, profile_enable,
                      profile_last, status_string, use_measure_library, version)
