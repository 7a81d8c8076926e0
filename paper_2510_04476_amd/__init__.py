"""MI355X-native prefill path of Compressed Convolutional Attention (CCA / CCGQA).

The work is done by hand-written HIP kernels in ``libcca.so`` (C ABI in
``include/cca.h``); this package is the thin ctypes binding around it.
"""
from .binding import *  # noqa: F401,F403
from .binding import (CCAConfig, CCAWeights, CCASaved, CCAError, load_library, cca_forward, cca_down_project,
                      cca_prologue, cca_attention, cca_attention_backward, cca_up_project, cca_workspace_size, cca_strerror, cca_version,
                      new_workspace, EXPORTS, LIB_PATH, CCAGrads, cca_backward, cca_backward_workspace_size,
                      cca_prologue_backward, new_backward_workspace, CCADecodeState, cca_decode_step,
                      cca_decode_workspace_size, cca_prepare, cca_prepared_size, cca_probe_mfma_rate, cca_decode_step_static, cca_decode_step_ragged, CCA_DECODE_STATIC_BYTES)
from .hostutil import config_from_workload, weights_to_device, forward_flops  # noqa: F401
