"""MI355X-native fused INT3/INT4 + low-rank linear layer (FBQuant inference hot path).

Thin ctypes binding over libfbq.so (see include/fbq.h).  Importing this package does not load the
library; the first call does, and fails loudly if it has not been built.
"""
from .fbq import (FbqError, Desc, lib_path, load, status_string, packed_bytes, workspace_bytes, pack,  # noqa: F401
                  linear, linear_static, linear_unfused, linear_group, make_group, reconstruct, unpack_codes, quantize_feedback, PackedLayer, DeviceLayer, upload_layer,
                  train_workspace_bytes, gram, train_state, train_step, TrainState, EXPORTED_SYMBOLS)
