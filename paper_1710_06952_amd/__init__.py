"""MI355X-native AD-PSGD worker-update engine: Python face of libadpsgd.so.

``binding`` mirrors the C ABI of include/adpsgd.h one to one; ``Engine`` adds
only what a caller needs around it: device buffers and a stream from PyTorch.
"""
from .binding import (AdpsgdError, Handle, adpsgd_make_schedule, adpsgd_plan_rounds,  # noqa: F401
                      adpsgd_synth_gradient, adpsgd_metropolis_weights, adpsgd_verify_plan, lib, EXPORTS, LIB_PATH, MODEL_LSQ, MODEL_LOGREG,
                      MODEL_SYNTH, MODEL_MLP, MODEL_EXTERNAL, FLAG_PROFILE, FLAG_DENSE_GRADIENT, FLAG_VERIFY_PLAN, FLAG_SYNC_IN_PLACE)
from .engine import Engine  # noqa: F401
from . import step_sizes  # noqa: F401
