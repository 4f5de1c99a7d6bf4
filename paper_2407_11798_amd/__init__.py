"""MI355X-native speculative-verification hot path of PipeInfer: Python binding of the C ABI."""
from .binding import (Model, KVCache, Run, stage_forward, stage_forward_multi, verify_greedy, kv_rollback, lib, strerror,
                      PiError, PI_OK, PI_CANCELLED, PI_E_ARG, PI_E_SHAPE, PI_E_OOM, PI_E_SLOT_LIVE,
                      PI_E_HIP, PI_E_STATE, PI_MAX_BATCH, PI_WINDOW)
from . import binding
