"""MI355X-native speculative-verification hot path of PipeInfer: Python binding of the C ABI."""
from .binding import (Model, KVCache, KVMeta, Scheduler, seq_bits, Run, stage_forward, stage_forward_multi, verify_greedy, verify_greedy_noalloc, verify_greedy_chained, kv_rollback, mapped_device_pointer, lib, strerror,
                      PiError, PI_OK, PI_CANCELLED, PI_E_ARG, PI_E_SHAPE, PI_E_OOM, PI_E_SLOT_LIVE,
                      PI_E_HIP, PI_E_STATE, PI_E_FULL, PI_E_BUSY, PI_MAX_BATCH, PI_WINDOW, PI_MAX_SEQ,
                      PI_POS_MAX, PI_DTYPE_FP8_E4M3, PI_DTYPE_FP4_E2M1, PI_DTYPE_FP4_E2M1_B32, PI_RUN_SUPERFLUOUS, PI_RUN_INVALIDATED)
from . import binding
