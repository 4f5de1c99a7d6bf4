"""CPU oracle (test infrastructure only): see decoder.py, kvmeta.py and scheduler.py."""
from .decoder import (PI_OK, PI_CANCELLED, OracleModel, OracleKV, stage_forward, verify_greedy, verify_greedy_chained,
                      kv_rollback, rmsnorm, linear, rope, attention, silu, visible_cells,
                      round_to_storage, to_f64, top2_gap)
from .kvmeta import OracleKVMeta, PI_E_FULL, PI_E_BUSY, POS_MAX
from .scheduler import OracleScheduler, SUPERFLUOUS, INVALIDATED
