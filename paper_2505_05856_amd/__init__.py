"""MI355X-native forward+backward step of one pipeline stage under a
keep / recompute / swap plan (libdpstage.so + a thin ctypes binding)."""
from . import binding  # noqa: F401
from .binding import (DpError, Stage, last_error, make_config, plan_len, plan_validate, stage_init,  # noqa: F401
                      stage_op_times, stage_set_debug, stage_set_profiling, stage_step)
