"""MI355X-native token-adapted transformer encoder (OTAS token adaptation): Python binding of the
C ABI in include/otas.h and include/otas_sched.h.  Argument marshalling only; every step runs in the HIP library."""
from .binding import (  # noqa: F401
    OTAS_F32, OTAS_BF16, OTAS_FLAG_SIZE_BIAS, OTAS_FLAG_TRACE, OTAS_PROMPT_REPLACE, OTAS_PROMPT_GROW, OtasError, Context, Scheduler, OTAS_GAMMA_SKIP, OTAS_GAMMA_UNDECIDED, lib_path, load_library,
    otas_schedule, otas_strerror, otas_sched_rate_table, OTAS_CLOCK_PROBE_MAX_SAMPLES,
)
