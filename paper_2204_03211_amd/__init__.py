"""GPU-resident parameter service for MI355X: model aggregation (sum of the
workers' gradient pushes + momentum-SGD update of the master copy) as HIP
kernels behind a C ABI.  See include/ps.h for the boundary."""
from .binding import (  # noqa: F401
    FLAG_FP_CONTRACT,
    OWNER_ELSEWHERE,
    OWNER_HERE,
    OWNER_LEAVING,
    PS_MAX_W,
    BlockInfo,
    BlockRef,
    BlockStats,
    ParameterService,
    PsError,
    Timing,
    WaveList,
    WaveStats,
    load_library,
)
from .sched_binding import PMaster, Scheduler  # noqa: F401,E402
