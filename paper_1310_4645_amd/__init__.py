"""MI355X (gfx950) library for constructing, timing and replaying pipelined
reduction schedules (Lowery & Langou, "A Greedy Algorithm for Optimally
Pipelining a Reduction").  This package is a thin ctypes binding over the C ABI
of include/prs.h; every step of the computation runs in the HIP kernels of
csrc/.  There is no CPU fallback: importing the binding without a built
libprs.so raises."""
from .binding import (  # noqa: F401
    PRS_UNI, PRS_BI, PRS_COST_I64, PRS_COST_F64, PRS_I32, PRS_F32, PRS_F64, PRS_I64, PRS_OP_SUM, PRS_OP_MAX,
    PRS_CALL_SIMULATE, PRS_CALL_SCHEDULE, PRS_CALL_REPLAY, PRS_CALL_OFFSETS, PRS_CALL_SEARCH, PRS_CALL_UNEQUAL,
    DeviceConfigs, load_library, library_path, exported_symbols,
    prs_workspace_bytes, simulate_completion_batch, optimal_segmentation_batch, unequal_segmentation_batch, prs_pair_offsets,
    greedy_schedule_batch, replay_reduction, replay_reduction_static, butterfly_threshold_batch, prs_measure_alu_ceiling, PrsError,
)
