"""One Zero-Bubble pipeline stage (arXiv 2401.10241) on one MI355X: F / B / W passes of a stack
of GPT decoder layers in ZB-H1 / ZB-H2 order and the post-validated AdamW step, as a C-ABI HIP
library (libzbstage.so, see include/zb_stage.h) plus this thin ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import (Stage, ZbError, schedule_order, schedule_stash_need, order_stash_need,  # noqa: F401
                      simulate_pipeline, auto_schedule, auto_schedule_search, order_memory_peak, order_group_w,
                      simulate_pipeline_w_runs,
                      schedule_order_v, simulate_pipeline_v, lib)
