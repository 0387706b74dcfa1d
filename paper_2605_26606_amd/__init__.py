"""MI355X-native group rollout generation with Pilot-Commit allocation.

The work is done by hand-written HIP kernels behind the C ABI of
``include/pc.h`` (built in-tree as ``libpc.so``); this package only marshals
arguments.  PyTorch supplies device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    PcError, Context, Scheduler, library, pc_prefill_shared, pc_fork, pc_fork_need, pc_decode_step, pc_decode_step_static, pc_release, pc_score, pc_sample,
    pc_group_stats, pc_select_commit, pc_select_commit_var, pc_advantages, pc_kv_blocks, pc_slots, pc_set_option, pc_saturation_count,
    pc_timing_read, PC_OPT_USE_GRAPH, PC_OPT_FORCE_SIMT, PC_OPT_TIME_NEXT_STEP, PC_OPT_FUSE_DECODE, PC_KERNEL_ATTN_DECODE,
    PC_KERNEL_GEMM_QKV, PC_KERNEL_GEMM_WO, PC_KERNEL_GEMM_GATE_UP, PC_KERNEL_GEMM_DOWN, PC_KERNEL_GEMM_LM_HEAD,
)
from .rollout import pilot_commit_step, generate, generate_wave, plan_waves, BoundPipeline  # noqa: F401
