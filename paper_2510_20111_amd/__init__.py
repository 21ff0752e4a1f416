"""MI355X-native shard-update hot path of hierarchical ZeRO parallelism (AsyncHZP).

The product is ``libhzp.so`` (HIP kernels for gfx950 behind the C ABI of ``include/hzp.h``);
this package is its thin ctypes binding.  Importing it requires the built library.
"""
from .binding import (  # noqa: F401
    HZP_CLASS_BF16, HZP_CLASS_F32, HZP_GRAD_DEFAULT, HZP_GRAD_BF16, HZP_GRAD_F32, HZP_MAX_GROUP,
    HZP_MAX_REPLICAS, HZP_ARENA_ALIGN, HZP_ARENA_VARIANTS,
    HZP_STREAM_GRAD, HZP_STREAM_MASTER, HZP_STREAM_M, HZP_STREAM_V, HZP_STREAM_PARAM_OUT, HZP_STREAM_RECV1,
    HZP_STREAM_SHARD3, HZP_STREAM_RECV3,
    HZP_OK, HZP_ERR_INVALID_ARG, HZP_ERR_RANGE, HZP_ERR_UNSUPPORTED, HZP_ERR_ALIGN,
    HZP_ERR_NOMEM, HZP_ERR_HIP,
    EXPORTS, LIB_PATH, HzpError, Plan, Sched, adamw_hyper, ptr_array,
    hzp_plan, hzp_plan_free, hzp_memory_model, hzp_choose_groups, hzp_reduce_shard, hzp_adamw_shard, hzp_adamw_scalars, hzp_adamw_shard_dev, hzp_gather_layer, hzp_gather_layer_static, hzp_gather_layers, hzp_gather_shard, hzp_gather_tensor,
    hzp_last_error,
)
