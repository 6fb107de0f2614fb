"""Pattern-pruned 3x3 convolution for AMD MI355X: thin ctypes binding over libpp_conv.so.

Every step of the convolution runs in the HIP library; this package only marshals arguments.
There is no CPU fallback: importing `pp_conv` fails if the library has not been built.
"""
from .pp_conv import (PP_OK, PP_ERR_NULL, PP_ERR_SHAPE, PP_ERR_PATTERN, PP_ERR_UNSUPPORTED, PP_ERR_ALLOC,
                      PP_ERR_DEVICE, PP_ERR_ALIGN, PP_ERR_SCRATCH, PP_F32, PP_F16, PP_FLAG_RELU, PP_FLAG_DENSE, PP_FLAG_HOST_ONLY, PP_FLAG_POOL2,
                      PPError, Tuning, Plan, KERNEL_REVISION, lib, library_path, pp_conv_plan, pp_conv_run, pp_conv_run_static, pp_conv_destroy,
                      pp_conv_plan_query, pp_conv_plan_unpack, pp_maxpool2x2_run, pp_status_string,
                      plan_from_layer)
from .autotune import autotune, default_candidates
from .pp_block_gemm import (BlockPlan, block_plan_from_layer, pp_block_gemm_plan, pp_block_gemm_run, pp_block_gemm_destroy,
                            pp_block_gemm_query, pp_block_gemm_unpack)
from .pp_deep_reuse import (ReusePlan, reuse_plan_from_layer, pp_reuse_plan, pp_reuse_run, pp_reuse_read_clusters, pp_reuse_destroy)
