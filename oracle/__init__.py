"""CPU checker (test infrastructure): ctypes access to oracle/pp_oracle.cpp.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It imports nothing from the GPU library's package.
"""
from .binding import (build, lib, expand_weights, conv, conv_at, brute, maxpool2, round_f16, widen_f16, plan_ref,
                      expand_weights_k, conv_k, conv_k_at, brute_k, out_size,
                      layer_dense_weights, layer_reference,
                      block_expand, gemm, gemm_at, block_brute, block_layer_reference,
                      reuse_signatures, reuse_representatives, reuse_layer)
