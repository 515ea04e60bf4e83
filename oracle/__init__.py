"""CPU oracle for the ConvBN block with frozen BatchNorm (test infrastructure only).

fp64, logical NCHW numpy arrays, direct loops in C (oracle/convbn_oracle.c).
Eval mode (Sec. 3.1, App. C, Table 2 "Eval") is the definition the GPU library is
compared with; Tune mode (Sec. 3.3, Table 2 "Tune") is carried as a second,
independent route so that Tune == Eval (Sec. 3.4.1) can be asserted on the CPU.
The t* functions are the same two routes for the TransposedConv-BN block (Sec. 3.2.1), the dw_*
functions for the depthwise ConvBN block (one filter per channel), the g_* functions for the grouped block.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
this package.  It imports nothing from the GPU package.
"""
from .oracle import (Dims, conv_fwd, conv_dgrad, conv_wgrad, eval_fwd, eval_bwd, fold,
                     tune_fwd, tune_bwd, num_threads, out_hw,
                     tconv_out_hw, tconv_fwd, tconv_dgrad, tconv_wgrad, teval_fwd, teval_bwd,
                     ttune_fwd, ttune_bwd,
                     dw_fwd, dw_dgrad, dw_wgrad, dw_eval_fwd, dw_eval_bwd, dw_tune_fwd, dw_tune_bwd,
                     g_fwd, g_dgrad, g_wgrad, g_eval_fwd, g_eval_bwd, g_tune_fwd, g_tune_bwd)

__all__ = ["Dims", "conv_fwd", "conv_dgrad", "conv_wgrad", "eval_fwd", "eval_bwd", "fold",
           "tune_fwd", "tune_bwd", "num_threads", "out_hw",
           "tconv_out_hw", "tconv_fwd", "tconv_dgrad", "tconv_wgrad", "teval_fwd", "teval_bwd",
           "ttune_fwd", "ttune_bwd",
           "dw_fwd", "dw_dgrad", "dw_wgrad", "dw_eval_fwd", "dw_eval_bwd", "dw_tune_fwd", "dw_tune_bwd",
           "g_fwd", "g_dgrad", "g_wgrad", "g_eval_fwd", "g_eval_bwd", "g_tune_fwd", "g_tune_bwd"]
