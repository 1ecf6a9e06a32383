"""CPU oracle for change-based convolution -- TEST INFRASTRUCTURE, not a product path.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package.
It never imports the HIP binding and shares no code with it.
"""
from .steps import (build, conv_dense, conv_update, maxpool, detect, update_ref, update_set,
                    extract, pool_set, round_bf16, max_threads)
from .net import OracleCBNet, dense_forward
