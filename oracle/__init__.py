"""CPU oracle (test infrastructure only): the plain fp64 definition the GPU library is checked against.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It never imports the GPU package.
"""
from .reference import (  # noqa: F401
    Hyper, OracleTensor, adam_step, lamb_step, build, half_to_double, float_to_half, grad_overflow,
    philox4x32_10, dropout_word, dropout_threshold, double_to_half, mp_epilogue,
)
