"""CPU oracle for the u8 x s8 -> s32 GEMM.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product package never does.
"""
from .ngemm_oracle import (  # noqa: F401
    build,
    gemm_u8s8s32,
    gemm_s8s8s32,
    gemm_u8u8s32,
    gemm_s16s16s32,
    gemm_u8s8s64,
    gemm_u8s8s32_sampled,
    gemm_u8s8u8_requant,
    gemm_u8s8u8_requant_channel,
    num_threads,
    requant_s32u8,
)
