"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws random lengths and random tensors.  It holds none of the
attention or balancing arithmetic: both the CPU oracle and the HIP path receive
what is generated here as plain arrays.
"""
from .bags import (  # noqa: F401
    CONFIG_NAMES,
    BagSpec,
    config_bag,
    cu_seqlens_of,
    data_code_lengths,
    parse_data_code,
    table1_streams,
)
from .tensors import (  # noqa: F401
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_qkv_dout,
)
