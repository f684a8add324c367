"""CPU oracle for the convolutional hot path.  TEST INFRASTRUCTURE ONLY.

A ctypes front end over ``conv_oracle.c`` (plain C, fp64, direct loops).  Only
``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg
may import this package; the product package never does, and this package
imports nothing from the product.

Every function takes numpy arrays of any float dtype, widens them to float64
exactly, and returns float64 arrays.  Layouts: activations NCHW, filters KCRS;
``H``/``W`` are always the *input* extent of the layer.
"""
from .oracle import (  # noqa: F401
    build,
    out_extent,
    pool_extent,
    conv_fwd,
    conv_bwd_data,
    conv_bwd_filter,
    conv_fwd_at,
    conv_bwd_data_at,
    conv_bwd_filter_at,
    conv_fwd_grouped,
    conv_bwd_data_grouped,
    conv_bwd_filter_grouped,
    relu_fwd,
    relu_bwd,
    maxpool3x3s2_fwd,
    maxpool3x3s2_bwd,
    bias_fwd,
    bias_bwd,
    conv_fwd_bias_relu,
    conv_bwd_data_relu,
    fc_fwd,
    fc_bwd_data,
    fc_bwd_filter,
    sgd_update,
    bf16_bits,
    bf16_round,
    num_threads,
    set_num_threads,
)
