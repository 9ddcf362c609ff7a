"""Seeded synthetic inputs for the VTC serving step.

This package only *generates inputs*: request arrival traces, batch shapes,
block tables and Q/K/V tensors.  It contains none of the method's arithmetic
(no attention, no counter update, no scheduling decision), so that both the
GPU library's tests and the CPU oracle can consume exactly the same arrays
without sharing any computation.
"""
from .traces import Request, poisson_trace, uniform_trace, trace_for_config  # noqa: F401
from .batches import StepBatch, ModelShape, make_step_batch, load_snapshot, CONFIG_IDS  # noqa: F401
from .tensors import (  # noqa: F401
    make_block_table,
    make_qkv_numpy,
    f32_to_storage_bits,
    poison_unused_rows,
    NAN_BITS,
)
from .device import (  # noqa: F401,E402
    DeviceStep,
    bits_to_tensor,
    make_device_step,
    sequence_rows_to_host,
    tensor_to_bits,
    torch_dtype,
)
