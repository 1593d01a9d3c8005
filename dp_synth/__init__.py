"""Seeded synthetic inputs and layer manifests for the DP-SGD clipped-gradient path.

This package holds none of the method's arithmetic: it only draws random tensors,
token ids and scalars with fixed seeds and lists the layer shapes of each workload.
Both the CPU oracle's tests and the GPU path's tests/bench draw their inputs here,
so the two sides see identical bits without sharing any code of the method itself.
"""
from .inputs import (  # noqa: F401
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    normal_f32,
    normal_bf16_bits,
    zipf_ids,
    position_ids,
    segment_ids,
    example_scales,
    synthetic_sqnorms,
)
from .manifest import (  # noqa: F401
    LayerSpec,
    bert_manifest,
    single_dense_manifest,
    manifest_param_count,
    CONFIGS,
)
from .device import device_layer_inputs, host_layer_slice  # noqa: F401,E402
