"""Seeded synthetic inputs for the RSD hot path.

This package holds no arithmetic of the method itself: only the workload
definitions (model shapes, batch sizes, decoding limits) and counter-based
generators that turn ``(seed, stream, tensor id, index)`` into weights,
prompts and uniforms.  Both the CPU checker and the HIP path take their
inputs from here, so neither has to trust the other for them.
"""
from .configs import ModelShape, Workload, WORKLOADS, workload, blob_layout
from .generate import (
    STREAMS,
    hash32_np,
    normal_table,
    weight_values_np,
    model_weights_np,
    model_blob_np,
    model_blob_torch,
    weights_from_blob,
    prompt_lengths,
    prompt_tokens,
    uniforms,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
)

__all__ = [
    "ModelShape", "Workload", "WORKLOADS", "workload", "blob_layout", "STREAMS",
    "hash32_np", "normal_table", "weight_values_np", "model_weights_np",
    "model_blob_np", "model_blob_torch", "weights_from_blob", "prompt_lengths", "prompt_tokens",
    "uniforms", "bf16_bits_to_f32", "f32_to_bf16_bits",
]
