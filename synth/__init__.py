"""Seeded synthetic inputs: model shapes, random-init weights, prompts, uniforms.

This package only *makes input data* and describes its format.  It contains none of
the method's arithmetic (no network forward, no acceptance rule, no sampling), so
both the CPU oracle's tests and the HIP library's tests/benchmarks may use it; the
oracle and the HIP path never import one another.
"""
from .shapes import ModelShape, Workload, WORKLOADS, workload, mini_moe_shape  # noqa: F401
from .weights import HostModel, make_model, bf16_bits_to_f32, f32_to_bf16_bits  # noqa: F401
from .data import make_prompts, make_uniforms, make_layer_inputs  # noqa: F401
