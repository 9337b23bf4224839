"""Seeded synthetic inputs (model configs, weights, request workloads).

This package is the only code shared by the CPU oracle and the HIP path. It holds
input generation only: no scheduling, no model arithmetic, no sampling.
"""
from .configs import MODEL_CONFIGS, ENGINE_CONFIGS, model_config, engine_config  # noqa: F401
from .weights import make_weights, pack_blob, tensor_order, f32_to_bf16_bits, bf16_bits_to_f32  # noqa: F401
from .workloads import make_workload, splitmix64, with_shared_prefixes, with_repetition  # noqa: F401
