"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package holds workload descriptions (shapes, decoding hyper-parameters) and a
counter-based generator for weights and prompts.  It contains none of the method's
arithmetic: no attention, no softmax, no commit/merge logic.
"""
from .configs import ModelShape, DecodeParams, Workload, workload, WORKLOAD_NAMES, EXTRA_WORKLOAD_NAMES  # noqa: F401
from .gen import weight_specs, gen_tensor, gen_weights, gen_prompt, gen_prompt_lengths  # noqa: F401
