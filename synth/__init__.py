"""Seeded synthetic inputs (model shapes, weights, prompts).

This package is the only code shared by the CPU oracle and the HIP library's
tests/bench.  It holds no arithmetic of the speculative-decoding method: it
only names shapes and fills buffers with reproducible pseudo-random bytes.
"""
from .configs import ModelConfig, CONFIGS, get_config          # noqa: F401
from .gen import (tensor_specs, make_weights, make_prompt,      # noqa: F401
                  fill_normal, fill_tokens, to_float64, STORAGE_NP)
