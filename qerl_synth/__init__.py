"""Seeded synthetic inputs and layer shapes shared by the tests, the smoke
check and the benchmark.  Holds no arithmetic of the method itself."""
from .inputs import (  # noqa: F401
    BASE_SEED, seed_for, normal_bf16, normal_f32, weights, activations,
    lora_pair, rms_gain, aqn_noise,
)
from .shapes import LinearShape, CONFIGS, config_linears  # noqa: F401
