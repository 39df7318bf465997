"""Seeded synthetic workloads shared by tests, the benchmark and the oracle checks.

This package holds no arithmetic of the method (no basis, no projection, no
attention): only shapes, random draws and dtype rounding.
"""

from .configs import (FAConfig, CONFIGS, PAPER_SETTING, get_config, one_launch_variants, random_variants,  # noqa: F401
                      small_variants)
from .synth import (  # noqa: F401
    round_to_bf16,
    bf16_bits,
    make_masks,
    make_context,
    rel_err,
)
