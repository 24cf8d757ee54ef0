"""Seeded synthetic inputs for the routed encoder-decoder training step.

This package only *draws* inputs (token ids, sentence lengths, batches, translation
directions, initial parameter values) and *describes* the five benchmark set-ups
(which modules exist, how many layers each has, which modules a direction uses).
It holds none of the method's arithmetic, so both the CPU checker and the GPU
library may be fed from it without sharing any computation.
"""
from .configs import CONFIGS, ModelShape, ModuleSpec, Setup, build_setup  # noqa: F401
from .data import (  # noqa: F401
    Batch,
    draw_content_ids,
    draw_lengths,
    make_batches,
    make_pool,
    sample_directions,
    task_probabilities,
    zipf_cdf,
)
from .init import fill_params  # noqa: F401
from .sharing import (  # noqa: F401
    PATTERNS,
    layerwise_tasks,
    parse_stack,
    pattern_setup,
    route_signature,
    sharing_name,
)
