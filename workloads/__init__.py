"""Seeded synthetic inputs for the model-aggregation path.

This package serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds tensor-shape lists and a counter-based value generator and
nothing of the aggregation method itself: no block splitting, no summation, no
optimizer arithmetic.
"""
from .shapes import (  # noqa: F401
    MODEL_BUILDERS,
    JobSpec,
    alexnet,
    awd_lm,
    bert_base,
    mlp,
    resnet50,
    vgg16,
    job_config,
    packed_wave_jobs,
)
from .values import fill_normal_like, draw_from, stream_key  # noqa: F401
