"""Seeded synthetic inputs for the packed ViT image encoder.

This module serves both the CPU oracle's tests and the HIP library's tests and
benchmark.  It produces *inputs only* (encoder shapes, weights, pixels, request
structure); it contains none of the encoder's arithmetic.
"""
from .configs import (  # noqa: F401
    CONFIGS,
    get_config,
    out_tokens_per_tile,
    tokens_per_tile,
    weight_count,
    weight_layout,
)
from .inputs import (  # noqa: F401
    CFG3_IMAGES_PER_REQUEST,
    CFG4_TILES_PER_IMAGE,
    make_arrivals,
    make_image_u8,
    make_pixels,
    make_weights,
    make_workload,
    round_to_bf16,
)
