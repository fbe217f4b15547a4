"""Seeded synthetic inputs for the KV-migration hot path.

This package holds input generation only: a counter-based random number
generator, request-length and page-table recipes, and pool fill patterns.
None of the method's arithmetic (routing, flattening, packing, unpacking)
lives here; both the CPU oracle's tests and the GPU path's tests draw their
inputs from here so that the two sides see identical bytes.
"""
from .splitmix import SplitMix64, mix64, stream_words, fill_words, fill_pool_u16
from .host import fill_words_fast
from .configs import (
    ModelShape, M8B, PairCase, make_case, CONFIG_NAMES, lengths_uniform,
    lengths_zipf, slots_fragmented, slots_contiguous, slots_zipf_runs,
    pages_from_slots, random_pages,
)

__all__ = [
    "SplitMix64", "mix64", "stream_words", "fill_words", "fill_pool_u16", "fill_words_fast",
    "ModelShape", "M8B", "PairCase", "make_case", "CONFIG_NAMES",
    "lengths_uniform", "lengths_zipf", "slots_fragmented", "slots_contiguous",
    "slots_zipf_runs", "pages_from_slots", "random_pages",
]
