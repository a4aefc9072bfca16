"""Seeded synthetic inputs for the DART drafting step.

This package only *draws data* (shapes, seeds, value distributions, storage
formats).  It holds none of the method's arithmetic: no normalisation,
attention, soft-max, scoring or tree logic lives here.  Both the CPU oracle's
tests and the HIP path's tests/bench read their inputs from these functions so
that the two sides always see the same bits.
"""
from .configs import DraftConfig, CONFIGS, get_config, scaled_config
from .tensors import (f32_to_bf16_bits, bf16_bits_to_f32, make_weights,
                      make_hidden, make_frontend_weights, make_features, WEIGHT_NAMES)
from .ngram import (make_ngram_counts, make_prune_case, make_bulk_trigram_counts, bulk_row_of,
                    plant_prune_case, make_backoff_counts, NgramCounts, PruneCase)

__all__ = [
    "DraftConfig", "CONFIGS", "get_config", "scaled_config",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "make_weights", "make_hidden",
    "make_frontend_weights", "make_features",
    "WEIGHT_NAMES", "make_ngram_counts", "make_prune_case", "make_bulk_trigram_counts",
    "bulk_row_of", "plant_prune_case", "make_backoff_counts", "NgramCounts",
    "PruneCase",
]
