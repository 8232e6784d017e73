"""Seeded synthetic inputs and the default formatbook table (data only)."""
from .formatbook import (DEFAULT_FORMATBOOK, E2M1_X2_FORMATBOOK, UNIFORM_STEP2_FORMATBOOK,
                         default_formatbook, range_buckets)
from . import synth

__all__ = ["DEFAULT_FORMATBOOK", "E2M1_X2_FORMATBOOK", "UNIFORM_STEP2_FORMATBOOK",
           "default_formatbook", "range_buckets", "synth"]
