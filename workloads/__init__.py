"""Seeded synthetic inputs for the SuffixDecoding draft-generation path.

This package holds input generators only (token streams, contexts, ground-truth
continuations).  It contains none of the method's arithmetic: no suffix
indexing, matching, scoring or acceptance logic lives here, so both the CPU
oracle's tests and the HIP path's tests may draw their inputs from it.
"""
from .synth import CONFIGS, Workload, make_workload, scaled  # noqa: F401
