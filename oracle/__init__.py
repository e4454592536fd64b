"""CPU oracle for SuffixDecoding draft generation.  TEST INFRASTRUCTURE ONLY.

A plain pointer suffix trie in C (suffix_trie.c) behind a ctypes wrapper.  It
shares no code with the HIP path and the product never imports it: only the
tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
from .trie import (Trie, accept, build_library, generate, library_path,  # noqa: F401
                   speculate_unit)
