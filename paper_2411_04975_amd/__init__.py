"""MI355X-native draft generation for SuffixDecoding (arxiv 2411.04975).

The work is done by hand-written HIP kernels behind the C ABI declared in
include/sd.h; this package is a thin ctypes binding with the same call names.
There is no CPU fallback: importing the binding without the built shared
object raises.
"""
from .binding import (SD_SCOPE_GLOBAL, SD_SCOPE_REQUESTS, SD_STATIC_SCRATCH_BYTES, SD_TICK_SLOTS,  # noqa: F401
                      SdError, Trees, lib_path, sd_accept, sd_accept_append,
                      sd_accept_append_speculate, sd_create, sd_debug_profile,
                      sd_debug_profile_read, sd_debug_read_global, sd_debug_read_request_ticks,
                      sd_debug_read_unit_ticks, sd_destroy, sd_get_stats, sd_index_append,
                      sd_index_build, sd_index_entropy, sd_index_insert, sd_speculate,
                      sd_speculate_static)
