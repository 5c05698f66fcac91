"""MI355X-native greedy self-speculative decode round with DEL (arXiv 2504.05598).

Thin ctypes binding over the C ABI in include/del.h; every step of the path runs
in the HIP library (paper_2504_05598_amd/libdel_hip.so).
"""
from .binding import (DelError, DelContext, lib_path, load_library, EXPORTS,
                      del_create, del_destroy, del_load_weights, del_prefill, del_round, del_round_dynamic,
                      del_layer_stats, del_set_layer_stats, del_last_timings)

__all__ = ["DelError", "DelContext", "lib_path", "load_library", "EXPORTS",
           "del_create", "del_destroy", "del_load_weights", "del_prefill", "del_round", "del_round_dynamic",
           "del_layer_stats", "del_set_layer_stats", "del_last_timings"]
