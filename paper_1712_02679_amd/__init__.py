"""libadacomp for MI355X: AdaComp residual-gradient compression (pack / unpack hot path).

The product is the C library ``libadacomp.so`` (sources in ``csrc/``, ABI in ``include/adacomp.h``);
this package is its ctypes binding.
"""
from .binding import (AdacompError, adacomp_compress, adacomp_compress_static, adacomp_compress_batch, adacomp_compress_batch_lazy, adacomp_compress_variant, adacomp_residue_sync, adacomp_copy_f32, adacomp_triad_f32, adacomp_triad_resident_f32, adacomp_fill_f32, adacomp_debug_keep_gmax, adacomp_packet_bound,  # noqa: F401
                      adacomp_packet_fixed_bytes, adacomp_selftest_binindex, adacomp_timing_enable, adacomp_tuning_unpack_min_groups, adacomp_tuning_fold_scan, adacomp_tuning_place_tiled,
                      adacomp_timing_read, adacomp_unpack_accumulate, adacomp_unpack_update, OPT_SGD_MOMENTUM, OPT_ADAM, adacomp_workspace_bytes, adacomp_workspace_bytes_batch,
                      adacomp_workspace_gmax, adacomp_workspace_init, adacomp_workspace_release,
                      read_packet_summary, RULE_ADACOMP, RULE_PRINTED_COMPARE, RULE_LOCAL_SELECTION)
