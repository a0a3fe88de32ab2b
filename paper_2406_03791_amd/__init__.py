"""MI355X (gfx950) engine for exact batched RNN-T / TDT greedy decoding.

The package is a thin binding over the C ABI in include/rnnt_greedy.h
(librnnt_greedy.so, built from csrc/ by build.py): the functions below carry the
C names and only marshal arguments; every step of the decode runs in the HIP
kernels.  There is no fallback: importing fails if the library is not built.
"""
from .binding import (  # noqa: F401
    RNNT_DEV_ABORTED,
    RNNT_DEV_LEN_CLAMPED,
    RNNT_DEV_OVERFLOW,
    RNNT_FLAG_BF16_WEIGHTS,
    RNNT_FLAG_FP8_WEIGHTS,
    RNNT_FLAG_PLAIN_LAUNCH,
    RNNT_FLAG_BF16_ARITHMETIC,
    RNNT_FLAG_MULTI_BLANK,
    Engine,
    RnntError,
    RnntStats,
    lib_path,
    load_library,
    rnnt_encoder_projection,
    rnnt_engine_configure,
    rnnt_engine_create,
    rnnt_engine_destroy,
    rnnt_engine_set_logp_output,
    rnnt_engine_set_done_flags,
    rnnt_engine_set_wait_limit,
    rnnt_engine_phase_timers,
    rnnt_engine_stats,
    rnnt_probe_e4m3_widening,
    rnnt_quantize_rows_e4m3,
    rnnt_quantize_blocks_e2m1,
    rnnt_probe_e2m1_widening,
    RNNT_FLAG_FP4_WEIGHTS,
    RNNT_FP4_BLOCK,
    rnnt_probe_exchange,
    rnnt_probe_mfma,
    rnnt_probe_stream,
    rnnt_engine_status,
    rnnt_greedy_decode,
    rnnt_label_looping_decode,
    rnnt_label_looping_decode_noalloc,
    rnnt_status_string,
    tdt_label_looping_decode,
)
