"""MI355X-native decode linear layers for Progressive Mixed-Precision Decoding.

Thin Python binding over the C ABI declared in ``include/pmpd.h``: argument
marshalling only.  Every step of the path (pack, unpack, the bit-plane GEMV, the
one-launch decode step, the schedule) runs in the native library; PyTorch is
used for device memory and streams.  There is no CPU fallback: importing the
binding without the built library raises.
"""
from .binding import (  # noqa: F401
    PMPDError, PackedLayer, Schedule, Stack, batch_step, decode_run, decode_step, gemm, gemv, lib_path, pack,
    packed_size, prefill_step, unpack, upload_layer, exported_symbols, schedule_grid, schedule_count, schedule_search, read_stream, Ordered, Fp16Stack, fp16_gemv, fp16_step, LearnedScheduler, schedule_from_class,
)
