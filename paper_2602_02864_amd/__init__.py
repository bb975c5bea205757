"""MI355X-native parallel decoding step for template-structured CoT.

`binding` wraps the C ABI of libfdc.so (declared in include/fdc.h); `build`
compiles the library for gfx950.  Nothing here computes: the decode path runs
entirely in the HIP kernels under csrc/.
"""
from . import binding  # noqa: F401
from .binding import (Context, FdcError, Scheduler, fdc_argmax, fdc_attention_plan, fdc_build_mask, fdc_dense_mask,  # noqa: F401
                      fdc_linear, fdc_linear_static, fdc_pack_weight, fdc_packed_weight_bytes, fdc_profile_calibrate,
                      fdc_schedule, fdc_stream_copy, lib)
