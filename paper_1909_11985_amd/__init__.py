"""MI355X-native data-parallel training step of an elastic deep-learning job.

`binding` mirrors the C boundary declared in include/edl.h; every step of the
path runs in the HIP kernels of libedl.so.  PyTorch is used by callers only
to allocate device memory and to provide streams.
"""
from .binding import (  # noqa: F401
    EdlError, Config, Sizes, Job, Pipeline, MODELS, DTYPES,
    edl_query, edl_shard_host, edl_init_params_host, edl_tensor_table,
    edl_adam_update, edl_average_update, edl_copy, edl_mfma_rate, edl_profile, edl_profile_report, lib,
    edl_set_option, edl_get_option, options,
)
