"""Ecco block codec for MI355X: HIP kernels behind a C ABI (include/ecco.h) and their ctypes binding.

`workloads` (seeded synthetic inputs) is importable on its own; the binding loads libecco.so lazily
and fails loudly if it has not been built.
"""
from .binding import (EccoError, Model, ecco_device_info, ecco_act_decode, ecco_act_encode, ecco_decode, ecco_decode_gemv, ecco_decode_indices, ecco_encode,  # noqa: F401
                      ecco_encode_minmax, ecco_fit_patterns, ecco_kv_append, ecco_kv_append_minmax, ecco_kv_attend, ecco_kv_attend_gqa, ecco_kv_attend_gqa_noalloc, ecco_kv_attend_gqa_splits, GQA_SCRATCH_BYTES, ecco_model_create, ecco_model_load,
                      ecco_model_save, ecco_model_to_device, ecco_read_stream, strerror,
                      PbModel, ecco_pb_decode, ecco_pb_decode_gemv, ecco_pb_encode, ecco_pb_fit, ecco_pb_model_create, ecco_pb_model_load,
                      ecco_pb_model_save, ecco_pb_model_to_device)
