"""MI355X-native MixLLM quantized linear layer (arxiv 2412.14590): thin Python binding over
the C-ABI library libmixllm_hip.so.  See include/mixllm.h for the contract of every call."""
from .binding import (PATH_AUTO, PATH_DECODE, PATH_DECODE_RESIDENT, PATH_DECODE_SPLIT, PATH_DECODE_STREAM, PATH_GENERIC,
                      PATH_MID, PATH_PREFILL, PATH_PREFILL_32, PATH_PREFILL_64, PATH_PREFILL_128, MixllmError, PackedLayer,
                      abi_version, build_feature_perm, channel_salience, debug_channel_sums, debug_group_partials, lib,
                      linear, linear_fp16, linear_fp16_static, mixed_linear, pack_weights, quantize_activations, quantize_weights,
                      query_sizes, select_salient, unpack_weights)

__all__ = ["PATH_AUTO", "PATH_DECODE", "PATH_DECODE_RESIDENT", "PATH_DECODE_SPLIT", "PATH_DECODE_STREAM", "PATH_GENERIC",
           "PATH_MID", "PATH_PREFILL", "PATH_PREFILL_32", "PATH_PREFILL_64", "PATH_PREFILL_128", "MixllmError", "PackedLayer",
           "abi_version", "build_feature_perm", "channel_salience", "debug_channel_sums", "debug_group_partials", "lib",
           "linear", "linear_fp16", "linear_fp16_static", "mixed_linear", "pack_weights", "quantize_activations", "quantize_weights",
           "query_sizes", "select_salient", "unpack_weights"]
