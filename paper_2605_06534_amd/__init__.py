"""MI355X-native sparse weight-delta synchronisation (ROSE, Sec. 4.2): shard_plan, delta_encode,
delta_apply and helpers, implemented in librose_delta.so (HIP, gfx950) and bound with ctypes.

The names of `binding` are served from here on first use, so that `paper_2605_06534_amd.build`
can be run while the library is missing or stale; any other use loads the library and fails
loudly if it is not built (there is no CPU fallback)."""
import importlib

__all__ = ["BF16", "FP32_RNE", "FUSED_ROWS", "REPLICATED", "SPLIT_COLS", "SPLIT_ROWS", "LAYER_FIRST", "LAYER_LAST",
           "Bucket", "Plan", "RoseError", "bucket_check", "bw_probe", "bw_probe_mixed", "bw_probe_lines", "delta_apply", "delta_encode",
           "delta_encode_refresh", "dense_copy", "ENCODE_ARITH", "ENCODE_REFRESH", "PAYLOAD_ARITH", "PAYLOAD_NEW",
           "delta_encode_ex", "delta_encode_static", "delta_apply_ex", "bucket_pack_ex", "bucket_pack", "object_apply",
           "object_bytes", "object_check", "ptr_table", "shard_plan", "workspace", "binding"]


def __getattr__(name):
    if name in __all__:
        binding = importlib.import_module(__name__ + ".binding")
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))
