"""MI355X-native sparse weight-delta synchronisation (ROSE, Sec. 4.2): shard_plan, delta_encode,
delta_apply and helpers, implemented in librose_delta.so (HIP, gfx950) and bound with ctypes."""
from .binding import (BF16, FP32_RNE, FUSED_ROWS, REPLICATED, SPLIT_COLS, SPLIT_ROWS, Bucket, Plan,  # noqa: F401
                      RoseError, bucket_check, bw_probe, bw_probe_mixed, delta_apply, delta_encode, delta_encode_refresh, dense_copy,
                      ENCODE_ARITH, ENCODE_REFRESH, PAYLOAD_ARITH, PAYLOAD_NEW, delta_encode_ex, delta_apply_ex, bucket_pack_ex,
                      LAYER_FIRST, LAYER_LAST,
                      bucket_pack, object_apply, object_bytes, object_check, ptr_table, shard_plan, workspace)
