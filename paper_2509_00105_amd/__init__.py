"""MI355X-native KV-cache level codec (kvh): thin ctypes binding over libkvh.so.

Every step of the path (statistics, quantisation, bit-packing, unpacking, dequantisation,
paged scatter) runs in the HIP kernels behind the C ABI of include/kvh.h; this package only
marshals arguments.  torch is used for device memory and streams.  There is no CPU fallback:
importing the binding without a built library raises.
"""
from .binding import (  # noqa: F401
    BF16, F16, KVHError, Loader, blob_size, decode_kept_batch, encode_kept_batch, make_kept_enc_items, make_kept_items, copy_probe, selftest_division, time_next_launch, decode, decode_batch, decode_chunked, stream_probe, decode_kept, encode, encode_batch,
    encode_chunked, encode_kept, kept_tokens, level_bits, lib, load_static, make_dec_items, make_enc_items, make_tc_items, num_levels,
    policy_marginal_utility_drop, policy_plan, policy_utility, strerror, transcode, transcode_batch,
)
