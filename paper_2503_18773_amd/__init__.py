"""MI355X-native low-bit-KV decode attention (BitDecoding's hot path) behind a C-ABI.

`workloads` (seeded inputs) is importable anywhere.  `binding` mirrors the C-ABI of
`libbitdecode.so` and raises at first use if the HIP library has not been built:
there is no CPU fallback.
"""
__all__ = ["workloads", "binding"]
