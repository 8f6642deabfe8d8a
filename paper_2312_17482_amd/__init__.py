"""MI355X-native unpad -> ALiBi varlen attention (fwd+bwd) -> pad.

`workloads` (seeded inputs) imports nothing else; `binding` loads the HIP
library and raises if it is missing.
"""
__all__ = ["workloads", "binding"]
