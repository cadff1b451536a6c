"""MI355X (gfx950) hot path of on-the-fly self-speculative greedy decoding.

The work is done by hand-written HIP kernels behind the C ABI in include/swift.h
(libswift_hip.so, built in-tree by build.py).  This package only marshals
arguments; PyTorch is used for device memory and streams.
"""
from .binding import (Optimizer, SwiftError, SwiftModel, check_config, device_bytes, expected_speedup, lib, match_prefix,
                      pass_bytes, KERNEL_CLASSES)
from .decode import generate_ar, generate_swift, generate_swift_tree, generate_swift_sample, generate_swift_on_the_fly, SAMPLE_U_PER_STEP

__all__ = ["Optimizer", "SwiftError", "SwiftModel", "check_config", "device_bytes", "expected_speedup", "lib", "match_prefix",
           "pass_bytes", "generate_ar", "generate_swift", "generate_swift_tree", "generate_swift_sample", "generate_swift_on_the_fly", "SAMPLE_U_PER_STEP", "KERNEL_CLASSES"]
