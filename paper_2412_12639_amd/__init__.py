"""MI355X-native tree verification for Falcon-style speculative decoding.

Thin ctypes binding over the C ABI in include/falcon_verify.h (argument marshalling
only; every step of the path runs in the HIP kernels of libfalcon_verify.so).
PyTorch is used for the device arena and the stream, nothing else."""
from .binding import FalconDrafter, FalconVerifier, FvError, features_device_ptr, load_library, lib_path, STATUS

__all__ = ["FalconDrafter", "FalconVerifier", "FvError", "features_device_ptr", "load_library", "lib_path", "STATUS"]
