"""MI355X-native server-side ciphertext x ciphertext attention path of CryptoGen.

All arithmetic runs in the HIP library (csrc/, built into libcryptogen_hip.so)
behind the C ABI declared in include/cryptogen.h.  This package only marshals
arguments: PyTorch owns device memory and streams.  There is no CPU fallback;
importing `binding` raises if the library has not been built.
"""
from .binding import Context, Library, load_library, to_device, to_host

__all__ = ["Context", "Library", "load_library", "to_device", "to_host"]
