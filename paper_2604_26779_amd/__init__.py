"""MI355X-native verify step of speculative decoding: hand-written HIP kernels (gfx950) behind a
C ABI (include/spec_verify.h), a ctypes binding of the same names, and device-memory plumbing.

    from paper_2604_26779_amd import binding as sv      # the C ABI, name for name
    from paper_2604_26779_amd.session import VerifySession
"""
from . import binding  # noqa: F401
