"""MI355X-native braided F/B/W computation units of one TP shard (paper Section 3).

Thin ctypes binding over libstp.so: argument marshalling only, every step of the
path runs in the library's HIP kernels.  Importing the package never builds; use
paper_2510_27257_amd.build.build() (or __graft_entry__.build()) first.  Every call
raises StpError when the library reports a non-zero status, and the loader raises
when libstp.so is missing: there is no CPU fallback.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
