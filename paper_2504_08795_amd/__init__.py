"""MI355X-native DARIS hot path: thin ctypes binding over libdaris.so (HIP kernels + host scheduler).

Every step of the path runs inside the shared library; this package only marshals arguments.  Importing the
package does not load the library; the first call does, and raises if it has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, DarisError  # noqa: F401
