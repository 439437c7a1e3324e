"""MI355X-native rollout engine for length-aware (SortedRL-style) RL training: thin ctypes binding over
librollout.so.  Every step of the path runs in the library's HIP kernels; this package only marshals
arguments.  Importing `binding` raises if the library has not been built (python -m paper_2603_23414_amd.build)."""
from .binding import *  # noqa: F401,F403
