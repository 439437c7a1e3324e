"""MI355X-native rollout engine for length-aware (SortedRL-style) RL training: thin ctypes binding over
librollout.so.  Every step of the path runs in the library's HIP kernels; this package only marshals
arguments.  The binding is loaded on first use and raises if the library has not been built
(python -m paper_2603_23414_amd.build); `paper_2603_23414_amd.build` itself imports without it."""
import importlib

_binding = None


def _load():
    global _binding
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    return _binding


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    return getattr(_load(), name)


def __dir__():
    return sorted(set(globals()) | set(_load().__all__))
