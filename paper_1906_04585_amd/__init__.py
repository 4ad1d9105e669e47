"""MI355X-native GALA-A2C hot path: batched A2C learner step of N agents sharing one GPU
plus gossip mixing of their parameters, in hand-written HIP behind a C ABI (include/gala.h).

`Gala` is a thin ctypes binding: it marshals arguments and owns nothing numerical."""
from .gala import Gala, GalaError, load_library, library_path

__all__ = ["Gala", "GalaError", "load_library", "library_path"]
