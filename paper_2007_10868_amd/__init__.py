"""MI355X-native DeepPoly back-substitution (the hot path of the GPU polyhedral verifier of
arxiv 2007.10868).  Thin ctypes binding over the C ABI in include/gpupoly.h."""
from .gpupoly import GpuPolyError, Net, lib_path, load_library  # noqa: F401
