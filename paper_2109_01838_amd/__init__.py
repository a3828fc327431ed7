"""MI355X-native primal-dual multicut (RAMA, arXiv 2109.01838): HIP kernels behind a C ABI.

`Rama` is the binding of librama_hip.so; `inputs` draws the seeded synthetic instances.
Importing the package does not load the library; constructing `Rama` does and raises if
the library or a GPU is missing.
"""
from .binding import (Rama, RamaError, RamaParams, RamaStats, default_params, load_library, EXPORTS, LIB_PATH)  # noqa: F401
from . import inputs  # noqa: F401
