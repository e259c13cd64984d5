"""MI355X-native sparsity-aware LDA sampler (hot path of SaberLDA) behind a C ABI.

``Saber`` wraps the ``saber_*`` calls of ``include/saber.h``; the work is done by
the HIP kernels in ``csrc/``.
"""
from .binding import (EXPORTS, Options, Saber, SaberError, Stats, bandwidth_probe, clear_hooks, library_path,
                      load_library, options_default, set_hooks, set_torch_hooks)

__all__ = ["EXPORTS", "Options", "Saber", "SaberError", "Stats", "bandwidth_probe", "clear_hooks", "library_path",
           "load_library", "options_default", "set_hooks", "set_torch_hooks"]
