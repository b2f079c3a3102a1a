"""MI355X-native DDG module step (arXiv 1804.10574): thin Python binding of libddg.so.

Everything numeric runs in the HIP kernels behind the C boundary declared in
include/ddg.h; this package only marshals arguments. Importing it never falls
back to a CPU implementation: if the library is missing, loading raises.
"""
from .ddg import (DDGError, Module, Pipeline, BlockDesc, ModuleDesc, load_library, library_path,
                  DDG_F32, DDG_BF16, DDG_OPT_SGD, DDG_OPT_ADAM, profile_kinds, version)

__all__ = ["DDGError", "Module", "Pipeline", "BlockDesc", "ModuleDesc", "load_library",
           "library_path", "DDG_F32", "DDG_BF16", "DDG_OPT_SGD", "DDG_OPT_ADAM", "profile_kinds", "version"]
