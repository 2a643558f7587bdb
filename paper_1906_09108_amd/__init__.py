"""MI355X-native FDG module worker (arXiv 1906.09108): thin Python binding over the C-ABI library
libfdg.so.  Importing the package does not load the library; `binding.load()` does and fails loudly
when it has not been built."""
from .binding import (FDG_SAVE_ACTIVATIONS, FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS, FDG_SAVE_INPUT_AND_REPLAY, FdgChain, FdgError, FdgModule, fdg_backward_delayed,
                      fdg_destroy, fdg_forward, fdg_module_create, fdg_module_create_ex, fdg_module_workspace_bytes,
                      fdg_module_workspace_bytes_ex, fdg_update, load)

__all__ = ["FdgChain", "FdgError", "FdgModule", "load", "fdg_module_workspace_bytes", "fdg_module_create", "fdg_forward",
           "fdg_backward_delayed", "fdg_update", "fdg_destroy", "fdg_module_workspace_bytes_ex", "fdg_module_create_ex",
           "FDG_SAVE_ACTIVATIONS", "FDG_SAVE_INPUT_AND_REPLAY", "FDG_SAVE_ACTIVATIONS_CURRENT_WEIGHTS"]
