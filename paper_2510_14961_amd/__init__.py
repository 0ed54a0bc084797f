"""MI355X-native hot path of the diffusion-forcing sampler for recurrent-depth LMs.

The work is done by librdlm.so (hand-written HIP for gfx950, C ABI in include/rdlm.h); this
package only marshals arguments.  Importing the package does not load the library; creating a
Context does, and fails loudly if the library has not been built.
"""
from .binding import (Context, RdlmError, load_library, library_path, weight_names,  # noqa: F401
                      upload_weights, workspace_bytes, EXPORTED_SYMBOLS, STATUS, STATIC_SCRATCH_BYTES)
