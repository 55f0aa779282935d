"""MI355X-native attention hot path of PipeDiT video-DiT inference.

A thin Python binding over the C-ABI library libpipedit_attn (hand-written HIP
kernels for gfx950).  Every step of the path runs in those kernels; this
package only marshals arguments.  There is no CPU fallback: if the library has
not been built, importing the binding raises.
"""
from .binding import (PdaError, attn_fwd, attn_merge, headchunk_run, last_error, lib, lib_path,  # noqa: F401
                      version, PDA_MAX_PARTIALS)
