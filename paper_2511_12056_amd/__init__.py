"""MI355X-native attention hot path of PipeDiT video-DiT inference.

A thin Python binding over the C-ABI library libpipedit_attn (hand-written HIP
kernels for gfx950).  Every step of the path runs in those kernels; this
package only marshals arguments.  There is no CPU fallback: if the library has
not been built, importing the binding raises.
"""
from .binding import (PdaError, attn_fwd, attn_fwd_base2, attn_fwd_bf16out, attn_fwd_noalloc, attn_fwd_strided, attn_fwd_variant, attn_tail_plan, attn_merge, headchunk_run, headchunk_run_ex, last_error, lib,  # noqa: F401
                      lib_path, pack_heads, pipesp_postprocess, plan_aco, plan_head_padding, plan_n_decode,
                      plan_ragged_groups, probe_loop_rate, probe_mfma_rate, version, PDA_MAX_LOCAL_HEADS, PDA_MAX_PARTIALS, PDA_NOALLOC_MAX_SLOTS, PDA_SINK_HEAD_MAJOR,
                      PDA_SINK_TOKEN_ARRIVAL, PDA_SINK_TOKEN_FINAL)
