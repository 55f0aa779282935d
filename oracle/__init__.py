"""CPU oracle for the attention hot path and the steps next to it.  TEST INFRASTRUCTURE ONLY.

Plain fp64 numpy implementations of what the HIP library computes, written
from the definitions and sharing no code with the HIP path.  Only tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the product (paper_2511_12056_amd) never does.
"""
from .attention import attention_head, attention, widen_bf16, merge_partials  # noqa: F401
from . import pipesp_layout, planner, pack  # noqa: F401,E402
