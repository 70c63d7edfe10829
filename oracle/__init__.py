"""CPU oracle for the W3A16 + low-rank expert linear (MiLo, arXiv 2504.02658).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the `paper_2504_02658_amd`
package, its HIP sources, or the C-ABI library) may import, call, link or execute
anything from this directory; only the tests, the smoke check and the CPU-baseline
leg of the benchmark do.  The oracle shares no code, table or helper with the HIP
path: it is a plain numpy / fp64 statement of what the path computes, written from
the paper's definitions (Eq. wq / wdq for the quantizer, the LoRC identity
W~ = Q^-1(W_q) + U V for the compensated weight, Eq. UV for the compensator) and
from the byte-layout description of the packed format.

Every function here is pinned by CPU tests against something other than itself
(closed forms, exact-arithmetic brute force, library routines, invariants).
The paper prints no worked numeric example for this path, so nothing is pinned
against paper-printed values.
"""
from .quantize import quantize_rtn, quantize_sym, dequantize   # noqa: F401
from .packing import (pack_w3, unpack_w3, unit_index, to_unit_order,  # noqa: F401
                      from_unit_order, packed_bytes, code_bytes)
from .linear import w3lr_linear, linear_from_dense        # noqa: F401
from .compensator import (svd_compensator, randomized_svd_compensator,  # noqa: F401
                          quantize_compensator, dequantize_compensator)
from .moe import moe_forward, silu                        # noqa: F401
from .compress import (milo_compress, hqq_zero_points, shrink_lp, fixed_scales,  # noqa: F401
                       quantize_with, stop_rule)
