"""CPU oracle (test infrastructure only; see oracle.py)."""
from .oracle import *  # noqa: F401,F403
from .oracle import build  # noqa: F401
from .quant import (conv2d_i8, fc_i8, pack_reference_i8, quantize_eq8,  # noqa: F401
                    requant_shift)
from .select import block_importance, incremental_step, select_mask  # noqa: F401
from . import select as select  # noqa: F401
from .spgemm import mask_blocks, matching_block_products, spgemm_nt  # noqa: F401
