"""ORACLE — test infrastructure only.

A plain, slow, double-precision CPU statement of what the hot path computes: the page packer, the
page-granular AdamW update and the one-step-stale delayed update.  Only tests/, the smoke check and
the bench's cpu_baseline leg may import this package; the product path (paper_2303_02868_amd)
never does, and the two share no code.
"""
from .adamw import Hyper, bf16_rne, bf16_bits_to_f64, page_reduce, page_adamw, PagedAdamWState  # noqa: F401
from .packer import plan_pack, pack, unpack, PackPlan, Segment, PageEntry  # noqa: F401
from .delayed import DelayedStepper  # noqa: F401
from .footprint import layer_footprint_bytes, model_state_bytes_per_param  # noqa: F401
from . import scheduler  # noqa: F401
