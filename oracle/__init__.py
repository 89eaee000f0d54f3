"""CPU oracle package (test infrastructure; never imported by the product)."""
from .ddp_oracle import *  # noqa: F401,F403
from .ddp_oracle import (DT_FP32, DT_FP16, DT_BF16, ESIZE, STORAGE, CAP_WHOLE_MODEL)  # noqa: F401
