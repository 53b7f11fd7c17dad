"""Test infrastructure only: the fp64 CPU oracle for the SFB hot path.

Nothing in the product path (the HIP library and its Python binding) may
import this package; it exists so that tests, the smoke check and the
bench's cpu_baseline leg have an independent definition to compare with.
"""
from .sfb_oracle import *  # noqa: F401,F403
from .ssp_oracle import SspOracle, halton_offsets, halton_receivers  # noqa: F401
from .sdca_oracle import SdcaMlrOracle, safe_fraction, mlr_conjugate  # noqa: F401
from .prox_oracle import prox, PROX_KINDS  # noqa: F401
