"""CPU oracle package (test infrastructure only; never imported by the product)."""
from .adadim_oracle import (  # noqa: F401
    OC, IC, quantize, pack, unpack, bits_per_weight, hessian,
    layer_error_direct, layer_error_rows, layer_error, layer_error_rows_from_X,
    select, clip_grid, search,
)
from .gemv_oracle import dequantize_ic, gemv_ic, abs_terms  # noqa: F401,E402
from . import gptq_oracle  # noqa: F401,E402
from . import meta16_oracle  # noqa: F401,E402
