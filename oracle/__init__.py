"""fp64 CPU oracle of the R-Sparse linear layer -- TEST INFRASTRUCTURE.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import this
package; the product (paper_2504_19449_amd) never does."""
from .rsparse_oracle import (  # noqa: F401
    F16, BF16, F64, RECIPE_BAND, rsparse_linear, dense_linear, quantile_tau, mask, decode16, max_threads,
    silu32, gated_input, gated_input_plain, round16, round16_from_double, dequant_q4, rsparse_linear_q4,
    rsparse_linear_masked, topk_mask, multiphase, multiphase_residual, static_bias,
)
