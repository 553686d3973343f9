"""MI355X-native R-Sparse linear layer: thin ctypes binding over librsparse.so.

`synth` (input generators) is importable without the library; everything else loads the
HIP library on first use and raises if it has not been built."""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    F16, BF16, F32, Config, Tuning, Layer, RSparseError, load_library, library_path,
    rsparse_prepare, rsparse_compute_factors, rsparse_prepare_factors, rsparse_prepare_q4, make_config, rsparse_linear, rsparse_linear_static, rsparse_linear_gated, rsparse_gated_input, rsparse_mlp_gate_up, rsparse_dense_ref, rsparse_linear_group, rsparse_dense_ref_group, rsparse_linear_group_planned,
    rsparse_last_active, rsparse_synchronize, rsparse_get_factors, rsparse_set_tau, rsparse_set_bias, rsparse_multiphase_bias, rsparse_set_tuning,
    rsparse_get_config, rsparse_calibrate_tau, rsparse_required_bytes, rsparse_dense_bytes, rsparse_io_model,
    rsparse_recipe, rsparse_plan_layer, rsparse_search_recipe, rsparse_debug_stamps, rsparse_destroy, rsparse_last_error, EXPORTED_SYMBOLS,
)
