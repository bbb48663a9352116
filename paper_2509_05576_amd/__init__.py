"""MI355X-native layer quantization (sensitivity-guided, row-parallel,
Hessian-compensated).  Thin ctypes binding over libfobq.so; every step of the
method runs in the HIP kernels of the library."""
from .binding import (  # noqa: F401
    FobqError, Ctx, LayerOutput,
    OK, EINVAL, ENOMEM, EHIP, ENOTPD, ESTATE,
    ORDER_NATURAL, ORDER_SENSI_DESC, ORDER_CUSTOM,
    ORDER_ERR_DESC, ORDER_W_DESC, ORDER_SENSI_ASC, ORDER_ERR_ASC, ORDER_W_ASC, ORDER_SENSI_DYNAMIC,
    STAGES, lib_path, load_library,
    fobq_create, fobq_destroy, fobq_last_error,
    HESSIAN_FP64, HESSIAN_INT8_SLICES, fobq_hessian_set_mode,
    fobq_hessian_begin, fobq_hessian_accumulate, fobq_hessian_accumulate_conv, fobq_hessian_finalize,
    fobq_quantize_layer, fobq_quantize_layers_batched, fobq_finish, fobq_spd_inverse, fobq_sensitivity, fobq_sensitivity_static,
    fobq_debug_fail_after, fobq_debug_offset_tables, fobq_workspace_bytes, fobq_obq_rows,
    fobq_hessian_form, FORM_FP64, FORM_INT8_SLICES, FORM_INT8_TAP_OFFSETS,
    fobq_probe_int8_matrix_rate, PROBE_EQUAL_BYTES, PROBE_RANDOM_BYTES, PROBE_RELU_DIGITS,
    fobq_profile_enable, fobq_profile_get, fobq_profile_reset, FOBQ_PROFILE_STAGE,
)
