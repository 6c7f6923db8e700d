"""MI355X-native order-2 wavelet scattering (1-D, 2-D, 3-D solid harmonic), HIP library + ctypes binding."""
from .binding import (EXPORTS, LIB_PATH, ScatError, Scattering, lib, scat_backward,  # noqa: F401
                      scat_forward, scat_forward_static, scat_plan_backward_workspace_bytes,
                      scat_plan_coeff_index, scat_plan_create, scat_plan_create_host,
                      scat_plan_create_ex, scat_plan_create_padded, scat_plan_create_padded_host,
                      scat_plan_grid_shape,
                      scat_plan_destroy, scat_plan_filter, scat_plan_num_coeffs,
                      scat_plan_out_shape, scat_plan_reserve, scat_plan_timing_begin, scat_plan_timing_end,
                      scat_plan_timing_row, scat_plan_workspace_bytes, scat_status_string)
