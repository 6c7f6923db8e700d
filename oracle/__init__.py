"""fp64 CPU oracle for the order-2 wavelet scattering cascade.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg.  The product path (the HIP library and its Python
binding) never imports or calls anything in here, and nothing in here imports the
product.
"""
from .filters import bank_1d, bank_2d  # noqa: F401
from .scattering import (coeff_index_1d, coeff_index_2d, pad_index, padded_size,  # noqa: F401
                         scattering1d, scattering1d_backward, scattering1d_padded,
                         scattering1d_padded_backward, scattering2d_padded,
                         scattering2d_padded_backward,
                         scattering1d_plain, scattering2d, scattering2d_backward,
                         scattering2d_plain)
