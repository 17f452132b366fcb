"""MI355X-native Einsum Networks: Python binding over the C ABI of libeinet.so.

The binding only marshals arguments (torch tensors as device memory, the
current torch stream); every step of the forward pass and of EM runs in the HIP
kernels of the shared library.  There is no CPU fallback: without the built
library, or without a GPU at bind time, calls raise.
"""
from .binding import (EiNet, EinetError, load_library, LIB_PATH,  # noqa: F401
                      einet_create, einet_destroy, einet_sizes, einet_structure, einet_bind, einet_refresh, einet_init_params,
                      einet_logp, einet_em_accumulate, einet_em_update, einet_em_reset, einet_em_epoch,
                      einet_mixture_logp, einet_sample, einet_last_error, einet_profile_enable, einet_profile_read, measure_peaks,
                      BERNOULLI, GAUSSIAN, BINOMIAL, CATEGORICAL, EXPORTED_SYMBOLS)
