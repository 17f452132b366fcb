"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

This package holds NONE of the method's arithmetic: it only names the five
benchmark configurations and draws random numbers (parameters, data, masks)
into buffers whose shapes the caller describes.  Both the float64 oracle and
the HIP library are fed from here, so that they see identical inputs.
"""
from .configs import CONFIGS, get_config, fig3_config, sec42_config, BERNOULLI, GAUSSIAN, BINOMIAL, CATEGORICAL  # noqa: F401
from .generate import draw_params, draw_data, draw_mask, config_seed  # noqa: F401
