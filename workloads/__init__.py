"""Seeded synthetic inputs for the RPTQ hot path (shapes and value structure only).

This package holds the input recipes shared by the CPU oracle's tests and the
HIP path's tests and benchmark.  It contains none of the method's arithmetic:
no quantizer, no clustering, no integer GEMM.
"""
from .synth import (  # noqa: F401
    BASE_SEED,
    CONFIGS,
    LayerConfig,
    SiteSpec,
    bf16_bits,
    bits_to_f32,
    round_to_bf16,
    site_seed,
    make_site,
    extra_batch,
    weight_rows,
    weight_matrix,
    tiny_site,
)
