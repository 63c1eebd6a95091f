"""Seeded synthetic input generators.

This package holds none of the method's arithmetic: it only draws the random
arrays (features, labels, initial parameters) that both the CPU oracle and the
HIP path are fed with.  Neither of those two imports the other; both may be fed
from here.
"""
from .inputs import (  # noqa: F401
    CONFIG_TINY_DIMS,
    CONFIG_FULL_DIMS,
    CONFIG_PAPER_DIMS,
    stream,
    param_count,
    init_theta,
    features_iid,
    feature_stats,
    features_speech_like,
    labels_uniform,
    zipf_cdf,
    labels_zipf,
    rbm_params,
    rbm_binary_input,
)
