"""Seeded synthetic detection frames shared by the tests, the benchmark and the smoke check.

This package only draws random boxes and scores.  It contains none of the
suppression arithmetic (no overlap measure, no ranking, no thresholding), so the
CPU oracle and the HIP library can both be fed from it without sharing any of
the method's code.
"""
from .synth import (  # noqa: F401
    CONFIG_NAMES,
    Workload,
    clustered_frame,
    crowd_frame,
    anchor_frame,
    make_config,
    random_frame,
    scores_of_every_kind,
)
