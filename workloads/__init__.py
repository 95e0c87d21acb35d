"""Seeded synthetic workloads shared by the tests, the benchmark and the CPU oracle.

This package only draws random inputs (planted-span keys, normal queries and
values) and names the configurations.  It contains none of the method's
arithmetic: no attention, no segmentation, no scoring.
"""
from .planted import (Workload, CONFIGS, draw_span_lengths, planted_stream,
                      theta_default, to_dtype)

__all__ = ["Workload", "CONFIGS", "draw_span_lengths", "planted_stream",
           "theta_default", "to_dtype"]
