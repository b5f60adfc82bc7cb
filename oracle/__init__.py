"""fp64 CPU oracle of the DualSparse-MoE layer forward pass.

Test infrastructure only: the test-suite, the smoke check and the benchmark's CPU-baseline leg
may import this package; the GPU library and its Python binding never do.
"""
from .oracle import build, route, forward, importance, perm_from_importance, n_threads, RouteResult, select_thresholds, ThresholdSelection, router_logits, complete_transform, thresholds_for_drop_rate, DropRateThresholds  # noqa: F401
