"""Seeded synthetic inputs for the Cool-SD verify step (shared by tests, bench and smoke).

Holds no arithmetic of the verify/resample method: it only makes logits, draft tokens
and uniforms with the shapes and statistics of the five benchmark configurations.
"""
from .synth import CONFIGS, Workload, make_neighbor_table, make_workload, uniforms24  # noqa: F401
