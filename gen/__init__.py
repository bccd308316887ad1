"""Seeded synthetic input generators (no method arithmetic; shared by oracle tests and GPU tests)."""
from .workloads import (COST_MAX, WORKLOADS, Workload, clean_hierarchy, hierarchical_matrix,  # noqa: F401
                        hierarchy_levels, make_matrix, probe_samples, random_matrix, random_perms)
