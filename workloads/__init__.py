"""Seeded synthetic input generators (shared by oracle tests and GPU tests)."""
from .graphs import (CONFIGS, CONFIG_ORDER, Workload, build, make_config,
                     power_law_degrees, random_csr, sample_columns)
from .hetero import HETERO_CONFIGS, HeteroWorkload, make_hetero
