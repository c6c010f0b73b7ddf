"""Seeded synthetic inputs (graphs, partition ids, initial parameters)."""
from . import rng  # noqa: F401
from .graphs import (Graph, Workload, bfs_partition, build_native, chung_lu,  # noqa: F401
                     describe, erdos_renyi, exploration_uniforms, from_edges, gumbel_uniforms,
                     init_params,
                     make_workload,
                     random_regular)
