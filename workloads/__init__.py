"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle.

Holds graph builders and objective-data generators only: none of the method's
arithmetic (no quantizer, no updates, no matching) lives here.  The paper's
experiments use image and translation datasets; these synthetic swarms stand in
for them with the same shapes (node counts 8..256, model sizes up to ~10^8,
2..5 local steps, 4- and 8-bit codes).
"""
from .graphs import complete_graph, torus_graph, random_regular_graph, adjacency, laplacian_lambda2
from .data import diag_quadratic_data, least_squares_data, mixture_data, CONFIGS

__all__ = ["complete_graph", "torus_graph", "random_regular_graph", "adjacency",
           "laplacian_lambda2", "diag_quadratic_data", "least_squares_data",
           "mixture_data", "CONFIGS"]
