"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only *draws inputs* (graphs, features, labels, starting weights, noise).
It contains none of the method's arithmetic: no normalisation of the adjacency matrix,
no augmentation, no forward pass and no ADMM update lives here.
"""
from .configs import Workload, WORKLOADS, get_workload, scaled_workload
from .graphs import erdos_renyi, preferential_attachment, make_graph
from .data import (stream_rng, make_features, make_labels, make_weights,
                   noise_like, perturb_state, perturb_layers, layer_window, planted_labels)

__all__ = ["Workload", "WORKLOADS", "get_workload", "scaled_workload", "erdos_renyi",
           "preferential_attachment", "make_graph", "stream_rng", "make_features",
           "make_labels", "make_weights", "noise_like", "perturb_state", "perturb_layers", "layer_window", "planted_labels"]
