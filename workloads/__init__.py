"""Seeded synthetic inputs shared by the oracle-side and the GPU-side tests.

Holds NONE of the method's arithmetic: only graphs, datasets, initial models
and the sizes of the benchmark configurations.  The random choices the method
itself draws (worker, neighbour, staleness, minibatch, synthetic gradients)
are NOT made here: each side implements the same counter-based generator.
"""
from .graphs import ring_graph, random_regular4_graph, hop_ring_graph, graph_is_valid  # noqa: F401
from .data import (lsq_data, logreg_data, mixture_data, mlp_init, f32_to_bf16_bits,  # noqa: F401
                   bf16_bits_to_f32, linear_data_on_device, mixture_data_on_device)
from .configs import CONFIGS, get_config  # noqa: F401
from .schedules import random_extra_pairs, with_identity_events  # noqa: F401
