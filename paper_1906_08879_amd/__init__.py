"""MI355X-native policy forward pass of Placeto (arXiv 1906.08879, Section 2.2).

Thin ctypes binding over libplaceto.so; every step of the path runs in HIP kernels.
Importing this package does not load the library; the first call does, and fails loudly
if it has not been built (`python -m paper_1906_08879_amd.build`).
"""
from .binding import (  # noqa: F401
    GraphBatch,
    ModelCfg,
    PlacetoError,
    Weights,
    embed_forward,
    embed_forward_static,
    embed_forward_static_bytes,
    embed_forward_static_limit,
    graph_batch_upload,
    episode_gradient,
    episode_run,
    episode_step,
    library_path,
    load_library,
    node_classes,
    policy_gradient,
    reinforce_coeff,
    simulate_reward,
    simulate_runtime,
    weights_count,
)
