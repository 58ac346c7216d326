"""Seeded synthetic workloads for the routed-attention layer.

This package only *draws inputs*: latent-grid shaped Q/K/V tensors and route
vectors.  It contains none of the method's arithmetic (no attention, no tile
or bucket logic) and is the one module both the CPU oracle's tests and the HIP
path's tests / benchmark may import.
"""
from .configs import LayerConfig, CONFIGS, get_config, ROUTE_FULL, ROUTE_WINDOW, ROUTE_CORESET
from .fields import make_qkv, make_routes, blur_matrix
from .router import make_router_inputs, timestep_embedding

__all__ = [
    "LayerConfig", "CONFIGS", "get_config", "make_qkv", "make_routes", "blur_matrix", "make_router_inputs", "timestep_embedding",
    "ROUTE_FULL", "ROUTE_WINDOW", "ROUTE_CORESET",
]
