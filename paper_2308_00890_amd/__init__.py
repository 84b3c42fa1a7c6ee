"""Quantization-aware GNN-layer primitives for MI355X: thin Python binding of the C-ABI library."""
from .binding import *  # noqa: F401,F403
from .binding import GatLayer, GatStack, GcnLayer, Graph, TangoError, TypedLayer, load_library  # noqa: F401
