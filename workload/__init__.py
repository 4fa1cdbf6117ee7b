"""Seeded synthetic inputs for the paged multi-LoRA path.

This module only *draws* inputs (adapter weights, activations, token->adapter maps, request
lengths, load/evict traces) and packs them into the byte layouts both the CPU oracle and the
HIP library take as arguments.  It holds none of the method's arithmetic and imports neither
side.  The inputs stand in for the paper's Azure-Functions-derived adapter trace, ShareGPT
length distribution and Llama/Mistral projection shapes (Sec. V-A): only their shapes and
distributions are used.
"""
from .gen import *  # noqa: F401,F403
from .predict import SyntheticPredictor  # noqa: F401
from .configs import CONFIGS, config_layout, BASE_SEED  # noqa: F401
