"""Seeded synthetic input generators (no layer arithmetic lives here)."""
from .inputs import (LayerShape, config_layers, make_layer, redraw_rows,  # noqa: F401
                     round_to_bf16, zipf_bias)
