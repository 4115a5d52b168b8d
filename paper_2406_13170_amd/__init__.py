"""Amphista draft+verify hot path on MI355X: C-ABI library (libamph.so) and its thin binding."""
from . import binding  # noqa: F401
from .binding import (AMPH_BF16, AMPH_F32, AmphError, Context, Tree, amph_config, amph_draft_w,  # noqa: F401
                      amph_layer_w, lib)
