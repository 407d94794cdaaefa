"""MI355X-native Ouroboros training step (arXiv 1909.06695): Python binding of libouro.so."""
from .binding import (Model, OuroError, create_model, exported_symbols, lib, make_config,
                      lr_schedule, query_arena_bytes, ring_depth, slot_index)

__all__ = ["Model", "OuroError", "create_model", "exported_symbols", "lib", "make_config",
           "lr_schedule", "query_arena_bytes", "ring_depth", "slot_index"]
