"""MI355X-native ZigzagAttention hot path: thin ctypes binding over libzz.so."""
from .binding import (ZZ_MIXED, ZZ_ZIGZAG, ZZ_TILE_SLOTS, ZZ_MAX_SPLITS, ZzConfig, ZzError, Context, lib,
                      arena_bytes, workspace_bytes, slot_of, strerror, ERR)

__all__ = ["ZZ_MIXED", "ZZ_ZIGZAG", "ZZ_TILE_SLOTS", "ZZ_MAX_SPLITS", "ZzConfig", "ZzError", "Context", "lib",
           "arena_bytes", "workspace_bytes", "slot_of", "strerror", "ERR"]
