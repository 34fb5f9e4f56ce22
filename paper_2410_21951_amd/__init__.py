"""MI355X-native VADUSA speculative decode step: thin Python binding over libvadusa.so."""
from .vadusa import (Vadusa, VadusaError, TreeArrays, load_library, pack_blob, DBG, build_tree,
                     MAX_TOPK, MAX_TREE_NODES, MAX_DRAFT_HEADS)

__all__ = ["Vadusa", "VadusaError", "TreeArrays", "load_library", "pack_blob", "DBG", "build_tree",
           "MAX_TOPK", "MAX_TREE_NODES", "MAX_DRAFT_HEADS"]
