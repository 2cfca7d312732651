"""Seeded synthetic inputs (frames, embeddings, random-init weights).

These generators feed both the CPU oracle and the HIP library with the same
arrays.  They hold none of the method's arithmetic: no similarity, no
selection, no attention, no decoder math.
"""
from .frames import (frame_pair, moving_box_stream, noisy_scene_stream, two_view_stream,
                     patch_pixels,
                     projection_matrix, visual_embeddings, text_embeddings)
from .model import ModelCfg, CONFIGS, make_layer, make_head, round_bf16

__all__ = [
    "frame_pair", "moving_box_stream", "noisy_scene_stream", "two_view_stream", "patch_pixels", "projection_matrix",
    "visual_embeddings", "text_embeddings", "ModelCfg", "CONFIGS",
    "make_layer", "make_head", "round_bf16",
]
