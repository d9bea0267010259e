"""Seeded synthetic inputs: pixel generators and a baseline JPEG encoder.

This package stands in for the paper's photo / video-frame datasets (Section 5,
"Datasets"), which are not redistributable.  It serves the decoder's tests, its
CPU oracle's tests and the benchmark alike, and contains none of the decoder's
arithmetic: no Huffman decoding, no synchronisation, no inverse transform.
"""
from .images import CONFIGS, BASE_SEED, config_image, config_jpeg, batch_image, small_image
from .jpeg import encode_jpeg, EncodedJpeg, build as build_encoder

__all__ = [
    "CONFIGS", "BASE_SEED", "config_image", "config_jpeg", "batch_image", "small_image",
    "encode_jpeg", "EncodedJpeg", "build_encoder",
]
