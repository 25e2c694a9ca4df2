"""Seeded synthetic inputs (images and model blobs) for the integer-only flow.

This package only draws random numbers and lays them out; it evaluates no part of
the flow. Both the CPU oracle's tests and the GPU library consume what it writes.
"""
from .configs import CONFIGS, FlowConfig, PLAIN, RESNET, DENSE, net_layers, flow_networks, macs_per_image
from .images import make_images, make_large_image
from .model import make_blob, parse_blob, BLOB_MAGIC

__all__ = ["CONFIGS", "FlowConfig", "PLAIN", "RESNET", "DENSE", "net_layers", "flow_networks",
           "macs_per_image", "make_images", "make_large_image", "make_blob", "parse_blob", "BLOB_MAGIC"]
