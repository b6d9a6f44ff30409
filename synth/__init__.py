"""Seeded synthetic workloads: quantized model blobs and uint8 images.

This package only *draws parameters and pixels* and serialises them.  It holds
none of the method's arithmetic (no sampler, no convolution, no requantisation,
no statistics): the CPU oracle and the HIP library each parse the bytes written
here with their own code.
"""
from .models import build_model, CONFIGS, model_macs  # noqa: F401
from .images import make_image  # noqa: F401
