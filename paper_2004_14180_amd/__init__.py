"""MI355X-native optimizer step of Quantized Adam with error feedback (arXiv 2004.14180).

The product is the gfx950 shared library ``libqadam_hip.so`` behind the C boundary declared in
``include/qadam.h``; :mod:`paper_2004_14180_amd.binding` is a thin argument-marshalling layer over
it with the same names.  PyTorch only provides device memory and streams.
"""
from .binding import (QADAM_IDENTITY, QAdam, QAdamConfig, QAdamError, library_path, load_library)  # noqa: F401
