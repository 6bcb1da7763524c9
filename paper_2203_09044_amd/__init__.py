"""MI355X-native CO3 gradient codec hot path (error correction, fp conversion, Huffman
compression; parameter-server decompression and averaging).

``binding`` exposes the C entry points of ``libco3.so`` one to one; ``pipeline`` only
allocates the device buffers of one workload and issues the calls of one iteration in order;
``training`` wraps Algorithm 1 around a PyTorch model (users' gradients in, SGD step out).
Importing the package requires the built library: there is no CPU fallback.
"""
from . import binding  # noqa: F401  (raises ImportError when libco3.so is missing)
from .binding import Fmt, Co3Error  # noqa: F401
from .pipeline import Co3Pipeline  # noqa: F401
from .training import Co3SGD  # noqa: F401
