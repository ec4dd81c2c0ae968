"""MI355X-native SQuat key-quantization path (arxiv 2503.24358).

`squat` is the thin Python binding over libsquat.so (argument marshalling
only); `synth` holds the seeded input generators; `build` compiles the library.
"""
from . import squat  # noqa: F401

__all__ = ["squat"]
