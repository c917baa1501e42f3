"""MI355X-native W4A8 / W4A16 quantized linear layer (hand-written HIP for
gfx950 behind the C-ABI library ``libmnnq.so``).

``synth`` draws the seeded synthetic inputs; ``binding`` marshals torch device
tensors into the C-ABI calls.  Nothing here computes on the CPU: if the HIP
library is missing, ``binding`` raises.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
