"""MI355X-native LoRDBA adapter forward branch (C-ABI library + thin binding).

``inputs`` (seeded synthetic tensors) imports without the HIP library; the
binding functions load ``liblordba.so`` on first use and raise if it is missing.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "lordba_pack_signs", "lordba_forward", "lordba_packed_words",
           "lordba_status_string", "load_library", "build_library"]


def __getattr__(name):
    if name in __all__:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
