"""MI355X-native forward pass of a dense SwiGLU FFN restructured as shared + routed experts.

`synth` draws seeded synthetic layers and token batches (numpy only).
`binding` is the thin ctypes layer over the C-ABI library `libcmoe.so`; it is imported
lazily so that the input generator stays usable on a machine without the built library.
"""
from . import synth  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
