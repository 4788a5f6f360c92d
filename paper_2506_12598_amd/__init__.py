"""MI355X-native co-located inference on pooled CU-masked streams (libeclip + ctypes binding).

The binding (and with it libeclip.so) is loaded on first use, so that `python -m
paper_2506_12598_amd.build` can run before the library exists."""
import importlib


def __getattr__(name):
    binding = importlib.import_module(".binding", __name__)
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
