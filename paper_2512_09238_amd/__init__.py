"""MI355X-native hot path of TCA-Attention behind a C ABI (libtca.so).

`binding` mirrors include/tca.h one to one; `buffers` allocates device memory
through torch; `schedule` sequences chunked prefill and mixed batches; `build`
compiles the library.  `binding` is loaded on first use of any of its names and
raises ImportError if libtca.so is missing or stale (there is no fallback path);
importing the bare package works without the library so that `build` can run.
"""


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    import importlib
    if name in ("binding", "buffers", "schedule", "build", "calibration"):
        return importlib.import_module("." + name, __name__)
    return getattr(importlib.import_module(".binding", __name__), name)
