"""MI355X-native Stream-K++ GEMM: thin Python face of libstreamk.so (see include/streamk.h).

The names of the C ABI live in .binding and are reachable from the package itself
(`import paper_2408_11417_amd as sk; sk.sk_plan(...)`).  The binding - and with it the shared
library - is loaded on first use, not at package import, so that the build module can be imported
before the library exists (or while an older build of it is lying around); a missing library still
fails loudly, at the first call.
"""
import importlib


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    if name in ("binding", "inputs", "build", "selector", "sweep", "fit_tile_model"):
        return importlib.import_module("." + name, __name__)
    return getattr(importlib.import_module(".binding", __name__), name)
